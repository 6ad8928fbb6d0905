// Prefill summary build (eq. (natural_cache)):
//   S[h][j][c] = sum_{i in M} phi_k(k_i)[j] v_i[c],   u[h][j] = sum_{i in M} phi_k(k_i)[j]
// with phi_k(k)[j] = exp(a * Wk[h][j] . k - c |k|^2 + bk[h][j]).
//
// The mid-region of each (problem, KV head) is split into chunks; one workgroup reduces a
// chunk into a partial [dphi][d] + [dphi], and a second kernel sums the partials of a head
// in chunk order, so the result does not depend on scheduling.
#include "block_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

constexpr int kTB = 16;   // tokens per batch in the generic kernel

// generic kernel (any storage type, fp32 arithmetic): grid (n_build_chunks, Hkv, n_problems)
// threads form a 16 x 16 grid over (feature block, channel block).
template <typename T>
__global__ __launch_bounds__(kThreads) void build_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                         char* __restrict__ ws) {
  __shared__ float kf[kTB][kMaxDim];
  __shared__ float vf[kTB][kMaxDim];
  __shared__ float ph[kTB][kMaxDim];
  constexpr int FJmax = kMaxDim / 16, FCmax = 128 / 16;

  const int ch = blockIdx.x, h = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int c0 = ch * g.build_chunk;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + g.build_chunk);
  const int d = g.d, dphi = g.dphi;
  const int FJ = dphi / 16, FC = d / 16;
  const int tj = tid / 16, tc = tid % 16;

  float acc[FJmax][FCmax];
  float uacc[FJmax];
#pragma unroll
  for (int a = 0; a < FJmax; ++a) {
    uacc[a] = 0.f;
#pragma unroll
    for (int b = 0; b < FCmax; ++b) acc[a][b] = 0.f;
  }
  const int64_t head_off = (int64_t)h * pr.stride_head;

  for (int base = c0; base < c1; base += kTB) {
    const int nt = min(kTB, c1 - base);
    __syncthreads();
    for (int i = tid; i < kTB * d; i += kThreads) {
      const int t = i / d, c = i % d;
      float kv = 0.f, vv = 0.f;
      if (t < nt) {
        const int64_t off = head_off + (int64_t)(g.n_sink + base + t) * pr.stride_tok + c;
        kv = Elem<T>::load1(pr.K, off);
        vv = Elem<T>::load1(pr.V, off);
      }
      kf[t][c] = kv; vf[t][c] = vv;
    }
    __syncthreads();
    // features: thread (t = tid / 16, j = tid % 16 + 16 * i)
    {
      const int t = tid / 16;
      float nrm = 0.f;
      for (int c = 0; c < d; ++c) nrm = fmaf(kf[t][c], kf[t][c], nrm);
      for (int i = 0; i < FJ; ++i) {
        const int j = (tid % 16) + 16 * i;
        const int64_t wbase = ((int64_t)h * dphi + j) * d;
        float dot = 0.f;
        for (int c = 0; c < d; ++c) dot = fmaf(Elem<T>::load1(pr.Wk, wbase + c), kf[t][c], dot);
        const float f = expf(g.a * dot - g.c * nrm + pr.bk[(int64_t)h * dphi + j]);
        ph[t][j] = t < nt ? f : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int a = 0; a < FJmax; ++a) {
      if (a < FJ) {
        const int j = tj * FJ + a;
        for (int t = 0; t < kTB; ++t) {
          const float f = ph[t][j];
          if (tc == 0) uacc[a] += f;
#pragma unroll
          for (int b = 0; b < FCmax; ++b)
            if (b < FC) acc[a][b] = fmaf(f, vf[t][tc * FC + b], acc[a][b]);
        }
      }
    }
  }

  float* bp = (float*)(ws + g.off_bpart) +
              ((size_t)(p * g.Hkv + h) * g.n_build_chunks + ch) * ((size_t)dphi * (d + 1));
#pragma unroll
  for (int a = 0; a < FJmax; ++a) {
    if (a < FJ) {
      const int j = tj * FJ + a;
#pragma unroll
      for (int b = 0; b < FCmax; ++b)
        if (b < FC) bp[(size_t)j * d + tc * FC + b] = acc[a][b];
      if (tc == 0) bp[(size_t)dphi * d + j] = uacc[a];
    }
  }
}

// sums the chunk partials of each (problem, KV head) in chunk order.
// grid (ceil(dphi*(d+1) / 256), Hkv, n_problems)
__global__ __launch_bounds__(kThreads) void build_reduce_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                char* __restrict__ ws) {
  const int h = blockIdx.y, p = blockIdx.z;
  const int L = probs[p].L;
  if (L < 1 || L > g.max_L) return;
  const int n = mid_size(L, g.n_sink, g.n_tail);
  const int n_chunks = (n + g.build_chunk - 1) / g.build_chunk;
  const int d = g.d, dphi = g.dphi;
  const size_t per = (size_t)dphi * (d + 1);
  const size_t e = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (e >= per) return;
  const float* bp = (const float*)(ws + g.off_bpart) + ((size_t)(p * g.Hkv + h) * g.n_build_chunks) * per + e;
  float s = 0.f;
  for (int c = 0; c < n_chunks; ++c) s += bp[(size_t)c * per];
  if (e < (size_t)dphi * d) probs[p].S[(size_t)h * dphi * d + e] = s;
  else probs[p].u[(size_t)h * dphi + (e - (size_t)dphi * d)] = s;
}

void launch_build(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  if (g.max_mid > 0) {
    dim3 grid(g.n_build_chunks, g.Hkv, g.n_problems);
    if (g.dtype == TKPHI_BF16)
      hipLaunchKernelGGL(build_kernel<uint16_t>, grid, dim3(kThreads), 0, s, g, probs, ws);
    else
      hipLaunchKernelGGL(build_kernel<float>, grid, dim3(kThreads), 0, s, g, probs, ws);
  }
  const int per = g.dphi * (g.d + 1);
  dim3 rgrid((per + kThreads - 1) / kThreads, g.Hkv, g.n_problems);
  hipLaunchKernelGGL(build_reduce_kernel, rgrid, dim3(kThreads), 0, s, g, probs, ws);
}

}  // namespace tkphi
