// Prefill summary build (eq. (natural_cache)):
//   S[h][j][c] = sum_{i in M} phi_k(k_i)[j] v_i[c],   u[h][j] = sum_{i in M} phi_k(k_i)[j]
// with phi_k(k)[j] = exp(a * Wk[h][j] . k - c |k|^2 + bk[h][j]).
//
// The mid-region of each (problem, KV head) is split into chunks; one workgroup reduces a
// chunk into a partial [dphi][d] + [dphi], and a second kernel sums the partials of a head
// in chunk order, so the result does not depend on scheduling.
//
// bf16 caches use the matrix cores for both contractions (features = K Wk^T, then
// S = Phi^T [V | 1]); other storage types use a generic fp32 kernel.
#include "block_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
union Frag {
  u32x4 u;
  bf16x8 v;
};

// ------------------------------------------------------------------------------------
// bf16 on the matrix cores: grid (n_build_chunks, Hkv, n_problems); D == d_head == d_phi.
//
// Tiles of 64 tokens.  GEMM1 (features): wavefront w takes tokens [16w, 16w+16) of the tile;
// the A operand is loaded straight from the key rows (lane (r, kg): token r, 8 consecutive
// channels per k-step), the B operand (all of Wk) stays in registers for the whole chunk.
// The exponentiated features are rounded to bf16 and written feature-major to LDS; the
// value rows are transposed in registers (4 tokens x 8 channels per lane) and written
// channel-major to LDS, so that both operands of GEMM2 (contraction over tokens) are plain
// 16-byte LDS reads.  GEMM2: wavefront w owns value channels [w*D/4, (w+1)*D/4) of S for all
// features, accumulated in registers over the chunk.  u is summed from the same rounded
// features.  The next tile's global loads are issued before GEMM2 of the current tile.
// ------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void build_mfma_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                              char* __restrict__ ws) {
  constexpr int KS = D / 32;            // k-steps of GEMM1 (over channels)
  constexpr int NT = D / 16;            // feature tiles
  constexpr int CW = D / 64;            // channel tiles of S per wavefront
  constexpr int TROW = 64 * 2 + 16;     // bytes per LDS row: 64 tokens of bf16 + pad
  constexpr int PROW = 2 * 64 * 2 + 16; // feature row: 64 tokens hi, 64 tokens lo, pad
  constexpr int VSEG = D / 8;           // 16-byte segments per value row
  __shared__ __attribute__((aligned(16))) char phi_t[D * PROW];   // [feature][hi tokens | lo tokens]
  __shared__ __attribute__((aligned(16))) char v_t[D * TROW];     // [channel][token]
  __shared__ float u_red[4][D];

  const int ch = blockIdx.x, h = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int c0 = ch * g.build_chunk;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + g.build_chunk);
  const int lane = tid & 63, wv = tid >> 6, r = lane & 15, kg = lane >> 4;

  // Wk fragments: wk[nt][j] = Wk[h][feature nt*16 + r][channels j*32 + kg*8 .. +8]
  Frag wk[NT][KS];
  {
    const uint16_t* wsrc = (const uint16_t*)pr.Wk + (size_t)h * D * D;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int j = 0; j < KS; ++j)
        wk[nt][j].u = *(const u32x4*)(wsrc + (size_t)(nt * 16 + r) * D + j * 32 + kg * 8);
  }
  float bias[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) bias[nt] = pr.bk[(size_t)h * D + nt * 16 + r];

  floatx4 sacc[NT][CW];
#pragma unroll
  for (int mt = 0; mt < NT; ++mt)
#pragma unroll
    for (int ct = 0; ct < CW; ++ct) sacc[mt][ct] = (floatx4){0.f, 0.f, 0.f, 0.f};
  float uacc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) uacc[nt] = 0.f;

  const size_t row_bytes = (size_t)pr.stride_tok * 2;
  const size_t base_off = ((size_t)h * pr.stride_head + (size_t)g.n_sink * pr.stride_tok) * 2;
  const char* Kb = (const char*)pr.K + base_off + (size_t)kg * 16;
  // value loads: thread (tq, sg) takes tokens 4*tq .. 4*tq+3 of the tile, 16-byte segment sg
  const bool v_active = tid < 16 * VSEG;
  const int tq = tid % 16, sg = tid / 16;
  const char* Vb = (const char*)pr.V + base_off + (size_t)sg * 16;

  Frag ka[KS];
  u32x4 vv[4];
  auto issue_loads = [&](int t0) {
    const int row = min(t0 + wv * 16 + r, c1 - 1);
    const char* rp = Kb + (size_t)row * row_bytes;
#pragma unroll
    for (int j = 0; j < KS; ++j) ka[j].u = __builtin_nontemporal_load((const u32x4*)(rp + j * 64));
    if (v_active) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int vrow = min(t0 + tq * 4 + i, c1 - 1);
        vv[i] = __builtin_nontemporal_load((const u32x4*)(Vb + (size_t)vrow * row_bytes));
      }
    }
  };

  issue_loads(c0);
  for (int t0 = c0; t0 < c1; t0 += 64) {
    // ---- GEMM1 + exponent on this wavefront's 16 tokens -----------------------------------
    float nrm = 0.f;
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      float x[8];
      Elem<uint16_t>::unpack(*(const uint4*)&ka[j].u, x);
#pragma unroll
      for (int e = 0; e < 8; ++e) nrm = fmaf(x[e], x[e], nrm);
    }
    nrm += __shfl_xor(nrm, 16);
    nrm += __shfl_xor(nrm, 32);
    float nr[4];
    bool ok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      nr[i] = __shfl(nrm, 4 * kg + i);
      ok[i] = (t0 + wv * 16 + 4 * kg + i) < c1;
    }
    // 4 tokens (4kg .. 4kg+3) of feature nt*16 + r as bf16 pairs (hi, lo), hi + lo = 16 bits
    u32x2 phi_hi[NT], phi_lo[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      floatx4 acc = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < KS; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[j].v, wk[nt][j].v, acc, 0, 0, 0);
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float f = __expf(g.a * acc[i] - g.c * nr[i] + bias[nt]);
        split_bf16(f, &hi[i], &lo[i]);
        if (!ok[i]) { hi[i] = 0u; lo[i] = 0u; }
        uacc[nt] += join_bf16(hi[i], lo[i]);
      }
      phi_hi[nt] = (u32x2){hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
      phi_lo[nt] = (u32x2){lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
    }
    // ---- transpose the value block: 4 tokens x 8 channels -> 8 channels x 4 tokens ----------
    u32x2 vt[8];
    if (v_active) {
      const bool vok[4] = {t0 + tq * 4 + 0 < c1, t0 + tq * 4 + 1 < c1, t0 + tq * 4 + 2 < c1, t0 + tq * 4 + 3 < c1};
      uint32_t w[4][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        w[i][0] = vok[i] ? vv[i].x : 0u; w[i][1] = vok[i] ? vv[i].y : 0u;
        w[i][2] = vok[i] ? vv[i].z : 0u; w[i][3] = vok[i] ? vv[i].w : 0u;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {      // dword q of a token holds channels 2q (low half) and 2q+1 (high half)
        vt[2 * q] = (u32x2){(w[0][q] & 0xffffu) | (w[1][q] << 16), (w[2][q] & 0xffffu) | (w[3][q] << 16)};
        vt[2 * q + 1] = (u32x2){(w[0][q] >> 16) | (w[1][q] & 0xffff0000u), (w[2][q] >> 16) | (w[3][q] & 0xffff0000u)};
      }
    }
    // registers are free again: fetch the next tile while this one goes through LDS and GEMM2
    if (t0 + 64 < c1) issue_loads(t0 + 64);

    __syncthreads();                     // the previous tile's GEMM2 has finished reading LDS
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      *(u32x2*)(phi_t + (nt * 16 + r) * PROW + (wv * 16 + 4 * kg) * 2) = phi_hi[nt];
      *(u32x2*)(phi_t + (nt * 16 + r) * PROW + 128 + (wv * 16 + 4 * kg) * 2) = phi_lo[nt];
    }
    if (v_active) {
#pragma unroll
      for (int e = 0; e < 8; ++e) *(u32x2*)(v_t + (sg * 8 + e) * TROW + tq * 8) = vt[e];
    }
    __syncthreads();

    // ---- GEMM2: S[features][this wavefront's channels] += Phi^T V over the tile's 64 tokens ----
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      Frag vb[CW];
#pragma unroll
      for (int ct = 0; ct < CW; ++ct)
        vb[ct].u = *(const u32x4*)(v_t + (wv * (D / 4) + ct * 16 + r) * TROW + (ks * 32 + kg * 8) * 2);
#pragma unroll
      for (int mt = 0; mt < NT; ++mt) {
        Frag pa_hi, pa_lo;
        pa_hi.u = *(const u32x4*)(phi_t + (mt * 16 + r) * PROW + (ks * 32 + kg * 8) * 2);
        pa_lo.u = *(const u32x4*)(phi_t + (mt * 16 + r) * PROW + 128 + (ks * 32 + kg * 8) * 2);
#pragma unroll
        for (int ct = 0; ct < CW; ++ct) {
          sacc[mt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo.v, vb[ct].v, sacc[mt][ct], 0, 0, 0);
          sacc[mt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi.v, vb[ct].v, sacc[mt][ct], 0, 0, 0);
        }
      }
    }
  }

  // ---- write the chunk partial: S part [D][D] then u part [D] ----------------------------------
  float* bp = (float*)(ws + g.off_bpart) + ((size_t)(p * g.Hkv + h) * g.n_build_chunks + ch) * ((size_t)D * (D + 1));
#pragma unroll
  for (int mt = 0; mt < NT; ++mt)
#pragma unroll
    for (int ct = 0; ct < CW; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        bp[(size_t)(mt * 16 + 4 * kg + i) * D + wv * (D / 4) + ct * 16 + r] = sacc[mt][ct][i];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float x = uacc[nt];
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    if (kg == 0) u_red[wv][nt * 16 + r] = x;
  }
  __syncthreads();
  if (tid < D) bp[(size_t)D * D + tid] = (u_red[0][tid] + u_red[1][tid]) + (u_red[2][tid] + u_red[3][tid]);
}

// ------------------------------------------------------------------------------------
// generic kernel (any storage type, fp32 arithmetic): grid (n_build_chunks, Hkv, n_problems)
// threads form a 16 x 16 grid over (feature block, channel block).
// ------------------------------------------------------------------------------------
constexpr int kTB = 16;   // tokens per batch

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
    if (g.use_mfma) {
      if (g.d == 128) TKPHI_LAUNCH(ST_UNTIMED, build_mfma_kernel<128>, grid, dim3(kThreads), 0, s, g, probs, ws);
      else TKPHI_LAUNCH(ST_UNTIMED, build_mfma_kernel<64>, grid, dim3(kThreads), 0, s, g, probs, ws);
    } else if (g.dtype == TKPHI_BF16) {
      TKPHI_LAUNCH(ST_UNTIMED, build_kernel<uint16_t>, grid, dim3(kThreads), 0, s, g, probs, ws);
    } else {
      TKPHI_LAUNCH(ST_UNTIMED, build_kernel<float>, grid, dim3(kThreads), 0, s, g, probs, ws);
    }
  }
  const int per = g.dphi * (g.d + 1);
  dim3 rgrid((per + kThreads - 1) / kThreads, g.Hkv, g.n_problems);
  TKPHI_LAUNCH(ST_UNTIMED, build_reduce_kernel, rgrid, dim3(kThreads), 0, s, g, probs, ws);
}

}  // namespace tkphi
