// Decode front end: the prologue (query feature map phi_q, workspace reset) and score_mid,
// the streaming pass s_i = q . k_i / sqrt(d_h) over the mid-region (eq. (full_attention)
// restricted to M, eq. (partition)), which reads each KV head's keys once for all query
// heads of its group and accumulates the first-level histogram of the Top-K radix select.
#include "block_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

// ------------------------------------------------------------------------------------
// prologue: grid (Hq, n_problems)
//   * clears the histogram and selection state of (problem, query head)
//   * block (0,0) recomputes the device status word from the problem lengths
//   * phi_q(q)[j] = exp(a * Wq[j] . q - c |q|^2 + bq[j])   (Sec. "Positive feature maps and
//     summary states": phi_q is evaluated per query head at decode time)
// ------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void prologue_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                            char* __restrict__ ws) {
  __shared__ float qf[kMaxDim];
  __shared__ int sh_i[4];
  const int gq = blockIdx.x, p = blockIdx.y, tid = threadIdx.x;
  char* blk = problem_block(g, ws, p);

  if (gq == 0 && p == 0) {
    int bad = 0;
    for (int i = tid; i < g.n_problems; i += kThreads) {
      const int L = probs[i].L;
      bad |= (L < 1 || L > g.max_L) ? 1 : 0;
    }
    bad = block_sum_int(bad, sh_i);
    if (tid == 0) *(uint32_t*)(ws + g.off_status) = bad ? TKPHI_DEV_BAD_LENGTH : 0u;
  }

  uint32_t* hist = (uint32_t*)(blk + g.off_hist) + (size_t)gq * kBins;
  for (int i = tid; i < kBins; i += kThreads) hist[i] = 0u;
  if (tid < (int)(sizeof(HeadState) / 4)) ((uint32_t*)((HeadState*)(blk + g.off_state) + gq))[tid] = 0u;

  const tkphi_problem pr = probs[p];
  float* phiq = (float*)(blk + g.off_phiq) + (size_t)gq * g.dphi;
  if (pr.L < 1 || pr.L > g.max_L) return;
  for (int c = tid; c < g.d; c += kThreads) qf[c] = Elem<T>::load1(pr.q, (int64_t)gq * g.d + c);
  __syncthreads();
  for (int j = tid; j < g.dphi; j += kThreads) {
    float dot = 0.f, nrm = 0.f;
    const int64_t wbase = ((int64_t)gq * g.dphi + j) * g.d;
    for (int c = 0; c < g.d; ++c) {
      const float x = qf[c];
      dot = fmaf(Elem<T>::load1(pr.Wq, wbase + c), x, dot);
      nrm = fmaf(x, x, nrm);
    }
    phiq[j] = expf(g.a * dot - g.c * nrm + pr.bq[(int64_t)gq * g.dphi + j]);
  }
}

// ------------------------------------------------------------------------------------
// score_mid, generic (any storage type): grid (n_scan_chunks, Hkv, n_problems)
// A key row is split over LPR = d / (elements per 16 bytes) lanes, each lane loads 16
// bytes and forms the partial dot products for all G query heads of the KV head; the
// partials are summed across the LPR lanes with butterfly shuffles.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void score_mid_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                             char* __restrict__ ws) {
  constexpr int EPL = Elem<T>::per16;
  extern __shared__ uint32_t lds_hist[];   // [G][kBins]
  const int p = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int c0 = blockIdx.x * g.scan_chunk;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + g.scan_chunk);
  const int G = g.G;
  char* blk = problem_block(g, ws, p);

  for (int i = tid; i < G * kBins; i += kThreads) lds_hist[i] = 0u;

  const int LPR = g.d / EPL;           // lanes per key row (8, 16 or 32)
  const int seg = tid % LPR, rsub = tid / LPR, RPI = kThreads / LPR;

  float qreg[kMaxGroup][EPL];
#pragma unroll
  for (int gl = 0; gl < kMaxGroup; ++gl)
#pragma unroll
    for (int e = 0; e < EPL; ++e)
      qreg[gl][e] = gl < G ? Elem<T>::load1(pr.q, (int64_t)(h * G + gl) * g.d + seg * EPL + e) : 0.f;
  __syncthreads();

  const char* Kb = (const char*)pr.K + ((int64_t)h * pr.stride_head + (int64_t)g.n_sink * pr.stride_tok) * sizeof(T);
  float* scores = (float*)(blk + g.off_scores);

  for (int base = c0; base < c1; base += RPI) {
    const int row = base + rsub;
    const bool valid = row < c1;
    const int rr = valid ? row : c1 - 1;
    const uint4 v = *(const uint4*)(Kb + ((int64_t)rr * pr.stride_tok + seg * EPL) * sizeof(T));
    float x[EPL];
    Elem<T>::unpack(v, x);
    float acc[kMaxGroup];
#pragma unroll
    for (int gl = 0; gl < kMaxGroup; ++gl) {
      float s = 0.f;
      if (gl < G) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) s = fmaf(x[e], qreg[gl][e], s);
      }
      acc[gl] = s;
    }
    for (int o = LPR >> 1; o >= 1; o >>= 1) {
#pragma unroll
      for (int gl = 0; gl < kMaxGroup; ++gl)
        if (gl < G) acc[gl] += __shfl_xor(acc[gl], o);
    }
    if (valid && seg < G) {           // lane `seg` of the row finishes query head `seg`
      float s = acc[0];
#pragma unroll
      for (int gl = 1; gl < kMaxGroup; ++gl) s = (seg == gl) ? acc[gl] : s;
      s = s * g.score_scale + 0.0f;   // + 0.0f turns -0 into +0 so equal scores have equal keys
      const int gq = h * G + seg;
      scores[(size_t)gq * g.mid_stride + row] = s;
      if (pr.scores) pr.scores[(size_t)gq * n + row] = s;
      atomicAdd(&lds_hist[seg * kBins + key_bin(score_key(s))], 1u);
    }
  }
  __syncthreads();
  uint32_t* hist = (uint32_t*)(blk + g.off_hist) + (size_t)h * G * kBins;
  for (int i = tid; i < G * kBins; i += kThreads) {
    const uint32_t c = lds_hist[i];
    if (c) atomicAdd(&hist[i], c);
  }
}

void launch_prologue(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  dim3 grid(g.Hq, g.n_problems);
  if (g.dtype == TKPHI_BF16)
    hipLaunchKernelGGL(prologue_kernel<uint16_t>, grid, dim3(kThreads), 0, s, g, probs, ws);
  else
    hipLaunchKernelGGL(prologue_kernel<float>, grid, dim3(kThreads), 0, s, g, probs, ws);
}

void launch_score_mid(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  if (g.max_mid == 0) return;
  dim3 grid(g.n_scan_chunks, g.Hkv, g.n_problems);
  const size_t lds = (size_t)g.G * kBins * sizeof(uint32_t);
  if (g.dtype == TKPHI_BF16)
    hipLaunchKernelGGL(score_mid_kernel<uint16_t>, grid, dim3(kThreads), lds, s, g, probs, ws);
  else
    hipLaunchKernelGGL(score_mid_kernel<float>, grid, dim3(kThreads), lds, s, g, probs, ws);
}

}  // namespace tkphi
