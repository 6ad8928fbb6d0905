// Decode back end.
//
// gather (exact_branch + residual_correct): one workgroup per tile of 64 retrieved tokens of
// a query head (and one per query head for the anchors) accumulates
//     m_loc = max s_i,  Z_loc = sum exp(s_i - m_loc),  nu_loc = sum exp(s_i - m_loc) v_i
// (eq. (exact_terms)), and the feature-space contributions to subtract from the summaries
// (eq. (subtraction)), kept as the already contracted sums
//     zsum = sum_i z_i,  zv = sum_i z_i v_i,   z_i = phi_q(q) . phi_k(k_i)
// with phi_k(k_i) recomputed from the gathered key, so that S_R is never materialised:
//     S_R^T phi_q = S_M^T phi_q - zv,      phi_q . u_R = phi_q . u_M - zsum.
// On the bf16 path phi_k(k_i) goes through the same arithmetic as in the summary build
// (bf16 MFMA with fp32 accumulation, fp32 exponent, result kept as a bf16 hi + lo pair),
// so what is subtracted is what was added.
//
// merge: combines the partials of a query head in a fixed order (log-sum-exp rescaling),
// evaluates the summary terms and applies the single-normalisation merge
// (eq. (hybrid_merge)) with the exact branch's max shift applied to the residual branch.
//
// All loops over tokens issue their (independent) row loads before consuming them: these
// kernels move little data and are bound by memory latency, not bandwidth.
#include "block_utils.h"
#include "gather_tile.h"
#include "merge_head.h"
#include "tkphi_internal.h"

namespace tkphi {

typedef GatherFrag Frag;

// ---- weighted sums of value rows ------------------------------------------------------------
// nu[c] = sum_i w[i] v_i[c], zv[c] = sum_i z[i] v_i[c] over `cnt` <= 64 rows given by tok[]
// (absolute token indices), rows of d elements.  Each row is read by LPR = d / (elements per
// 16 bytes) lanes with one 16-byte load; 256 threads cover 256 / LPR rows per pass and all
// passes' loads are issued together.  Results land in part[4 .. 4+d) and part[4+d .. 4+2d).
// LDS scratch `red` must hold 2 * 256 * 8 floats.
template <typename T>
__device__ __forceinline__ void weighted_value_sums(const Geom& g, const tkphi_problem& pr, int64_t head_off,
                                                    const int* tok, const float* w, const float* z, int cnt,
                                                    float* red, float* part, bool with_z) {
  constexpr int EPL = Elem<T>::per16;
  const int tid = threadIdx.x, d = g.d;
  const int LPR = d / EPL, RPP = kThreads / LPR;      // rows per pass
  const int seg = tid % LPR, rsub = tid / LPR;
  constexpr int MAXP = 8;                              // 64 rows / (256 / 32 lanes) passes at most
  const int n_pass = (cnt + RPP - 1) / RPP;
  uint4 v[MAXP];
#pragma unroll
  for (int ps = 0; ps < MAXP; ++ps) {
    if (ps < n_pass) {
      const int i = min(ps * RPP + rsub, cnt - 1);
      const u32x4 t = gload128((const char*)pr.V + (head_off + (int64_t)tok[i] * pr.stride_tok + seg * EPL) * sizeof(T));
      v[ps] = make_uint4(t.x, t.y, t.z, t.w);
    }
  }
  float an[EPL], az[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) { an[e] = 0.f; az[e] = 0.f; }
#pragma unroll
  for (int ps = 0; ps < MAXP; ++ps) {
    if (ps < n_pass) {
      const int i = ps * RPP + rsub;
      if (i < cnt) {
        float x[EPL];
        Elem<T>::unpack(v[ps], x);
        const float wi = w[i], zi = with_z ? z[i] : 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) { an[e] = fmaf(wi, x[e], an[e]); az[e] = fmaf(zi, x[e], az[e]); }
      }
    }
  }
  // reduce over the RPP row groups: red[rsub][channel]
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    red[rsub * d + seg * EPL + e] = an[e];
    red[kThreads * 8 + rsub * d + seg * EPL + e] = az[e];
  }
  __syncthreads();
  if (tid < d) {
    float a0 = 0.f, a1 = 0.f;
    for (int k = 0; k < RPP; ++k) { a0 += red[k * d + tid]; a1 += red[kThreads * 8 + k * d + tid]; }
    part[4 + tid] += a0;
    part[4 + d + tid] += a1;
  }
  __syncthreads();
}

// ---- anchors: exact terms over [0, n_sink) u [L - n_tail, L) (or every token if M is empty) --------
// One workgroup per batch of 64 anchors (`batch` = 0, 1, ...): scores with LPR lanes per key
// row (16-byte loads, butterfly sum), then the same weighted value sums as a retrieved tile.
template <typename T>
__device__ void anchor_partial(const Geom& g, const tkphi_problem& pr, int gq, int n, int batch, float* part,
                               float* red) {
  constexpr int EPL = Elem<T>::per16;
  __shared__ int a_tok[64];
  __shared__ float a_s[64], a_w[64];
  __shared__ float a_acc[2 * kMaxDim + 4];           // [-, -, -, -, nu[d], zv[d]] in the partial's layout
  __shared__ float a_m;
  const int tid = threadIdx.x, d = g.d;
  const int h = gq / g.G;
  const int n_prefill = n > 0 ? g.n_sink + g.n_tail : pr.L;             // exact anchors of the prefill segment
  const int n_anchor = n_prefill + min(max(pr.n_gen, 0), g.max_gen);    // + generated tokens, rows [L, L + n_gen)
  const int base = batch * 64;
  if (base >= n_anchor) return;
  const int cnt = min(64, n_anchor - base);
  const int64_t head_off = (int64_t)h * pr.stride_head;
  const int LPR = d / EPL, RPP = kThreads / LPR;
  const int seg = tid % LPR, rsub = tid / LPR;
  float qreg[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) qreg[e] = Elem<T>::load1(pr.q, (int64_t)gq * d + seg * EPL + e);
  for (int i = tid; i < 2 * d + 4; i += kThreads) a_acc[i] = 0.f;
  if (tid < 64) {
    const int a = base + min(tid, cnt - 1);
    a_tok[tid] = a >= n_prefill ? pr.L + (a - n_prefill) : (n > 0 && a >= g.n_sink) ? (pr.L - g.n_tail + (a - g.n_sink)) : a;
  }
  __syncthreads();
  // scores of the batch
  constexpr int MAXP = 8;
  const int n_pass = (cnt + RPP - 1) / RPP;
  uint4 kv[MAXP];
#pragma unroll
  for (int ps = 0; ps < MAXP; ++ps) {
    if (ps < n_pass) {
      const int i = min(ps * RPP + rsub, cnt - 1);
      const u32x4 t = gload128((const char*)pr.K + (head_off + (int64_t)a_tok[i] * pr.stride_tok + seg * EPL) * sizeof(T));
      kv[ps] = make_uint4(t.x, t.y, t.z, t.w);
    }
  }
#pragma unroll
  for (int ps = 0; ps < MAXP; ++ps) {
    if (ps < n_pass) {
      float x[EPL];
      Elem<T>::unpack(kv[ps], x);
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) s = fmaf(x[e], qreg[e], s);
      for (int o = LPR >> 1; o >= 1; o >>= 1) s += __shfl_xor(s, o);
      const int i = ps * RPP + rsub;
      if (seg == 0 && i < cnt) a_s[i] = s * g.score_scale + 0.0f;
    }
  }
  __syncthreads();
  if (tid < 64) {
    float mb = tid < cnt ? a_s[tid] : -INFINITY;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mb = fmaxf(mb, __shfl_xor(mb, o));
    a_w[tid] = tid < cnt ? __expf(a_s[tid] - mb) : 0.f;
    if (tid == 0) a_m = mb;
  }
  __syncthreads();
  weighted_value_sums<T>(g, pr, head_off, a_tok, a_w, a_w, cnt, red, a_acc, false);
  if (tid == 0) {
    float Z = 0.f;
    for (int i = 0; i < cnt; ++i) Z += a_w[i];
    part[0] = a_m; part[1] = Z; part[2] = 0.f; part[3] = (float)cnt;
  }
  if (tid < d) { part[4 + tid] = a_acc[4 + tid]; part[4 + d + tid] = 0.f; }
}

// ------------------------------------------------------------------------------------
// gather, bf16 on the matrix cores: grid (n_tiles + n_atiles, Hq, n_problems); D == d_head == d_phi.
// Wavefront w owns 16 retrieved tokens: their key rows are the A operand (lane (r, kg): token
// r, 8 consecutive channels per k-step), Wk of the KV head is staged once per workgroup in
// LDS (rows padded by 16 B: conflict-free ds_read_b128) and provides the B operand per
// 16-feature tile.
// ------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void gather_mfma_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                               char* __restrict__ ws) {
  constexpr int KS = D / 32;
  constexpr int WROW = wk_row_bytes(D);            // bytes per staged Wk row
  // the staged Wk and the reduction scratch of the value sums are never live together
  constexpr int kRedBytes = 2 * kThreads * 8 * (int)sizeof(float);
  constexpr int kBufBytes = D * WROW > kRedBytes ? D * WROW : kRedBytes;
  __shared__ __attribute__((aligned(16))) char lds_buf[kBufBytes];
  char* wk_lds = lds_buf;
  float* red = (float*)lds_buf;
  __shared__ int p_tok[kPairsPerWG];
  __shared__ float p_s[kPairsPerWG], p_w[kPairsPerWG], p_z[kPairsPerWG];
  __shared__ float acc_part[2 * D + 4];
  __shared__ float sh_m;

  const int tile = blockIdx.x, gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  char* blk = problem_block(g, ws, p);
  float* part = (float*)(blk + g.off_part) + ((size_t)gq * (g.n_tiles + g.n_atiles) + tile) * g.part_stride;
  if (tile >= g.n_tiles) { anchor_partial<uint16_t>(g, pr, gq, n, tile - g.n_tiles, part, red); return; }
  const int Ksel = ((const SelPlan*)(blk + g.off_plan))[gq].n_sel;
  const int i0 = tile * kPairsPerWG;
  if (i0 >= Ksel) return;
  const int cnt = min(kPairsPerWG, Ksel - i0);
  const int h = gq / g.G;
  const int lane = tid & 63, wv = tid >> 6, r = lane & 15, kg = lane >> 4;

  // the tile's retrieved tokens
  if (tid < kPairsPerWG) {
    const int i = i0 + min(tid, cnt - 1);
    p_tok[tid] = g.n_sink + min(max(((const int32_t*)(blk + g.off_selidx))[(size_t)gq * g.max_K + i], 0), n - 1);
    p_s[tid] = tid < cnt ? ((const float*)(blk + g.off_selscore))[(size_t)gq * g.max_K + i] : -INFINITY;
  }
  for (int i = tid; i < 2 * D + 4; i += kThreads) acc_part[i] = 0.f;
  // stage Wk[h] ([D features][D channels] bf16) with padded rows
  {
    const char* wsrc = (const char*)pr.Wk + (size_t)h * D * D * 2;
    constexpr int SEGS = D * 2 / 16;               // 16-byte segments per row
    constexpr int PER = D * SEGS / kThreads;
    u32x4 t[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const int i = tid + k * kThreads;
      t[k] = gload128(wsrc + (size_t)(i / SEGS) * D * 2 + (i % SEGS) * 16);
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) {
      const int i = tid + k * kThreads;
      *(u32x4*)(wk_lds + (i / SEGS) * WROW + (i % SEGS) * 16) = t[k];
    }
  }
  __syncthreads();
  if (tid < 64) {                                  // m_loc = max score of the tile
    float m = p_s[tid];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (tid == 0) sh_m = m;
  }

  const int64_t head_off = (int64_t)h * pr.stride_head;
  if (wv * 16 < cnt) {
    // A operand: key rows of this wavefront's 16 tokens
    const int tok = p_tok[wv * 16 + r];
    const char* rp = (const char*)pr.K + (head_off + (int64_t)tok * pr.stride_tok) * 2 + kg * 16;
    Frag a[KS];
#pragma unroll
    for (int j = 0; j < KS; ++j) a[j].u = gload128(rp + j * 64);
    const float* phiq = (const float*)(blk + g.off_phiq) + (size_t)gq * D;
    float zacc[4];
    wave_feature_dots<D>(a, wk_lds, pr.bk + (size_t)h * D, phiq, g.a, g.c, zacc);
    if (r == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) p_z[wv * 16 + 4 * kg + i] = zacc[i];
    }
  }
  __syncthreads();
  if (tid < kPairsPerWG) p_w[tid] = tid < cnt ? __expf(p_s[tid] - sh_m) : 0.f;
  __syncthreads();

  weighted_value_sums<uint16_t>(g, pr, head_off, p_tok, p_w, p_z, cnt, red, acc_part, true);
  if (tid < D) { part[4 + tid] = acc_part[4 + tid]; part[4 + D + tid] = acc_part[4 + D + tid]; }
  if (tid == 0) {
    float Z = 0.f, zs = 0.f;
    for (int i = 0; i < cnt; ++i) { Z += p_w[i]; zs += p_z[i]; }
    part[0] = sh_m; part[1] = Z; part[2] = zs; part[3] = (float)cnt;
  }
}

// ------------------------------------------------------------------------------------
// gather, generic (any storage type, fp32 arithmetic): same grid.  The key rows of the tile's
// (at most 64) tokens are staged in LDS as fp32; thread (token t = tid % 64, group fg = tid / 64)
// evaluates the features j = fg, fg + 4, ... of token t (Wk rows are read with 16-byte loads
// that all 64 lanes of a wavefront share), so the 64 tokens advance together.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void gather_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                          char* __restrict__ ws) {
  constexpr int EPL = Elem<T>::per16;
  constexpr int KFS = 128 + 1;                     // padded row stride (d <= 128): conflict-free column reads
  __shared__ float kf[kPairsPerWG * KFS];
  __shared__ float red[2 * kThreads * 8];
  __shared__ int p_tok[kPairsPerWG];
  __shared__ float p_s[kPairsPerWG], p_w[kPairsPerWG], p_z[kPairsPerWG];
  __shared__ float z_part[4][kPairsPerWG];
  __shared__ float acc_part[2 * 128 + 4];
  __shared__ float sh_m;
  const int tile = blockIdx.x, gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  char* blk = problem_block(g, ws, p);
  float* part = (float*)(blk + g.off_part) + ((size_t)gq * (g.n_tiles + g.n_atiles) + tile) * g.part_stride;
  if (tile >= g.n_tiles) { anchor_partial<T>(g, pr, gq, n, tile - g.n_tiles, part, red); return; }
  const int Ksel = ((const SelPlan*)(blk + g.off_plan))[gq].n_sel;
  const int i0 = tile * kPairsPerWG;
  if (i0 >= Ksel) return;
  const int cnt = min(kPairsPerWG, Ksel - i0);
  const int h = gq / g.G, d = g.d, dphi = g.dphi;
  const float* phiq = (const float*)(blk + g.off_phiq) + (size_t)gq * dphi;
  const int64_t head_off = (int64_t)h * pr.stride_head;

  if (tid < kPairsPerWG) {
    const int i = i0 + min(tid, cnt - 1);
    p_tok[tid] = g.n_sink + min(max(((const int32_t*)(blk + g.off_selidx))[(size_t)gq * g.max_K + i], 0), n - 1);
    p_s[tid] = tid < cnt ? ((const float*)(blk + g.off_selscore))[(size_t)gq * g.max_K + i] : -INFINITY;
  }
  for (int i = tid; i < 2 * d + 4; i += kThreads) acc_part[i] = 0.f;
  __syncthreads();
  {
    // key rows -> LDS (fp32): 16-byte pieces, (row, segment) pairs dealt over the threads
    const int SEGS = d / EPL;
    for (int idx = tid; idx < kPairsPerWG * SEGS; idx += kThreads) {
      const int row = idx / SEGS, seg = idx % SEGS;
      const u32x4 t = gload128((const char*)pr.K + (head_off + (int64_t)p_tok[row] * pr.stride_tok + seg * EPL) * sizeof(T));
      float x[EPL];
      Elem<T>::unpack(make_uint4(t.x, t.y, t.z, t.w), x);
#pragma unroll
      for (int e = 0; e < EPL; ++e) kf[row * KFS + seg * EPL + e] = x[e];
    }
  }
  __syncthreads();
  if (tid < 64) {                                  // m_loc = max score of the tile
    float m = p_s[tid];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (tid == 0) sh_m = m;
  }
  {
    // z_t = phi_q . phi_k(k_t): thread (t, fg) sums its features in ascending order
    const int t = tid % kPairsPerWG, fg = tid / kPairsPerWG;
    const float* kt = kf + t * KFS;
    float nrm = 0.f;
    for (int c = 0; c < d; ++c) nrm = fmaf(kt[c], kt[c], nrm);
    float z = 0.f;
    for (int j = fg; j < dphi; j += kThreads / kPairsPerWG) {
      const char* wrow = (const char*)pr.Wk + ((int64_t)h * dphi + j) * d * sizeof(T);
      float dot = 0.f;
      for (int c0 = 0; c0 < d; c0 += EPL) {
        const u32x4 wv4 = gload128(wrow + c0 * sizeof(T));
        float wx[EPL];
        Elem<T>::unpack(make_uint4(wv4.x, wv4.y, wv4.z, wv4.w), wx);
#pragma unroll
        for (int e = 0; e < EPL; ++e) dot = fmaf(wx[e], kt[c0 + e], dot);
      }
      z = fmaf(expf(g.a * dot - g.c * nrm + pr.bk[(int64_t)h * dphi + j]), phiq[j], z);
    }
    z_part[fg][t] = z;
  }
  __syncthreads();
  if (tid < kPairsPerWG) {
    p_z[tid] = tid < cnt ? (z_part[0][tid] + z_part[1][tid]) + (z_part[2][tid] + z_part[3][tid]) : 0.f;
    p_w[tid] = tid < cnt ? __expf(p_s[tid] - sh_m) : 0.f;
  }
  __syncthreads();

  weighted_value_sums<T>(g, pr, head_off, p_tok, p_w, p_z, cnt, red, acc_part, true);
  if (tid < d) { part[4 + tid] = acc_part[4 + tid]; part[4 + d + tid] = acc_part[4 + d + tid]; }
  if (tid == 0) {
    float Z = 0.f, zs = 0.f;
    for (int i = 0; i < cnt; ++i) { Z += p_w[i]; zs += p_z[i]; }
    part[0] = sh_m; part[1] = Z; part[2] = zs; part[3] = (float)cnt;
  }
}

// ------------------------------------------------------------------------------------
// gather from cached key features (cfg.cache_features): same grid and partial layout; instead
// of reading the key rows and recomputing phi_k, every retrieved token's feature row (d_phi
// fp32 values stored by the build) is read with 16-byte loads, d_phi / 4 lanes per row, all
// rows of the tile in flight together, and z_i = phi_q . phi_k(k_i) is a butterfly sum.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void gather_cached_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                 char* __restrict__ ws) {
  __shared__ float red[2 * kThreads * 8];
  __shared__ int p_tok[kPairsPerWG];
  __shared__ float p_s[kPairsPerWG], p_w[kPairsPerWG], p_z[kPairsPerWG];
  __shared__ float acc_part[2 * 128 + 4];
  __shared__ float sh_m;
  const int tile = blockIdx.x, gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  char* blk = problem_block(g, ws, p);
  float* part = (float*)(blk + g.off_part) + ((size_t)gq * (g.n_tiles + g.n_atiles) + tile) * g.part_stride;
  if (tile >= g.n_tiles) { anchor_partial<T>(g, pr, gq, n, tile - g.n_tiles, part, red); return; }
  const int Ksel = ((const SelPlan*)(blk + g.off_plan))[gq].n_sel;
  const int i0 = tile * kPairsPerWG;
  if (i0 >= Ksel) return;
  const int cnt = min(kPairsPerWG, Ksel - i0);
  const int h = gq / g.G, d = g.d, dphi = g.dphi;
  const int64_t head_off = (int64_t)h * pr.stride_head;

  if (tid < kPairsPerWG) {
    const int i = i0 + min(tid, cnt - 1);
    p_tok[tid] = g.n_sink + min(max(((const int32_t*)(blk + g.off_selidx))[(size_t)gq * g.max_K + i], 0), n - 1);
    p_s[tid] = tid < cnt ? ((const float*)(blk + g.off_selscore))[(size_t)gq * g.max_K + i] : -INFINITY;
  }
  for (int i = tid; i < 2 * d + 4; i += kThreads) acc_part[i] = 0.f;
  __syncthreads();
  if (tid < 64) {                                  // m_loc = max score of the tile
    float m = p_s[tid];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (tid == 0) sh_m = m;
  }
  {
    // LPR lanes per feature row (a power of two <= 64; d_phi is a multiple of 16), RPP rows per pass
    int LPR = 4;
    while (LPR * 2 <= min(dphi / 4, 64)) LPR *= 2;
    const int RPP = kThreads / LPR, seg = tid % LPR, rsub = tid / LPR;
    const float* phiq = (const float*)(blk + g.off_phiq) + (size_t)gq * dphi;
    // feature row of tile entry `row`: the cached row of its token, or (MLP maps without a cache) row i0 + row of
    // the features the step recomputed for this head's retrieved list
    const float* cache_h = g.sel_feat ? (const float*)(blk + g.off_selphi) + ((size_t)gq * g.max_K + i0) * dphi
                                      : pr.phi_cache + (size_t)h * n * dphi;
    auto feat_row = [&](int row) -> size_t { return g.sel_feat ? (size_t)min(row, cnt - 1) : (size_t)(p_tok[row] - g.n_sink); };
    for (int r0 = 0; r0 < kPairsPerWG; r0 += RPP * 4) {
      float zz[4] = {0.f, 0.f, 0.f, 0.f};
      for (int c4 = seg; c4 < dphi / 4; c4 += LPR) {        // (one round when d_phi <= 256)
        const float4 pq = *(const float4*)(phiq + c4 * 4);
        float4 f[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int row = min(r0 + k * RPP + rsub, kPairsPerWG - 1);
          const u32x4 t = gload128(cache_h + feat_row(row) * dphi + c4 * 4);
          f[k] = make_float4(__uint_as_float(t.x), __uint_as_float(t.y), __uint_as_float(t.z), __uint_as_float(t.w));
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
          zz[k] = fmaf(pq.x, f[k].x, fmaf(pq.y, f[k].y, fmaf(pq.z, f[k].z, fmaf(pq.w, f[k].w, zz[k]))));
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        for (int o = LPR >> 1; o >= 1; o >>= 1) zz[k] += __shfl_xor(zz[k], o);
        const int row = r0 + k * RPP + rsub;
        if (seg == 0 && row < kPairsPerWG) p_z[row] = row < cnt ? zz[k] : 0.f;
      }
    }
  }
  __syncthreads();
  if (tid < kPairsPerWG) p_w[tid] = tid < cnt ? __expf(p_s[tid] - sh_m) : 0.f;
  __syncthreads();

  weighted_value_sums<T>(g, pr, head_off, p_tok, p_w, p_z, cnt, red, acc_part, true);
  if (tid < d) { part[4 + tid] = acc_part[4 + tid]; part[4 + d + tid] = acc_part[4 + d + tid]; }
  if (tid == 0) {
    float Z = 0.f, zs = 0.f;
    for (int i = 0; i < cnt; ++i) { Z += p_w[i]; zs += p_z[i]; }
    part[0] = sh_m; part[1] = Z; part[2] = zs; part[3] = (float)cnt;
  }
}

// ------------------------------------------------------------------------------------
// merge: grid (Hq, n_problems); see merge_head.h
// ------------------------------------------------------------------------------------
template <bool PRE>
__global__ __launch_bounds__(kThreads) void merge_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                         char* __restrict__ ws, int mode) {
  merge_head<PRE>(g, probs, ws, (int)blockIdx.x, (int)blockIdx.y, mode);
}

void launch_gather(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  dim3 grid(g.n_tiles + g.n_atiles, g.Hq, g.n_problems);
  if (g.cache || g.sel_feat) {
    if (g.dtype == TKPHI_BF16) TKPHI_LAUNCH(ST_GATHER, gather_cached_kernel<uint16_t>, grid, dim3(kThreads), 0, s, g, probs, ws);
    else TKPHI_LAUNCH(ST_GATHER, gather_cached_kernel<float>, grid, dim3(kThreads), 0, s, g, probs, ws);
  } else if (g.use_mfma) {
    if (g.d == 128) TKPHI_LAUNCH(ST_GATHER, gather_mfma_kernel<128>, grid, dim3(kThreads), 0, s, g, probs, ws);
    else TKPHI_LAUNCH(ST_GATHER, gather_mfma_kernel<64>, grid, dim3(kThreads), 0, s, g, probs, ws);
  } else if (g.dtype == TKPHI_BF16) {
    TKPHI_LAUNCH(ST_GATHER, gather_kernel<uint16_t>, grid, dim3(kThreads), 0, s, g, probs, ws);
  } else {
    TKPHI_LAUNCH(ST_GATHER, gather_kernel<float>, grid, dim3(kThreads), 0, s, g, probs, ws);
  }
}

void launch_merge(const Geom& g, const tkphi_problem* probs, char* ws, int mode, bool pre, hipStream_t s) {
  dim3 grid(g.Hq, g.n_problems);
  if (pre) TKPHI_LAUNCH(ST_MERGE, merge_kernel<true>, grid, dim3(kThreads), 0, s, g, probs, ws, mode);
  else TKPHI_LAUNCH(ST_MERGE, merge_kernel<false>, grid, dim3(kThreads), 0, s, g, probs, ws, mode);
}

}  // namespace tkphi
