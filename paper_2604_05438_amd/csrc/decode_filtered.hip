// Decode front end of the filtered pipeline (bf16 caches on the matrix cores).
//
// The exhaustive Top-K over the mid-region (Sec. "Models, tasks, and protocol") needs every score
// s_i = q . k_i / sqrt(d_h) once, but only the scores that can still reach the top K have to
// leave the chip.  Two kernels:
//
//   decode_prep     one small launch of independent jobs that need no selection:
//                   * sample: per KV head, the scores of an evenly spaced sample of mid-region rows
//                     -> per query head a lower bound of the K-th largest score (a bin edge chosen so
//                     that the sample count above it exceeds its expectation at the K-th score by six
//                     standard deviations); the bound only prunes: the select kernel verifies that at
//                     least K tokens passed and otherwise rescans the head without a bound
//                   * phi:    phi_q(q) of a query head (App. "Head-wise phi architecture": per query
//                     head, once per step) and the summary terms S_M^T phi_q, phi_q . u_M that
//                     eq. (subtraction) and eq. (hybrid_merge) start from
//                   * anchor: the exact terms of eq. (exact_terms) over a tile of 64 anchors (sink,
//                     tail, generated tokens of eq. (implemented_decode))
//   score_filtered  the streaming pass over all mid-region keys, each KV head read once for its G
//                   query heads; a score goes to memory only if its key is >= the head's bound
//                   (about 2-3 K tokens per head instead of |M|), appended to per-wavefront lists.
#include <algorithm>

#include "decode_side.h"
#include "score_tile.h"
#include "tkphi_internal.h"

namespace tkphi {

#ifdef TKPHI_PHASE_CLOCK
#define TKPHI_WAVE_MARK(ws, base)                                                                               \
  do {                                                                                                          \
    if ((threadIdx.x & 63) == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)                       \
      ((unsigned long long*)((ws) + 16))[(base) + (threadIdx.x >> 6)] = wall_clock64();                         \
  } while (0)
#else
#define TKPHI_WAVE_MARK(ws, base) do {} while (0)
#endif

constexpr int kPrepThreads = 1024;
constexpr int kPrepWaves = kPrepThreads / 64;

// Rows of the mid-region whose scores are sampled for a problem with n mid tokens: everything up to 1024
// tokens; beyond that n / 64 rows (at least 512, at most 1024) in evenly spaced groups of 16 consecutive rows
// (one matrix-core tile, one 4 KB page of 256-byte rows: scattered single rows cost a page walk each).
__device__ __forceinline__ int sample_size(int n) {
  return n <= 1024 ? n : min(1024, max(512, n / 64)) / 16 * 16;
}
// mid row of sample si (0 <= si < m)
__device__ __forceinline__ int sample_row(int si, int n, int m) {
  return m >= n ? si : (si >> 4) * (n / (m >> 4)) + (si & 15);
}

// ---- sample job: one workgroup per (problem, KV head) ------------------------------------------------
// LDS: sc [G][1024] sampled scores, hist [G][kBins], nin [G], inb [G][kInBin] keys of the boundary bin
constexpr int kInBin = 256;
constexpr int kSigmas = 4;             // margin of the sampled bound in standard deviations (a miss costs one rescan)
template <int D, int TPI>
__device__ __forceinline__ void prep_sample(const Geom& g, const tkphi_problem& pr, char* blk, int h, float* sc, uint32_t* hist,
                                            uint32_t* inb, int* nin, char* stage_all) {
  constexpr int KS = D / 32, TOK = TPI * 16;
  // The sampled key rows are loaded whole-row-wise (a load instruction covers 64 / LPRW complete rows: one
  // workgroup pulls 2.6 times the bytes per second that it gets with the 16 rows x 64 bytes of the MFMA operand
  // layout) and pass through a wavefront-private LDS strip of one 16-row tile into the operand layout.
  constexpr int LPRW = D / 8, RPI = 64 / LPRW, NLD = TOK / RPI, ROWP = D * 2 + 16;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, r = lane & 15, kg = lane >> 4;
  const int G = g.G;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int Ksel = max(0, min(min(pr.topk, n), g.max_K));
  uint32_t* thr = (uint32_t*)(blk + g.off_thr) + h * G;
  if (n == 0 || Ksel == 0 || g.sel_test == 1) {         // nothing to retrieve (or test: a bound nothing passes)
    if (tid < G) thr[tid] = 0xffffffffu;
    return;
  }
  if (g.sel_test == 2) {                                // test: no pruning at all
    if (tid < G) thr[tid] = 0u;
    return;
  }
  const int m = sample_size(n);
  TKPHI_PHASE((blk - g.off_problem0), 3);
  TKPHI_WAVE_MARK((blk - g.off_problem0), 64);       // sample job entered
  for (int i = tid; i < G * kBins; i += kPrepThreads) hist[i] = 0u;
  if (tid < G) nin[tid] = 0;
  ScoreFrag bq[KS];
  load_query_frags<D>(g, pr, h, bq);
  const size_t row_bytes = (size_t)pr.stride_tok * 2;
  const char* K0 = (const char*)pr.K + ((size_t)h * pr.stride_head + (size_t)g.n_sink * pr.stride_tok) * 2 + (size_t)(lane % LPRW) * 16;
  char* stage = stage_all + (size_t)wv * 16 * ROWP;
  TKPHI_WAVE_MARK((blk - g.off_problem0), 80);       // before the key loads
  for (int i0 = wv * TOK; i0 < m; i0 += kPrepWaves * TOK) {
    u32x4 raw[NLD];
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
      const int si = min(i0 + u * RPI + lane / LPRW, m - 1);
      raw[u] = gload128(K0 + (size_t)sample_row(si, n, m) * row_bytes);
    }
    __builtin_amdgcn_sched_barrier(0);
    TKPHI_WAVE_MARK((blk - g.off_problem0), 96);     // loads issued
#ifdef TKPHI_PHASE_CLOCK
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
    TKPHI_WAVE_MARK((blk - g.off_problem0), 112);    // loads complete
#pragma unroll
    for (int t = 0; t < TPI; ++t) {
      // tile t = rows 16 t .. 16 t + 15 of the wavefront's share = load instructions 16 t / RPI .. ; LDS operations of
      // one wavefront execute in order, so the strip needs no barrier
#pragma unroll
      for (int u = t * 16 / RPI; u < (t + 1) * 16 / RPI; ++u)
        *(u32x4*)(stage + (u * RPI + lane / LPRW - t * 16) * ROWP + (lane % LPRW) * 16) = raw[u];
      ScoreFrag a[KS];
#pragma unroll
      for (int j = 0; j < KS; ++j) a[j].u = *(const u32x4*)(stage + r * ROWP + j * 64 + kg * 16);
      st_floatx4 acc = (st_floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < KS; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j].v, bq[j].v, acc, 0, 0, 0);
      // lane (r < G, kg) holds head r's scores of samples i0 + t 16 + 4 kg + {0..3}: to LDS, so that every lane
      // takes part in what follows (12 of 64 lanes hold all the scores here)
      if (r < G) *(st_floatx4*)(sc + r * 1024 + i0 + t * 16 + 4 * kg) = acc;
    }
  }
  __syncthreads();
  TKPHI_PHASE((blk - g.off_problem0), 4);
  // thread t <-> sample t: first-level histogram per head
  uint32_t key[kMaxGroup];
#pragma unroll
  for (int gl = 0; gl < kMaxGroup; ++gl) {
    if (gl < G && tid < m) {
      key[gl] = score_key(sc[gl * 1024 + tid] * g.score_scale + 0.0f);
      atomicAdd(&hist[gl * kBins + key_bin(key[gl])], 1u);
    }
  }
  __syncthreads();
  TKPHI_PHASE((blk - g.off_problem0), 5);
  // The whole mid-region sampled: the bound is the K-th score itself.  Otherwise: the tau-th largest sampled
  // score, tau = mu + kSigmas sqrt(mu) + 2 with mu = K m / n: the number of samples above the true K-th
  // score has mean <= mu and standard deviation <= sqrt(mu), so the bound lies below the K-th score except
  // with the tail probability of kSigmas standard deviations.
  int tau = Ksel;
  if (m < n) {
    const float mu = (float)Ksel * (float)m / (float)n;
    tau = (int)ceilf(mu + (float)kSigmas * sqrtf(mu) + 2.f);
  }
  __shared__ int sh_bin[kMaxGroup], sh_rem[kMaxGroup];
  if (wv < G) {
    const uint32_t* hrow = hist + wv * kBins + lane * 8;               // lane owns bins 8 lane .. 8 lane + 7
    uint32_t sfx[8], run = 0;
#pragma unroll
    for (int e = 7; e >= 0; --e) { run += hrow[e]; sfx[e] = run; }
    uint32_t x = run;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t y = __shfl_down(x, o);
      if (lane + o < 64) x += y;
    }
    const uint32_t above = x - run;
    int best = -1, rem = 0;                                            // highest bin b with count(>= b) >= tau; tau - count(> b)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if ((int)(sfx[e] + above) >= tau) { best = lane * 8 + e; rem = tau - (int)(sfx[e] + above - hrow[e]); }
    }
    int top = best;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) top = max(top, __shfl_xor(top, o));
    if (best == top && best >= 0 && (lane * 8 <= top && top < lane * 8 + 8)) { sh_bin[wv] = top; sh_rem[wv] = rem; }
    if (top < 0 && lane == 0) { sh_bin[wv] = -1; sh_rem[wv] = 0; }
  }
  __syncthreads();
  // inside that bin: the rem-th largest sampled key is the bound (ranked by counting; the bin holds a few dozen samples)
#pragma unroll
  for (int gl = 0; gl < kMaxGroup; ++gl) {
    if (gl < G && tid < m && sh_bin[gl] >= 0 && key_bin(key[gl]) == sh_bin[gl]) {
      const int at = atomicAdd(&nin[gl], 1);
      if (at < kInBin) inb[gl * kInBin + at] = key[gl];
    }
  }
  __syncthreads();
  if (wv < G) {
    const int gl = wv, cnt = nin[gl], rem = sh_rem[gl], b = sh_bin[gl];
    uint32_t edge;
    if (tau > m || b < 0) edge = 0u;                                   // more than the sample holds: no pruning
    else if (cnt > kInBin) edge = bin_lower_key(b);                    // (a very full bin: its lower edge)
    else {
      edge = 0u;
      for (int j = lane; j < cnt; j += 64) {
        const uint32_t mine = inb[gl * kInBin + j];
        int ge = 0;                                                    // samples of the bin with key >= mine, ties included
        for (int i = 0; i < cnt; ++i) ge += inb[gl * kInBin + i] >= mine ? 1 : 0;
        // the largest key with at least rem keys >= it
        if (ge >= rem) edge = max(edge, mine);
      }
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) edge = max(edge, (uint32_t)__shfl_xor((int)edge, o));
    }
    if (lane == 0) thr[gl] = edge;
  }
}

// ---- phi job: one workgroup per query head ----------------------------------------------------------------
// phi_q -> workspace; sphi[c] = sum_j phi_q[j] S[h][j][c]; uphi = sum_j phi_q[j] u[h][j].  Every global load
// (S, u, the rows of Wq, q, the biases) is issued before anything is consumed: one memory round trip.
// Sums run in a fixed order.
__device__ __forceinline__ void prep_phi(const Geom& g, const tkphi_problem& pr, char* blk, int gq, float* pu /*[kMaxDim]*/,
                                         float* sh_phiq /*[kMaxDim]*/, float* red /*[4096]*/) {
  const int tid = threadIdx.x, d = g.d, dphi = g.dphi, h = gq / g.G;
  const int QPR = d / 4, NG = kPrepThreads / QPR;     // float4 per row of S; feature groups (32 for d = 128, 64 for d = 64)
  const int jg = tid / QPR, c4 = tid % QPR;
  const int per = (dphi + NG - 1) / NG;               // features per group (<= 8)
  const int j0 = jg * per, j1 = min(dphi, j0 + per);
  const float* __restrict__ S = pr.S + (size_t)h * dphi * d;
  constexpr int MAXF = 8;
  u32x4 sv[MAXF];
#pragma unroll
  for (int k = 0; k < MAXF; ++k)
    if (j0 + k < j1) sv[k] = gload128(S + (size_t)(j0 + k) * d + c4 * 4);
  const float uj = tid < dphi ? pr.u[(size_t)h * dphi + tid] : 0.f;
  // rows of Wq: LPR lanes per row (16 bytes each), rows_pp rows per pass, at most 4 passes (d_phi <= 256)
  const int LPR = d / 8, seg = tid % LPR, row_in = tid / LPR, rows_pp = kPrepThreads / LPR;
  constexpr int MAXP = 4;
  u32x4 wv[MAXP];
  float bj[MAXP];
#pragma unroll
  for (int k = 0; k < MAXP; ++k) {
    if (k * rows_pp >= dphi) break;                   // (uniform)
    const int j = min(k * rows_pp + row_in, dphi - 1);
    wv[k] = gload128((const char*)pr.Wq + (((size_t)gq * dphi + j) * d + seg * 8) * 2);
    bj[k] = pr.bq[(size_t)gq * dphi + j];
  }
  const u32x4 qv = gload128((const char*)pr.q + ((size_t)gq * d + seg * 8) * 2);
  float qx[8];
  Elem<uint16_t>::unpack(make_uint4(qv.x, qv.y, qv.z, qv.w), qx);
  float nrm = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) nrm = fmaf(qx[e], qx[e], nrm);
  for (int o = LPR >> 1; o >= 1; o >>= 1) nrm += __shfl_xor(nrm, o);
  float* phiq = (float*)(blk + g.off_phiq) + (size_t)gq * dphi;
#pragma unroll
  for (int k = 0; k < MAXP; ++k) {
    if (k * rows_pp >= dphi) break;
    const int jr = k * rows_pp + row_in;
    float x[8];
    Elem<uint16_t>::unpack(make_uint4(wv[k].x, wv[k].y, wv[k].z, wv[k].w), x);
    float dot = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) dot = fmaf(x[e], qx[e], dot);
    for (int o = LPR >> 1; o >= 1; o >>= 1) dot += __shfl_xor(dot, o);
    if (jr < dphi && seg == 0) {
      const float f = expf(g.a * dot - g.c * nrm + bj[k]);
      phiq[jr] = f;
      sh_phiq[jr] = f;
    }
  }
  __syncthreads();
  float4 sacc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int k = 0; k < MAXF; ++k) {
    if (j0 + k < j1) {
      const float pj = sh_phiq[j0 + k];
      sacc.x = fmaf(pj, __uint_as_float(sv[k].x), sacc.x); sacc.y = fmaf(pj, __uint_as_float(sv[k].y), sacc.y);
      sacc.z = fmaf(pj, __uint_as_float(sv[k].z), sacc.z); sacc.w = fmaf(pj, __uint_as_float(sv[k].w), sacc.w);
    }
  }
  *(float4*)(red + jg * d + c4 * 4) = sacc;           // NG d = 4096 floats
  if (tid < dphi) pu[tid] = sh_phiq[tid] * uj;        // phi_q[j] u[j], summed below in feature order
  __syncthreads();
  if (tid < d) {
    float a = 0.f;
    for (int k = 0; k < NG; ++k) a += red[k * d + tid];
    ((float*)(blk + g.off_sphi))[(size_t)gq * d + tid] = a;
  } else if (tid == 64 * (kPrepWaves - 1)) {
    float a = 0.f;
    for (int j = 0; j < dphi; ++j) a += pu[j];
    ((float*)(blk + g.off_uphi))[gq] = a;
  }
}

// ---- anchor job: one workgroup per (query head, tile of 64 anchors) -------------------------------------------
// Anchors are the rows [0, n_sink) u [L - n_tail, L) (every row if the mid-region is empty) followed by the
// generated tokens [L, L + n_gen).  Writes the tile's partial in the layout of the gather kernels:
// [m_loc, Z_loc, 0, count, nu_loc[d], 0[d]].
__device__ __forceinline__ void prep_anchor(const Geom& g, const tkphi_problem& pr, char* blk, int gq, int batch, float* a_s /*[64]*/,
                                            float* a_w /*[64]*/, float* red /*[16][128]*/) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, d = g.d, h = gq / g.G;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int n_prefill = n > 0 ? g.n_sink + g.n_tail : pr.L;
  const int n_anchor = n_prefill + min(max(pr.n_gen, 0), g.max_gen);
  const int base = batch * 64;
  if (base >= n_anchor) return;
  const int cnt = min(64, n_anchor - base);
  float* part = (float*)(blk + g.off_part) + ((size_t)gq * (g.n_tiles + g.n_atiles) + g.n_tiles + batch) * g.part_stride;
  const int LPR = d / 8, seg = tid % LPR, row = tid / LPR;          // 16-byte segments per row; rows >= 64 idle (d = 64)
  const bool live = row < cnt;
  const int a = base + min(row, cnt - 1);
  const int tok = a >= n_prefill ? pr.L + (a - n_prefill) : (n > 0 && a >= g.n_sink) ? (pr.L - g.n_tail + (a - g.n_sink)) : a;
  const size_t off = ((size_t)h * pr.stride_head + (size_t)tok * pr.stride_tok + seg * 8) * 2;
  const u32x4 kv = gload128((const char*)pr.K + off), vv = gload128((const char*)pr.V + off);
  const u32x4 qv = gload128((const char*)pr.q + ((size_t)gq * d + seg * 8) * 2);
  float kx[8], vx[8], qx[8];
  Elem<uint16_t>::unpack(make_uint4(kv.x, kv.y, kv.z, kv.w), kx);
  Elem<uint16_t>::unpack(make_uint4(vv.x, vv.y, vv.z, vv.w), vx);
  Elem<uint16_t>::unpack(make_uint4(qv.x, qv.y, qv.z, qv.w), qx);
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) s = fmaf(kx[e], qx[e], s);
  for (int o = LPR >> 1; o >= 1; o >>= 1) s += __shfl_xor(s, o);
  if (seg == 0 && row < 64) a_s[row] = live ? s * g.score_scale + 0.0f : -INFINITY;
  __syncthreads();
  if (wv == 0) {
    const float sl = a_s[lane];
    float mb = sl;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mb = fmaxf(mb, __shfl_xor(mb, o));
    const float w = lane < cnt ? __expf(sl - mb) : 0.f;
    a_w[lane] = w;
    float Z = w;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) Z += __shfl_xor(Z, o);
    if (lane == 0) { part[0] = mb; part[1] = Z; part[2] = 0.f; part[3] = (float)cnt; }
  }
  __syncthreads();
  const float w = live ? a_w[row] : 0.f;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = w * vx[e];
  // rows of one wavefront that share a segment: lanes seg, seg + LPR, ...
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], o);
  }
  if (lane < LPR) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wv * 128 + lane * 8 + e] = acc[e];
  }
  __syncthreads();
  if (tid < d) {
    float x = 0.f;
    for (int k = 0; k < kPrepWaves; ++k) x += red[k * 128 + tid];
    part[4 + tid] = x;
    part[4 + d + tid] = 0.f;
  }
}

// grid (jobs, Hkv, n_problems), 1024 threads; job = job0 + blockIdx.x of 1 + G (1 + n_atiles).  Job 0: sample; jobs
// 1 .. G: phi of the group's query heads; then n_atiles anchor tiles per query head.  One launch for a few
// problems; for batches the sample jobs (which need ~90 KB of LDS: one workgroup per CU) and the rest (16 KB) are
// two launches, so that the many small jobs are not held to one workgroup per CU.
template <int D, int TPI>
__global__ __launch_bounds__(kPrepThreads) void decode_prep_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                   char* __restrict__ ws, int job0) {
  // sample job: sc [G][1024] floats + hist [G][kBins] + inb [G][kInBin] (G (4096 + 2048 + 1024) bytes), then the
  // staging strips, 16 wavefronts x 16 rows x (2 D + 16) bytes; phi / anchor jobs: 16 KB of reduction scratch
  extern __shared__ __attribute__((aligned(16))) float sh_dyn[];
  __shared__ float sh_a[kMaxDim], sh_b[kMaxDim];
  __shared__ int sh_nin[kMaxGroup];
  const int job = job0 + (int)blockIdx.x, h = blockIdx.y, p = blockIdx.z;
  TKPHI_PHASE(ws, 0);
  TKPHI_WAVE_MARK(ws, 32);                           // kernel entered

  if (job == 0 && h == 0 && p == 0) write_device_status(g, probs, ws, true);
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  char* blk = problem_block(g, ws, p);
  TKPHI_PHASE(ws, 1);
  TKPHI_WAVE_MARK(ws, 48);                           // problem record loaded
#ifdef TKPHI_PHASE_CLOCK
  if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) ((unsigned long long*)(ws + 16))[26] = clock64();
#endif
  if (job == 0) {
    uint32_t* hist = (uint32_t*)(sh_dyn + g.G * 1024);
    prep_sample<D, TPI>(g, pr, blk, h, sh_dyn, hist, hist + g.G * kBins, sh_nin, (char*)(hist + g.G * (kBins + kInBin)));
    TKPHI_PHASE(ws, 2);
#ifdef TKPHI_PHASE_CLOCK
    if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) ((unsigned long long*)(ws + 16))[27] = clock64();
#endif
  } else if (job <= g.G) {
    // (also: nobody has arrived yet at this head's merge, see the fused select + gather kernel)
    if (threadIdx.x == 0) ((uint32_t*)(blk + g.off_mcount))[h * g.G + job - 1] = 0u;
    prep_phi(g, pr, blk, h * g.G + job - 1, sh_a, sh_b, sh_dyn);
  } else {
    const int j = job - 1 - g.G;
    prep_anchor(g, pr, blk, h * g.G + j / g.n_atiles, j % g.n_atiles, sh_a, sh_b, sh_dyn);
  }
}

// grid (n_scan_chunks, Hkv, n_problems), 256 threads: wavefront w is slot w of the workgroup's chunk.
template <int D, int TPI, bool STREAM>
__global__ __launch_bounds__(kThreads) void score_filtered_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                  char* __restrict__ ws) {
  const int p = blockIdx.z, h = blockIdx.y;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int n_chunks = (n + g.scan_chunk - 1) / g.scan_chunk;
  // (chunk indices rotated per head and problem: workgroups go to the 8 XCDs round-robin by linear
  // index and the short sequences of a ragged batch have no late chunks)
  const int chunk = ((int)blockIdx.x + h + p * g.Hkv) % (int)gridDim.x;
  if (chunk >= n_chunks) return;
  char* blk = problem_block(g, ws, p);
  const int r = threadIdx.x & 15;
  ScoreFrag bq[D / 32];
  load_query_frags<D>(g, pr, h, bq);
  const uint32_t edge_r = r < g.G ? ((const uint32_t*)(blk + g.off_thr))[h * g.G + r] : 0xffffffffu;
  extern __shared__ __attribute__((aligned(16))) uint2 sh_heads[];      // [4 wavefronts][G][cand_T]
  const int wv = (int)(threadIdx.x >> 6);
  scan_wave_slot<D, TPI, TPI, STREAM>(g, pr, blk, h, n, n_chunks, chunk, wv, bq, edge_r, -1, false,
                         g.head_strip ? sh_heads + (size_t)wv * g.G * g.cand_T : nullptr);
}

// The phi and anchor jobs of a batch: grid (G (1 + n_atiles), Hkv, n_problems), 256 threads; job j < G: phi of query
// head h G + j (and that head's arrival counter <- 0), then n_atiles anchor tiles per query head.
__global__ __launch_bounds__(kThreads) void decode_side_kernel(Geom g, const tkphi_problem* __restrict__ probs, char* __restrict__ ws) {
  __shared__ __attribute__((aligned(16))) float sh_f[2 * kMaxDim + 1024];
  const int job = blockIdx.x, h = blockIdx.y, p = blockIdx.z;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  char* blk = problem_block(g, ws, p);
  if (job < g.G) {
    if (threadIdx.x == 0) ((uint32_t*)(blk + g.off_mcount))[h * g.G + job] = 0u;
    side_phi(g, pr, blk, h * g.G + job, sh_f, sh_f + kMaxDim, sh_f + 2 * kMaxDim);
  } else {
    const int j = job - g.G;
    side_anchor(g, pr, blk, h * g.G + j / g.n_atiles, j % g.n_atiles, sh_f, sh_f + 64, sh_f + 128);
  }
}

void launch_prep(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  dim3 grid(1 + g.G * (1 + g.n_atiles), g.Hkv, g.n_problems);
  // <= 56 KB at G = 8, plus 68 KB (d = 128) / 36 KB (d = 64) of staging strips
  const size_t lds = std::max((size_t)g.G * (1024 + kBins + kInBin) * 4 + (size_t)kPrepWaves * 16 * (g.d * 2 + 16), (size_t)16384);
  const void* fn = g.d == 128 ? (const void*)decode_prep_kernel<128, 4> : (const void*)decode_prep_kernel<64, 8>;
  const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) { set_error("hipFuncSetAttribute(%zu bytes of LDS): %s", lds, hipGetErrorString(e)); return; }
  const int n_jobs = 1 + g.G * (1 + g.n_atiles);
  if ((long)n_jobs * g.Hkv * g.n_problems <= 1024) {
    if (g.d == 128) TKPHI_LAUNCH(ST_PREP, (decode_prep_kernel<128, 4>), grid, dim3(kPrepThreads), lds, s, g, probs, ws, 0);
    else TKPHI_LAUNCH(ST_PREP, (decode_prep_kernel<64, 8>), grid, dim3(kPrepThreads), lds, s, g, probs, ws, 0);
    return;
  }
  dim3 grid_a(1, g.Hkv, g.n_problems), grid_b(n_jobs - 1, g.Hkv, g.n_problems);
  if (g.d == 128) TKPHI_LAUNCH(ST_PREP, (decode_prep_kernel<128, 4>), grid_a, dim3(kPrepThreads), lds, s, g, probs, ws, 0);
  else TKPHI_LAUNCH(ST_PREP, (decode_prep_kernel<64, 8>), grid_a, dim3(kPrepThreads), lds, s, g, probs, ws, 0);
  TKPHI_LAUNCH(ST_PHIQ, decode_side_kernel, grid_b, dim3(kThreads), 0, s, g, probs, ws);
}

void launch_score_filtered(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  if (g.max_mid == 0) return;
  dim3 grid(g.n_scan_chunks, g.Hkv, g.n_problems);
  const size_t lds = g.head_strip ? (size_t)4 * g.G * g.cand_T * sizeof(uint2) : 0;   // the wavefronts' strips of list heads
  if (g.d == 128 && g.stream_keys) TKPHI_LAUNCH(ST_SCORE, (score_filtered_kernel<128, 4, true>), grid, dim3(kThreads), lds, s, g, probs, ws);
  else if (g.d == 128) TKPHI_LAUNCH(ST_SCORE, (score_filtered_kernel<128, 4, false>), grid, dim3(kThreads), lds, s, g, probs, ws);
  else TKPHI_LAUNCH(ST_SCORE, (score_filtered_kernel<64, 8, false>), grid, dim3(kThreads), lds, s, g, probs, ws);
}

}  // namespace tkphi
