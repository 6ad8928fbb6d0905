// Internal definitions shared by the host layer and the HIP kernels of libtkphi.
#pragma once

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tkphi.h"

namespace tkphi {

constexpr int kThreads = 256;          // default workgroup: 256 threads (4 wavefronts)
constexpr int kSelThreads = 1024;      // topk_select: one 1024-thread workgroup per query head
constexpr int kMaxGroup = 8;           // query heads per KV head
constexpr int kMaxDim = 256;           // d_head / d_phi upper bound of the generic kernels

// ---- score histogram --------------------------------------------------------------
// First-level bins of the radix select: a monotone non-decreasing map of the score to
// [0, kBins): sign, 16 exponents (2^-8 .. 2^8, clamped outside) and 4 mantissa bits.
// Only monotonicity matters for correctness; the resolution keeps the boundary bin (the
// tokens whose exact rank must still be resolved) small for attention-like scores.
constexpr int kExpLo = 119;
constexpr int kExpHi = 134;
constexpr int kMagBins = (kExpHi - kExpLo + 1) * 16;   // 256
constexpr int kBins = 2 * kMagBins;                     // 512
constexpr int kCandCap = 4096;         // boundary-bin candidates resolved in LDS
constexpr int kPairsPerWG = 64;        // gather: retrieved tokens per workgroup (16 per wavefront)

// ---- launch geometry + workspace layout -------------------------------------------
struct Geom {
  int Hq, Hkv, G, d, dphi, n_sink, n_tail, dtype;
  int use_mfma;          // bf16 storage with d_phi == d_head: matrix-core kernels
  int n_problems, max_L, max_K, max_mid;
  int mid_stride;        // floats per score row (multiple of 64)
  int scan_chunk, n_scan_chunks;     // score_mid: mid tokens per workgroup
  int scan_unit;         // tokens a score_mid workgroup takes per iteration (scan_chunk is a multiple)
  int phi_kind, d_emb;   // tkphi_phi_kind; MLP width
  int max_gen;           // bound of tkphi_problem::n_gen (generated tokens, exact)
  int mlp_mode;          // MLP build: tkphi_tuning::mlp_mode
  int mlp_block;         // MLP build: tokens per KV head whose activations are held at once (multiple of 64)
  int mlp_group;         // MLP maps: problems per chain launch (their packed weights are held together)
  int sel_feat;          // 1: MLP maps without a feature cache: decode recomputes the features of the retrieved keys
  int cache;             // 1: key features are stored by the build and gathered by decode (cfg.cache_features)
  int diag;              // 1: the select emit pass also reduces the entropy / mass diagnostics
  int interleave;        // 1: chunk c owns the units c, c + n_chunks, c + 2 n_chunks, ... of its problem
                         // (all workgroups sweep the key cache together); 0: one contiguous range
  int filtered;          // 1: decode may run the filtered pipeline (prep, score_filtered, select_gather, merge):
                         // bf16 matrix-core shapes, exp-affine maps, budgets well below the mid-region size
  int cand_T;            // filtered pipeline: entries of a candidate list kept in the compact array (multiple of 12)
  int head_strip;        // 1: the score pass collects the compact list heads in LDS (4 G cand_T entries fit 32 KB)
  int stream_keys;       // 1: the filtered score pass reads the keys with non-temporal loads
  int sel_test;          // tkphi_tuning::select_test (0 unless a test forces the rescan or the no-pruning path)
  int n_tiles;           // gather: ceil(max_K / kPairsPerWG) retrieved-token tiles per query head; one partial each
  int sg_split;          // filtered pipeline: workgroups per query head of the fused select + gather kernel (0 if it cannot run);
                         // that pipeline's launchers get a Geom whose n_tiles is this number
  int n_atiles;          // gather: ceil((n_sink + n_tail + max_gen) / 64) tiles of exact anchors + generated tokens per query head (>= 1)
  int build_chunk, n_build_chunks;   // summary_build: mid tokens per workgroup
  int part_stride;       // floats per partial: 2*d + 4
  float score_scale, a, c;
  // byte offsets inside the workspace
  size_t off_status;     // uint32 device status word
  size_t off_problem0;   // first per-problem block
  size_t per_problem;    // bytes per problem block
  // offsets inside a per-problem block
  size_t off_scores;     // float    [Hq][mid_stride]            mid-region scores (spill pipeline)
  size_t off_candf;      // uint2    [Hq][n_scan_chunks][4][scan_chunk/4]  candidate lists (score bits, mid index) of the filtered
                         //                                       pipeline at full capacity (entries past the first cand_T of a
                         //                                       list land here); shares its memory with off_scores
  size_t off_candc;      // uint2    [Hq][n_scan_chunks][4][cand_T]  the first cand_T entries of every list
  size_t off_ccount;     // uint32   [Hq][n_scan_chunks][4]      lengths of the candidate lists
  size_t off_resf, off_resc, off_rescount;  // the rescan set: a second candf / candc / ccount, written when the select kernel
                         //                                       rescans a head without a bound, read by its second attempt
  size_t off_thr;        // uint32   [Hq]                        lower bound of the score key per query head
  size_t off_mcount;     // uint32   [Hq]                        filtered pipeline: workgroups of the fused select + gather kernel
                         //                                       that have finished their share of the head (cleared by prep)
  size_t off_sphi;       // float    [Hq][d]                     S_M^T phi_q
  size_t off_uphi;       // float    [Hq]                        phi_q . u_M
  size_t off_hist;       // uint16   [n_scan_chunks][Hq][kBins]  per-chunk histograms
  size_t off_plan;       // SelPlan  [Hq]
  size_t off_diag;       // float    [n_scan_chunks][Hq][4]      per-chunk (max, sum exp, sum (s-max) exp) of the scores
  size_t off_chunkoff;   // int32    [Hq][n_scan_chunks][2]      output offsets of each chunk (above b*, in b*)
  size_t off_cand;       // uint2    [Hq][kCandCap]              boundary-bin candidates (key, mid index)
  size_t off_selidx;     // int32    [Hq][max_K]                 retrieved mid indices
  size_t off_selscore;   // float    [Hq][max_K]                 their scores
  size_t off_phiq;       // float    [Hq][dphi]
  size_t off_mlpq;       // float    [Hq][2][d_emb]                  MLP phi_q: stem / residual stream g, hidden h
  size_t off_selphi;     // float    [Hq][max_K][d_phi]              MLP maps without a feature cache: phi_k of the retrieved keys,
                         //                                       in the order of the retrieved list
  size_t off_part;       // float    [Hq][n_tiles + n_atiles][part_stride]  (retrieved tiles, then anchor tiles)
  size_t off_bpart;      // float    [Hkv][n_build_chunks][dphi*(d+1)]   (build only; aliases the block)
  size_t off_act;        // float    2 x [Hkv][mlp_block][d_emb]          (MLP build only: activations g, h of a token block)
  size_t off_wpack;      // bf16     [mlp_group][Hkv][Ws | W1 | W2 | Wo]  (MLP maps: a group's key-side weights in MFMA-fragment order)
  size_t off_feat;       // float    [mlp_group][Hkv][max_mid][d_phi]     (MLP build without a feature cache: a group's key features)
  size_t decode_bytes;   // what a decode call alone uses (status word + per-problem blocks)
  size_t build_bytes;    // what a summary build alone uses
  size_t total_bytes;    // the larger of decode and build
};

// Fills g for the given bounds; returns TKPHI_OK or the reason the config is unsupported.
tkphi_status make_geom(const tkphi_config* cfg, int n_problems, int max_L, int max_K, Geom* g);
void set_error(const char* fmt, ...);

// Optional per-kernel timing: while g_kernel_timer is set (by tkphi_decode_stage_times, on
// the calling thread) a launch records the kernel's own begin / end on the two events.
enum Stage { ST_SCORE = 0, ST_PLAN, ST_EMIT, ST_RESOLVE, ST_GATHER, ST_MERGE, ST_PHIQ, ST_PREP, ST_SELECT, ST_COUNT, ST_UNTIMED = -1 };
struct KernelTimer {
  hipEvent_t start[ST_COUNT], stop[ST_COUNT];
  bool used[ST_COUNT];
};
extern thread_local KernelTimer* g_kernel_timer;
#define TKPHI_LAUNCH(stage, kernel, grid, block, lds, stream, ...)                                       \
  do {                                                                                                   \
    if (tkphi::g_kernel_timer && (stage) >= 0) {                                                         \
      tkphi::g_kernel_timer->used[(stage)] = true;                                                       \
      hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, tkphi::g_kernel_timer->start[(stage)],     \
                            tkphi::g_kernel_timer->stop[(stage)], 0, __VA_ARGS__);                       \
    } else {                                                                                             \
      hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                                 \
    }                                                                                                    \
  } while (0)

// what `plan` hands to `emit` / `resolve` / gather for one query head
struct SelPlan {
  int32_t bstar;   // boundary bin, -1: nothing to retrieve
  int32_t krem;    // tokens still to take from the boundary bin
  int32_t c_hi;    // tokens in bins above the boundary bin
  int32_t nb;      // tokens in the boundary bin
  int32_t n_sel;   // retrieved tokens K' = min(topk, |M|, max_K)
};
constexpr int kMlpChainWGs = 512;       // persistent workgroups of the one-launch MLP build (two per CU)
constexpr int kMaxScanChunks = 2048;   // chunk offsets are scanned in LDS by `plan`

// kernel launchers (each defined next to its kernels)
void launch_score_mid(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);
void launch_select(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);
void launch_prep(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);              // filtered pipeline
void launch_score_filtered(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);
void launch_select_gather(const Geom& g, const tkphi_problem* probs, char* ws, int mode, hipStream_t s);  // includes the merge
void launch_gather(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);
// `pre`: the prep kernel has already produced the anchor partials and the summary terms S_M^T phi_q, phi_q . u_M
void launch_merge(const Geom& g, const tkphi_problem* probs, char* ws, int mode, bool pre, hipStream_t s);
void launch_build(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);
void launch_mlp_build(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);        // key features + chunk partials
void launch_mlp_sel_features(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);  // -> off_selphi
void launch_mlp_phi_q(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s);        // -> phi_q of every query head
void launch_summary_from_cache(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s, int p0, int np); // -> chunk partials

#ifdef __HIPCC__
// ---- device helpers ------------------------------------------------------------------
__device__ __forceinline__ uint32_t score_key(float s) {
  // order-preserving map float -> uint32 (larger score <=> larger key)
  uint32_t u = __float_as_uint(s);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_score(uint32_t key) {   // inverse of score_key
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

__device__ __forceinline__ int key_bin(uint32_t key) {
  const bool pos = (key & 0x80000000u) != 0;
  const uint32_t mag = pos ? (key & 0x7fffffffu) : (~key & 0x7fffffffu);
  const int e = (int)(mag >> 23);
  const int m4 = (int)((mag >> 19) & 15u);
  int mb;
  if (e < kExpLo) mb = 0;
  else if (e > kExpHi) mb = kMagBins - 1;
  else mb = (e - kExpLo) * 16 + m4;
  return pos ? (kMagBins + mb) : (kMagBins - 1 - mb);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// round-to-nearest-even float -> bf16 bits (finite inputs)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// A feature value as the sum of two bf16 numbers, hi = bf16(f) and lo = bf16(f - hi): 16
// significant bits, which is what the matrix-core summary build contracts against the
// values and what the decode side subtracts for a retrieved token.
// Two features at a time with the packed hardware conversion (v_cvt_pk_bf16_f32, round to
// nearest even): *hi / *lo hold (f0, f1) in their (low, high) halves.
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
__device__ __forceinline__ void split_bf16_pair(float f0, float f1, uint32_t* hi, uint32_t* lo) {
  const bf16x2_t h = {(__bf16)f0, (__bf16)f1};
  const uint32_t hb = __builtin_bit_cast(uint32_t, h);
  const bf16x2_t l = {(__bf16)(f0 - __uint_as_float(hb << 16)), (__bf16)(f1 - __uint_as_float(hb & 0xffff0000u))};
  *hi = hb;
  *lo = __builtin_bit_cast(uint32_t, l);
}
// hi + lo of the low half of a pair
__device__ __forceinline__ float join_bf16_lo(uint32_t hi, uint32_t lo) {
  return __uint_as_float(hi << 16) + __uint_as_float(lo << 16);
}
__device__ __forceinline__ float join_bf16_hi(uint32_t hi, uint32_t lo) {
  return __uint_as_float(hi & 0xffff0000u) + __uint_as_float(lo & 0xffff0000u);
}
// phi(x)[j] = exp(a W_j.x - c |x|^2 + b_j) evaluated as exp2(a2 * (W_j.x) + t2) with
// a2 = a log2(e) and t2 = (b_j - c |x|^2) log2(e): one FMA and one v_exp_f32.  The summary build
// and the decode-side recompute both go through this function.
constexpr float kLog2e = 1.4426950408889634f;
__device__ __forceinline__ float phi_exp2(float dot, float a2, float t2) {
  return __builtin_amdgcn_exp2f(fmaf(a2, dot, t2));
}

// 16-byte loads from global memory.  Pointers that come out of the problem table are
// generic to the compiler; casting to the global address space gives global_load
// instead of flat_load instructions.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* gptr128;
__device__ __forceinline__ u32x4 gload128(const void* p) { return *(gptr128)p; }
__device__ __forceinline__ u32x4 gload128_stream(const void* p) { return __builtin_nontemporal_load((gptr128)p); }

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int per16 = 4;
  __device__ static __forceinline__ void unpack(const uint4& v, float* x) {
    x[0] = __uint_as_float(v.x); x[1] = __uint_as_float(v.y);
    x[2] = __uint_as_float(v.z); x[3] = __uint_as_float(v.w);
  }
  __device__ static __forceinline__ float load1(const void* p, int64_t i) { return ((const float*)p)[i]; }
};
template <> struct Elem<uint16_t> {   // bf16 bits
  static constexpr int per16 = 8;
  __device__ static __forceinline__ void unpack(const uint4& v, float* x) {
    x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xffff0000u);
    x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xffff0000u);
    x[4] = __uint_as_float(v.z << 16); x[5] = __uint_as_float(v.z & 0xffff0000u);
    x[6] = __uint_as_float(v.w << 16); x[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  __device__ static __forceinline__ float load1(const void* p, int64_t i) {
    return bf16_bits_to_float(((const uint16_t*)p)[i]);
  }
};


// ---- query features and device status (side workgroups of the select plan launch) ----
// phi_q(q_g)[j] = exp(a Wq[g][j] . q_g - c |q_g|^2 + bq[g][j]) for query head gq
// (App. "Head-wise phi architecture": the query-side map belongs to the query head and runs once per
// decode step).  LPR lanes per Wq row with one 16-byte load each; all row loads of a head are in flight
// together.  Works for any workgroup size that is a multiple of 64.  qf: LDS, >= kMaxDim floats.
template <typename T>
__device__ __forceinline__ void phi_q_head(const Geom& g, const tkphi_problem& pr, char* blk, int gq, float* qf) {
  constexpr int EPL = Elem<T>::per16;
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int LPR = g.d / EPL, seg = tid % LPR, rows_pp = nthr / LPR;
  constexpr int MAXP = 8;                        // row passes held in flight (128 rows at 16 per pass)
  {
    float* phiq = (float*)(blk + g.off_phiq) + (size_t)gq * g.dphi;
    for (int c = tid; c < g.d; c += nthr) qf[c] = Elem<T>::load1(pr.q, (int64_t)gq * g.d + c);
    __syncthreads();
    for (int j0 = 0; j0 < g.dphi; j0 += rows_pp * MAXP) {
      u32x4 t[MAXP];
      float bj[MAXP];
#pragma unroll
      for (int k = 0; k < MAXP; ++k) {
        if (j0 + k * rows_pp >= g.dphi) break;                          // (uniform) no rows left for this pass
        const int j = min(j0 + k * rows_pp + tid / LPR, g.dphi - 1);   // clamped: every lane loads
        t[k] = gload128((const char*)pr.Wq + (((int64_t)gq * g.dphi + j) * g.d + seg * EPL) * sizeof(T));
        bj[k] = pr.bq[(int64_t)gq * g.dphi + j];
      }
#pragma unroll
      for (int k = 0; k < MAXP; ++k) {
        if (j0 + k * rows_pp >= g.dphi) break;
        const int jr = j0 + k * rows_pp + tid / LPR;
        float x[EPL];
        Elem<T>::unpack(make_uint4(t[k].x, t[k].y, t[k].z, t[k].w), x);
        float dot = 0.f, nrm = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
          const float qe = qf[seg * EPL + e];
          dot = fmaf(x[e], qe, dot);
          nrm = fmaf(qe, qe, nrm);
        }
        for (int o = LPR >> 1; o >= 1; o >>= 1) { dot += __shfl_xor(dot, o); nrm += __shfl_xor(nrm, o); }
        if (jr < g.dphi && seg == 0) phiq[jr] = expf(g.a * dot - g.c * nrm + bj[k]);
      }
    }
  }
}

// out[j] = W[j] . in for a bf16 matrix W [N][Kd] (row-major, 16-byte aligned rows) and an fp32
// vector `in` in LDS; epi(j, dot) consumes row j.  Kd / 8 / SPL lanes share a row with SPL (1 or 2)
// 16-byte loads each; eight loads per lane are in flight and cover rows [j0, j0 + rows_pp 8 / SPL).
// gemv_load issues the loads of one such row group, gemv_consume reduces them: a caller can issue
// the first group early (before `in` is ready) and hand it to gemv_bf16_rows as `pre`.
template <int SPL>
__device__ __forceinline__ void gemv_load(const void* W, int N, int Kd, int j0, u32x4 (&t)[8]) {
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int LPR = Kd / 8 / SPL;
  const int rows_pp = nthr / LPR, row_in = tid / LPR, sl = tid % LPR;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int pass = k / SPL, sg = sl + (k % SPL) * LPR;
    if (j0 + pass * rows_pp >= N) break;                             // (uniform) no rows left for this pass
    const int j = min(j0 + pass * rows_pp + row_in, N - 1);          // clamped: every lane loads
    t[k] = gload128((const char*)W + ((size_t)j * Kd + sg * 8) * 2);
  }
}

template <int SPL, typename F>
__device__ __forceinline__ void gemv_consume(int N, int Kd, int j0, const u32x4 (&t)[8], const float* in, F&& epi) {
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int LPR = Kd / 8 / SPL;
  const int rows_pp = nthr / LPR, row_in = tid / LPR, sl = tid % LPR;
  float dot = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int pass = k / SPL, sg = sl + (k % SPL) * LPR;
    if (j0 + pass * rows_pp >= N) break;
    float x[8];
    Elem<uint16_t>::unpack(make_uint4(t[k].x, t[k].y, t[k].z, t[k].w), x);
#pragma unroll
    for (int e = 0; e < 8; ++e) dot = fmaf(x[e], in[sg * 8 + e], dot);
    if (k % SPL == SPL - 1) {                                        // the row's last segment of this lane
      for (int o = LPR >> 1; o >= 1; o >>= 1) dot += __shfl_xor(dot, o);
      const int jr = j0 + pass * rows_pp + row_in;
      if (sl == 0 && jr < N) epi(jr, dot);
      dot = 0.f;
    }
  }
}

// `pre`: the row group j0 = 0, already loaded with gemv_load<SPL>(W, N, Kd, 0, pre)
template <int SPL, typename F>
__device__ __forceinline__ void gemv_bf16_rows(const void* W, int N, int Kd, const float* in, const u32x4 (&pre)[8], F&& epi) {
  const int rows_pi = (int)blockDim.x / (Kd / 8 / SPL) * (8 / SPL);
  gemv_consume<SPL>(N, Kd, 0, pre, in, epi);
  for (int j0 = rows_pi; j0 < N; j0 += rows_pi) {
    u32x4 t[8];
    gemv_load<SPL>(W, N, Kd, j0, t);
    gemv_consume<SPL>(N, Kd, j0, t, in, epi);
  }
}

// GeLU(x) = x Phi(x) with Phi(x) = erfc(-x / sqrt 2) / 2.  erfc(z) for z >= 0 by the classical
// five-term rational approximation erfc(z) ~ t (a1 + t (a2 + ... + t a5)) exp(-z^2), t = 1 / (1 + p z)
// (Abramowitz & Stegun 7.1.26: absolute error <= 1.5e-7 on erfc, hence <= 0.75e-7 |x| on GeLU, and
// no cancellation for x < 0): a reciprocal, an exponential and seven FMAs instead of the library
// erff, which dominated the hidden layer's epilogue.
__device__ __forceinline__ float gelu_erf(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __frcp_rn(fmaf(0.3275911f, z, 1.0f));
  const float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f), -0.284496736f), 0.254829592f);
  const float erfc_z = poly * __expf(-z * z);                       // erfc(|x| / sqrt 2)
  return 0.5f * x * (x < 0.f ? erfc_z : 2.0f - erfc_z);
}

// device status word: recomputed from the problem lengths by one workgroup per call (decode also
// checks the generated-token counts, which the build does not read)
__device__ __forceinline__ void write_device_status(const Geom& g, const tkphi_problem* probs, char* ws, bool check_gen) {
  int bad = 0;
  for (int i = threadIdx.x; i < g.n_problems; i += blockDim.x) {
    const int Li = probs[i].L, gi = probs[i].n_gen;
    bad |= (Li < 1 || Li > g.max_L || (check_gen && (gi < 0 || gi > g.max_gen))) ? 1 : 0;
  }
  bad = __syncthreads_or(bad);
  if (threadIdx.x == 0) *(uint32_t*)(ws + g.off_status) = bad ? TKPHI_DEV_BAD_LENGTH : 0u;
}

// Development aid (compiled in only with -DTKPHI_PHASE_CLOCK): thread 0 of workgroup (0, 0, 0) stores the
// 100 MHz wall clock at numbered points of a kernel behind the status word (ws + 16 + 8 slot).
#ifdef TKPHI_PHASE_CLOCK
#define TKPHI_PHASE(ws, slot)                                                                                   \
  do {                                                                                                          \
    if (threadIdx.x == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)                              \
      ((unsigned long long*)((ws) + 16))[(slot)] = wall_clock64();                                              \
  } while (0)
#define TKPHI_PHASE_VALUE(ws, slot, v) (((unsigned long long*)((ws) + 16))[(slot)] = (unsigned long long)(v))
#else
#define TKPHI_PHASE(ws, slot) do {} while (0)
#define TKPHI_PHASE_VALUE(ws, slot, v) do {} while (0)
#endif

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits for every global load the wavefront
// has in flight (its fences cover global memory); where a barrier only hands LDS data from one wavefront to
// another, this one lets prefetched global loads stay in flight across it.  Not for data exchanged through
// global memory.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Loads that write LDS directly.  The compiler cannot tell which LDS bytes a pending one will touch and would
// wait for all of them before every LDS read, so they are issued from inline assembly and counted by hand:
// wait_vm_loads<N>() returns when at most N vector memory operations of the wavefront are still in flight
// (they complete in order), and a barrier after it makes every wavefront's share visible to the workgroup.
// 64 lanes x 16 bytes from global memory into LDS at lds_addr (uniform) + 16 * lane; counted by vmcnt.
// (M0 is not on the clobber list - the compiler reserves it; nothing else in these kernels uses it)
// _stream: data read once (non-temporal); the plain form for data other workgroups read again from L2.
__device__ __forceinline__ void load_to_lds16(const void* gsrc, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gsrc), "s"(lds_addr) : "memory");
}
__device__ __forceinline__ void load_to_lds16_stream(const void* gsrc, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" : : "v"(gsrc), "s"(lds_addr) : "memory");
}
// the same with the address as a uniform base plus a 32-bit offset per lane
__device__ __forceinline__ void load_to_lds16(const void* base, uint32_t off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(base), "s"(lds_addr) : "memory");
}
__device__ __forceinline__ void load_to_lds16_stream(const void* base, uint32_t off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" : : "v"(off), "s"(base), "s"(lds_addr) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm_loads() {   // at most N vector memory operations still in flight
  static_assert(N >= 0 && N < 64, "vmcnt has 6 bits");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  asm volatile("" ::: "memory");                    // no LDS read moves above the wait
}

// Stores and loads that are coherent across the whole GPU (the 8 XCDs have separate L2 caches; ordinary accesses may
// stay in, or be served from, the L2 of the XCD they were issued on until a kernel boundary).  For the few words
// one workgroup hands to another inside a launch: much cheaper than a device-wide fence, which writes back a
// whole L2.
__device__ __forceinline__ void store_agent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float load_agent(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// mid-region size of a problem; 0 if the anchors cover everything
__device__ __forceinline__ int mid_size(int L, int n_sink, int n_tail) {
  const int n = L - n_sink - n_tail;
  return n > 0 ? n : 0;
}

// first token of unit k (k = 0 .. scan_chunk / scan_unit - 1) of chunk `chunk`; n_chunks is the chunk
// count of the problem at hand.  Units never overlap, so "token < n" is the only bound to check.
__device__ __forceinline__ int chunk_unit_token(const Geom& g, int n_chunks, int chunk, int k) {
  return g.interleave ? (chunk + k * n_chunks) * g.scan_unit : chunk * g.scan_chunk + k * g.scan_unit;
}

__device__ __forceinline__ char* problem_block(const Geom& g, char* ws, int p) {
  return ws + g.off_problem0 + (size_t)p * g.per_problem;
}
#endif  // __HIPCC__

}  // namespace tkphi
