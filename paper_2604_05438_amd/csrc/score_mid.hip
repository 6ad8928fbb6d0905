// score_mid: the streaming pass s_i = q . k_i / sqrt(d_h) over the mid-region
// (eq. (full_attention) restricted to M of eq. (partition)).  Every key row of a KV head is
// read once for all G query heads of its group.  Besides the scores, each workgroup writes
// the first-level histogram of its chunk (per query head, uint16 suffix counts) for the Top-K
// radix select; nothing is accumulated with atomics in global memory.
//
// Two kernels: a matrix-core one for bf16 caches and a generic fp32-arithmetic one for any
// storage type.
#include "tkphi_internal.h"

namespace tkphi {

// Chunk histogram write-out.  The row of a query head is stored as suffix sums,
// row[b] = number of the chunk's tokens in bins >= b (uint16: a chunk has < 65536 tokens), so
// that the select plan reads "tokens above bin b" with one load per chunk.  One wavefront per
// head: lane l owns bins 8l .. 8l+7.
__device__ __forceinline__ void write_suffix_hist(const uint32_t* lds_hist, uint16_t* out, int G) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  for (int gl = wv; gl < G; gl += kThreads / 64) {
    const uint32_t* hrow = lds_hist + gl * kBins + lane * 8;
    uint32_t s[8];
    uint32_t run = 0;
#pragma unroll
    for (int e = 7; e >= 0; --e) { run += hrow[e]; s[e] = run; }     // suffix sums inside the lane
    uint32_t x = run;                                                  // inclusive suffix over lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t y = __shfl_down(x, o);
      if (lane + o < 64) x += y;
    }
    const uint32_t above = x - run;                                    // tokens in the bins of higher lanes
    u32x4 v;
    v.x = (s[0] + above) | ((s[1] + above) << 16);
    v.y = (s[2] + above) | ((s[3] + above) << 16);
    v.z = (s[4] + above) | ((s[5] + above) << 16);
    v.w = (s[6] + above) | ((s[7] + above) << 16);
    *(u32x4*)(out + gl * kBins + lane * 8) = v;
  }
}

// ------------------------------------------------------------------------------------
// bf16 on the matrix cores.
//
// The contraction [tokens x d] . [d x G] has a tiny N: the G query heads are padded to the
// 16 columns of v_mfma_f32_16x16x32_bf16, whose A operand is exactly what a 16-byte row
// segment load delivers (lane (r, kg) holds 8 consecutive bf16 of token r), so the keys go
// from HBM to the MFMA without unpacking on the vector ALU.  Per wavefront and iteration:
// TPI tiles of 16 tokens -> TPI * D/32 loads of 16 B per lane, the same number of MFMAs;
// the G valid columns are transposed through a wave-private LDS strip so that score stores
// are coalesced and every lane takes part in the histogram update.
// ------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union Frag {
  u32x4 u;
  bf16x8 v;
};

// grid (n_scan_chunks, Hkv, n_problems); dynamic LDS: hist [G][kBins] + strips [4][G][TPI*16]
template <int D, int TPI>
__global__ __launch_bounds__(kThreads) void score_mid_mfma_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                  char* __restrict__ ws) {
  constexpr int KS = D / 32;            // MFMA k-steps per token tile
  constexpr int TOK = TPI * 16;         // tokens per wavefront iteration
  extern __shared__ uint32_t lds[];
  const int p = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int n_chunks = (n + g.scan_chunk - 1) / g.scan_chunk;
  // Workgroups go to the 8 XCDs round-robin by linear index.  In a ragged batch the short
  // sequences have no late chunks, so chunk indices are rotated per (head, problem): otherwise
  // the XCDs that serve the early chunks get most of the work.
  const int chunk = ((int)blockIdx.x + h + p * g.Hkv) % (int)gridDim.x;
  if (chunk >= n_chunks) return;
  const int c1 = n;                     // units of different chunks never overlap
  const int G = g.G;
  char* blk = problem_block(g, ws, p);

  uint32_t* lds_hist = lds;
  float* strips = (float*)(lds + G * kBins);
  for (int i = tid; i < G * kBins; i += kThreads) lds_hist[i] = 0u;

  const int lane = tid & 63, wv = tid >> 6;
  const int r = lane & 15, kg = lane >> 4;

  // B operand: column r = query head r of the group (zero for r >= G)
  Frag bq[KS];
#pragma unroll
  for (int j = 0; j < KS; ++j) {
    bq[j].u = (u32x4){0u, 0u, 0u, 0u};
    if (r < G) bq[j].u = *(const u32x4*)((const uint16_t*)pr.q + (size_t)(h * G + r) * D + j * 32 + kg * 8);
  }
  __syncthreads();

  const size_t row_bytes = (size_t)pr.stride_tok * 2;
  const char* Kb = (const char*)pr.K + ((size_t)h * pr.stride_head + (size_t)g.n_sink * pr.stride_tok) * 2 +
                   (size_t)kg * 16;
  float* scores = (float*)(blk + g.off_scores) + (size_t)h * G * g.mid_stride;
  float* strip = strips + (size_t)wv * G * TOK;
  const float scale = g.score_scale;

  const int n_units = g.scan_chunk / (4 * TOK);      // host guarantees scan_unit == 4 * TOK
  for (int k = 0; k < n_units; ++k) {
    const int base = chunk_unit_token(g, n_chunks, chunk, k) + wv * TOK;
    if (base >= c1) { if (g.interleave) break; else continue; }
    Frag a[TPI][KS];
#pragma unroll
    for (int t = 0; t < TPI; ++t) {
      const int row = min(base + t * 16 + r, c1 - 1);
      const char* rp = Kb + (size_t)row * row_bytes;
#pragma unroll
      for (int j = 0; j < KS; ++j) a[t][j].u = gload128(rp + j * 64);
    }
    __builtin_amdgcn_sched_barrier(0);   // all loads of the iteration are in flight before the first MFMA
    floatx4 acc[TPI];
#pragma unroll
    for (int t = 0; t < TPI; ++t) {
      acc[t] = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < KS; ++j)
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t][j].v, bq[j].v, acc[t], 0, 0, 0);
    }
    // acc[t][i] = score of token base + t*16 + 4*kg + i for query head r
    if (r < G) {
#pragma unroll
      for (int t = 0; t < TPI; ++t)
        *(floatx4*)(strip + r * TOK + t * 16 + kg * 4) = acc[t];
    }
    __builtin_amdgcn_wave_barrier();
    for (int gl = 0; gl < G; ++gl) {
#pragma unroll
      for (int tt = lane; tt < TOK; tt += 64) {
        const int tok = base + tt;
        if (tok < c1) {
          const float s = strip[gl * TOK + tt] * scale + 0.0f;   // + 0.0f: -0 -> +0, equal scores get equal keys
          scores[(size_t)gl * g.mid_stride + tok] = s;
          if (pr.scores) pr.scores[(size_t)(h * G + gl) * n + tok] = s;
          atomicAdd(&lds_hist[gl * kBins + key_bin(score_key(s))], 1u);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();
  write_suffix_hist(lds_hist, (uint16_t*)(blk + g.off_hist) + ((size_t)chunk * g.Hq + (size_t)h * G) * kBins, G);
}

// ------------------------------------------------------------------------------------
// generic (any storage type, fp32 arithmetic): grid (n_scan_chunks, Hkv, n_problems)
// A key row is split over LPR = d / (elements per 16 bytes) lanes, each lane loads 16
// bytes and forms the partial dot products for all G query heads; the partials are summed
// across the LPR lanes with butterfly shuffles.
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
  const int c0 = blockIdx.x * g.scan_chunk;           // always one contiguous range here
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

  constexpr int UNR = 8;               // row loads in flight per thread
  for (int base0 = c0; base0 < c1; base0 += RPI * UNR) {
    u32x4 v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int rr = min(base0 + u * RPI + rsub, c1 - 1);      // clamped: every lane loads
      v[u] = gload128(Kb + ((int64_t)rr * pr.stride_tok + seg * EPL) * sizeof(T));
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int row = base0 + u * RPI + rsub;
      const bool valid = row < c1;
      float x[EPL];
      Elem<T>::unpack(make_uint4(v[u].x, v[u].y, v[u].z, v[u].w), x);
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
  }
  __syncthreads();
  write_suffix_hist(lds_hist, (uint16_t*)(blk + g.off_hist) + ((size_t)blockIdx.x * g.Hq + (size_t)h * G) * kBins, G);
}

void launch_score_mid(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  if (g.max_mid == 0) return;
  dim3 grid(g.n_scan_chunks, g.Hkv, g.n_problems);
  const size_t hist_lds = (size_t)g.G * kBins * sizeof(uint32_t);
  if (g.use_mfma) {
    if (g.d == 128)
      TKPHI_LAUNCH(ST_SCORE, (score_mid_mfma_kernel<128, 4>), grid, dim3(kThreads), hist_lds + (size_t)4 * g.G * 64 * 4, s,
                         g, probs, ws);
    else
      TKPHI_LAUNCH(ST_SCORE, (score_mid_mfma_kernel<64, 8>), grid, dim3(kThreads), hist_lds + (size_t)4 * g.G * 128 * 4, s,
                         g, probs, ws);
  } else if (g.dtype == TKPHI_BF16) {
    TKPHI_LAUNCH(ST_SCORE, score_mid_kernel<uint16_t>, grid, dim3(kThreads), hist_lds, s, g, probs, ws);
  } else {
    TKPHI_LAUNCH(ST_SCORE, score_mid_kernel<float>, grid, dim3(kThreads), hist_lds, s, g, probs, ws);
  }
}

}  // namespace tkphi
