// Matrix-core score tiles shared by the filtered score pass and the select kernel's rescan:
// s_i = q . k_i / sqrt(d_h) (eq. (full_attention)) for the mid-region rows of one wavefront's share
// of a score chunk, with the candidates of the Top-K selection appended to per-wavefront lists.
#pragma once

#include "tkphi_internal.h"

namespace tkphi {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 st_bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float st_floatx4;
union ScoreFrag {
  u32x4 u;
  st_bf16x8 v;
};

// B operand of the score MFMA: column r = query head h G + r of the group (zero for r >= G);
// lane (r, kg) holds channels j 32 + kg 8 .. + 8 of k-step j.
template <int D>
__device__ __forceinline__ void load_query_frags(const Geom& g, const tkphi_problem& pr, int h, ScoreFrag (&bq)[D / 32]) {
  const int lane = threadIdx.x & 63, r = lane & 15, kg = lane >> 4;
#pragma unroll
  for (int j = 0; j < D / 32; ++j) {
    bq[j].u = (u32x4){0u, 0u, 0u, 0u};
    if (r < g.G) bq[j].u = *(const u32x4*)((const uint16_t*)pr.q + (size_t)(h * g.G + r) * D + j * 32 + kg * 8);
  }
}

// Candidate lists of the filtered selection.  A score chunk is scanned by four wavefront slots; slot
// `wslot` of chunk `chunk` appends, per query head, every token whose order-preserving score key is
// >= that head's lower bound to its own list (capacity: the slot's tokens, scan_chunk / 4), in the
// fixed order it visits them, and finally stores the list length.  No atomics: a list has one writer.
// Entry i of a list lives in a compact array (i < cand_T: what the select kernel reads in one sweep)
// or at position i of the list's full-capacity region.
__device__ __forceinline__ size_t cand_region(const Geom& g, int gq, int chunk, int wslot) {
  return (((size_t)gq * g.n_scan_chunks + chunk) * 4 + wslot) * (size_t)(g.scan_chunk / 4);
}

// One wavefront: slot `wslot` of chunk `chunk` of KV head h (n mid tokens, n_chunks chunks).
//   edge_r   lower bound of the score key for the query head of this lane's column r (ignored for r >= G)
//   only_gl  -1: every head of the group; else only head h G + only_gl is written
//   strip    null, or this wavefront's LDS strip of G x cand_T entries: the compact heads of the G lists are
//            collected there and go to memory at the end as whole lines (a head is cand_T contiguous entries, the
//            four slots of a chunk adjoin), instead of one 8-byte store per candidate scattered through the scan:
//            fewer partly written lines for the L2 to write back in the middle of the read stream
//   rescan   write the rescan set of lists, compact heads and counts (the select kernel's second attempt reads
//            only that set, so what a first attempt reads is never overwritten while another workgroup reads it)
// Lane (r, kg) ends up with the scores of head r for tokens base + t 16 + 4 kg + i, so each list is
// written by the four lanes of its column, in the order (unit, t, i, kg).
// SUB: 16-token tiles whose loads are in flight together (the rescan keeps registers low); STREAM: non-temporal key loads
template <int D, int TPI, int SUB = TPI, bool STREAM = false>
__device__ __forceinline__ void scan_wave_slot(const Geom& g, const tkphi_problem& pr, char* blk, int h, int n, int n_chunks,
                                               int chunk, int wslot, const ScoreFrag (&bq)[D / 32], uint32_t edge_r,
                                               int only_gl, bool rescan = false, uint2* strip = nullptr) {
  constexpr int KS = D / 32;
  constexpr int TOK = TPI * 16;         // tokens per wavefront and unit
  const int lane = threadIdx.x & 63, r = lane & 15, kg = lane >> 4;
  const int G = g.G;
  const bool col_live = r < G && (only_gl < 0 || r == only_gl);
  const int gq = h * G + min(r, G - 1);
  uint2* list = (uint2*)(blk + (rescan ? g.off_resf : g.off_candf)) + cand_region(g, gq, chunk, wslot);
  uint2* head = (uint2*)(blk + (rescan ? g.off_resc : g.off_candc)) + (((size_t)gq * g.n_scan_chunks + chunk) * 4 + wslot) * (size_t)g.cand_T;
  const int cap = g.scan_chunk / 4, T = g.cand_T;
  const uint64_t col_lanes = 0x0001000100010001ull << r;     // the four lanes of this column
  const uint64_t lanes_below = (1ull << lane) - 1ull;
  const size_t row_bytes = (size_t)pr.stride_tok * 2;
  const char* Kb = (const char*)pr.K + ((size_t)h * pr.stride_head + (size_t)g.n_sink * pr.stride_tok) * 2 + (size_t)kg * 16;
  const float scale = g.score_scale;
  float* export_row = pr.scores ? pr.scores + (size_t)gq * n : nullptr;
  int cnt = 0;                          // length of this column's list (the same in its four lanes)

  const int n_units = g.scan_chunk / (4 * TOK);
  for (int k = 0; k < n_units; ++k) {
    const int base = chunk_unit_token(g, n_chunks, chunk, k) + wslot * TOK;
    if (base >= n) { if (g.interleave) break; else continue; }
#pragma unroll
    for (int t0 = 0; t0 < TPI; t0 += SUB) {
      ScoreFrag a[SUB][KS];
#pragma unroll
      for (int t = 0; t < SUB; ++t) {
        const int row = min(base + (t0 + t) * 16 + r, n - 1);
        const char* rp = Kb + (size_t)row * row_bytes;
#pragma unroll
        for (int j = 0; j < KS; ++j) a[t][j].u = STREAM ? gload128_stream(rp + j * 64) : gload128(rp + j * 64);
      }
      __builtin_amdgcn_sched_barrier(0);   // all loads of the group are in flight before the first MFMA
      st_floatx4 acc[SUB];
#pragma unroll
      for (int t = 0; t < SUB; ++t) {
        acc[t] = (st_floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KS; ++j) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t][j].v, bq[j].v, acc[t], 0, 0, 0);
      }
#pragma unroll
      for (int t = 0; t < SUB; ++t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = base + (t0 + t) * 16 + 4 * kg + i;
          const float s = acc[t][i] * scale + 0.0f;            // + 0.0f: -0 -> +0, equal scores get equal keys
          const bool live = col_live && tok < n;
          if (export_row && live) export_row[tok] = s;
          const bool pass = live && score_key(s) >= edge_r;
          const uint64_t mask = __ballot(pass);
          if (mask) {
            const uint64_t mine = mask & col_lanes;
            const int at = cnt + __popcll(mine & lanes_below);
            if (pass) {
              const uint2 e = make_uint2(__float_as_uint(s), (uint32_t)tok);
              if (at < T) { if (strip) strip[min(r, G - 1) * T + at] = e; else head[at] = e; }
              else if (at < cap) list[at] = e;
            }
            cnt += __popcll(mine);
          }
        }
      }
    }
  }
  if (strip) {                          // (LDS operations of one wavefront execute in order: no barrier)
    for (int gl = 0; gl < G; ++gl) {
      const int c = min(__shfl(cnt, gl), T);          // lane gl is lane (r = gl, kg = 0) of column gl
      uint2* hd = (uint2*)(blk + (rescan ? g.off_resc : g.off_candc)) + (((size_t)(h * G + gl) * g.n_scan_chunks + chunk) * 4 + wslot) * (size_t)T;
      for (int i = lane; i < c; i += 64) hd[i] = strip[gl * T + i];
    }
  }
  if (col_live && kg == 0)
    ((uint32_t*)(blk + (rescan ? g.off_rescount : g.off_ccount)))[((size_t)gq * g.n_scan_chunks + chunk) * 4 + wslot] = (uint32_t)min(cnt, cap);
}

// Smallest score key whose first-level bin is >= t (key_bin is monotone in the key), so that
// "bin(key) >= t" is the single comparison "key >= bin_lower_key(t)".  t <= 0: every key; t >= kBins: none.
__device__ __forceinline__ uint32_t bin_lower_key(int t) {
  auto mag_edge = [](int mb) { return ((uint32_t)(kExpLo + mb / 16) << 23) | ((uint32_t)(mb % 16) << 19); };
  if (t <= 0) return 0u;
  if (t >= kBins) return 0xffffffffu;
  if (t >= kMagBins) { const int mb = t - kMagBins; return 0x80000000u | (mb == 0 ? 0u : mag_edge(mb)); }
  const int M = kMagBins - 1 - t;       // negative scores: magnitude bins 0 .. M qualify
  return 0x7fffffffu - (mag_edge(M + 1) - 1u);
}

}  // namespace tkphi
