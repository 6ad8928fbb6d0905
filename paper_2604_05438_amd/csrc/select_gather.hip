// Fused Top-K select + gather of the filtered pipeline (bf16 caches on the matrix cores):
// topk_select, exact_branch and residual_correct for the retrieved tokens in one launch.
// grid (split, Hq, n_problems), NTHR = 1024 or 512 threads: `split` workgroups share a query head.
//
// The score pass left, per query head, every token whose score key reaches the head's lower bound, in
// per-wavefront lists (score_tile.h): the first cand_T entries of a list in a compact array, the rest in
// the list's full-capacity region.  If at least K candidates exist, the K best mid tokens
// (Sec. "Models, tasks, and protocol": exhaustive Top-K, ties to the lower index) are all among them.
//
// Every workgroup of a head first finds the same selection threshold, on its own (the candidates of a
// head are ~100 KB and the search is a few thousand instructions: cheaper than a launch boundary):
//   * the candidates are visited in "sweeps" in which a thread owns kSweepEntries consecutive entries of
//     one list; the first sweep's addresses depend on the launch geometry only and are loaded together
//     with the problem record, so the common case is one memory round trip
//   * histogram of a fine monotone binning of the score keys -> boundary bin b* (tokens in higher bins
//     are retrieved); the candidates in b* are ranked by counting (or, beyond kBCap of them, by radix
//     passes over the sweeps) -> the K-th best composite (score key, lower index first), `thr`
//   * fewer than K candidates (the sampled bound was too high: a ~1e-5 event per head by design, and what
//     tkphi_tuning::select_test = 1 forces): the workgroup first rescans its head's keys with no bound,
//     which makes every mid token a candidate
// Then workgroup `part` takes the lists [part, part + 1) n_lists / split: their winners (composite >=
// thr), in list order, are written to the head's retrieved list at the offset given by the winners in
// earlier lists, and gathered 256 or 512 at a time (16-token tiles, one or two per wavefront):
//     m_loc = max s_i,  Z_loc = sum exp(s_i - m_loc),  nu_loc = sum exp(s_i - m_loc) v_i     (eq. (exact_terms))
//     zsum = sum z_i,  zv = sum z_i v_i,  z_i = phi_q . phi_k(k_i) recomputed                (eq. (subtraction))
// into one partial per workgroup, [m, Z, zsum, count, nu[d], zv[d]], which the merge kernel combines in
// part order.  No atomics on global memory; every sum runs in a fixed order.
#include "gather_tile.h"
#include "merge_head.h"
#include "score_tile.h"
#include "select_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

constexpr int kBCap = 1024;            // boundary-bin candidates ranked in LDS
constexpr int kSweepEntries = 12;      // entries per thread and sweep (Geom::cand_T is a multiple)
constexpr int kSweepLoads = kSweepEntries / 2;
// winners gathered per round: 16-token tile t of a round goes to wavefront t mod 16.  Two tiles per wavefront at
// d = 64 (one round for most heads of a batch of short sequences); at d = 128 the second tile's rows do not fit
// the registers
template <int D, int NTHR> constexpr int kBatchOf = (D == 64 && NTHR == 1024) ? 512 : 256;
// candidates of a head that the select phase packs into LDS
template <int NTHR> constexpr int kDenseOf = NTHR == 1024 ? 8192 : 4096;
// winners of a workgroup kept in LDS (the rest are re-read from the retrieved list)
template <int NTHR> constexpr int kWinLdsOf = NTHR == 1024 ? 1536 : 1024;

// every mid token of query head gq becomes a candidate: the head's lists are written again with no bound, into
// the rescan set (what the score pass wrote stays as it is: other workgroups of the head may still be reading it)
// (one 16-token tile in flight per wavefront: the rare path must not cost the common one registers)
template <int D, int TPI, int NTHR>
__device__ __forceinline__ void rescan_head(const Geom& g, const tkphi_problem& pr, char* blk, int gq, int n, int n_chunks) {
  const int h = gq / g.G, wv = threadIdx.x >> 6;
  ScoreFrag bq[D / 32];
  load_query_frags<D>(g, pr, h, bq);
  for (int reg = wv; reg < n_chunks * 4; reg += NTHR / 64)
    scan_wave_slot<D, TPI, 1>(g, pr, blk, h, n, n_chunks, reg >> 2, reg & 3, bq, 0u, gq % g.G, true);
}

// The selecting and gathering work of workgroup (part, gq, p); returns early where there is nothing to retrieve
template <int D, int TPI, int NTHR>
__device__ __forceinline__ void select_gather_body(const Geom& g, const tkphi_problem* __restrict__ probs, char* __restrict__ ws,
                                                   int part, int gq, int p) {
  constexpr int KS = D / 32;
  constexpr int WROW = wk_row_bytes(D);
  // select phase: histogram (8 KB) + boundary candidates (8 KB); gather phase: reduction scratch of the value sums
  __shared__ __attribute__((aligned(16))) char lds_a[16384];
  __shared__ __attribute__((aligned(16))) char wk_lds[D * WROW];
  constexpr int kDense = kDenseOf<NTHR>, kWinLds = kWinLdsOf<NTHR>, NWV = NTHR / 64;
  __shared__ uint2 dense[kDense];                   // the candidates of the head, packed (select phase)
  __shared__ int w_tok[kWinLds];
  __shared__ float w_s[kWinLds];
  constexpr int kBatch = kBatchOf<D, NTHR>;
  __shared__ float b_w[kBatch], b_z[kBatch];
  __shared__ float sh_bk[D], sh_pq[D];              // bk[h] and phi_q of the head, staged with Wk
  __shared__ int sh_scan[NWV];
  __shared__ uint64_t sh_prefix, sh_thr;
  __shared__ int sh_want, sh_tot, sh_r0, sh_r1;
  __shared__ int sh_bstar, sh_krem, sh_chi, sh_nb, sh_nbc;
  __shared__ uint32_t sh_total, sh_ovp;
  __shared__ float sh_m, sh_Z, sh_zs;
  uint32_t* sh_hist = (uint32_t*)lds_a;
  uint64_t* bcand = (uint64_t*)(lds_a + 8192);
  float* red = (float*)lds_a;                       // [16 wavefronts][2][128]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  TKPHI_PHASE(ws, 10);
  char* blk = problem_block(g, ws, p);
  const int T = g.cand_T;
  const int n_reg_max = g.n_scan_chunks * 4;
  const uint32_t cap_w = (uint32_t)(g.scan_chunk / 4);
  // (after a rescan these three point at the rescan set)
  const uint32_t* ccount = (const uint32_t*)(blk + g.off_ccount) + (size_t)gq * n_reg_max;
  const uint2* compact = (const uint2*)(blk + g.off_candc) + (size_t)gq * n_reg_max * T;
  const uint2* sparse = (const uint2*)(blk + g.off_candf) + (size_t)gq * n_reg_max * cap_w;

  // ---- first sweep, speculatively: addresses depend on the launch geometry only --------------------------
  u32x4 e0[kSweepLoads];
  uint32_t c0 = 0;
  const uint32_t edge0 = ((const uint32_t*)(blk + g.off_thr))[gq];   // the bound the score pass pruned this head with
  {
    const int s = kSweepEntries * tid, list = s / T;
    if (list < n_reg_max) {
      c0 = ccount[list];
#pragma unroll
      for (int u = 0; u < kSweepLoads; ++u) e0[u] = gload128(compact + s + 2 * u);
    }
  }
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int Ksel = max(0, min(min(pr.topk, n), g.max_K));
  SelPlan* plan = (SelPlan*)(blk + g.off_plan) + gq;
  if (Ksel == 0) {
    if (tid == 0 && part == 0) *plan = SelPlan{-1, 0, 0, 0, 0};
    return;
  }
  const int h = gq / g.G;
  const int n_chunks = (n + g.scan_chunk - 1) / g.scan_chunk;
  const int n_reg = n_chunks * 4;
  const int rounds = (n_reg * T + NTHR * kSweepEntries - 1) / (NTHR * kSweepEntries);
  int32_t* sel_idx = (int32_t*)(blk + g.off_selidx) + (size_t)gq * g.max_K;
  float* sel_score = (float*)(blk + g.off_selscore) + (size_t)gq * g.max_K;

  // entries [0, nvalid) at src are the share of thread t in sweep sw; they belong to list `list`
  struct Share { const uint2* src; int nvalid; int list; };
  int max_passes = 0;                               // overflow sweeps per round (set below)
  auto share_of = [&](int sw, int t, int known = -1) -> Share {   // known: the list's length if the caller has it
    const int r = sw < rounds ? sw : (sw - rounds) / max_passes;
    const int s = kSweepEntries * (t + NTHR * r), list = s / T, pos = s % T;
    if (list >= n_reg) return Share{compact, 0, list};
    const int c = (int)min(known >= 0 ? (uint32_t)known : ccount[list], cap_w);
    if (sw < rounds) return Share{compact + s, max(0, min(min(c, T) - pos, kSweepEntries)), list};
    const int k = (sw - rounds) % max_passes;
    const int start = T + (k * (T / kSweepEntries) + pos / kSweepEntries) * kSweepEntries;
    return Share{sparse + (size_t)list * cap_w + start, max(0, min(c - start, kSweepEntries)), list};
  };
  auto load_share = [&](const Share& sh, u32x4 (&e)[kSweepLoads]) {
#pragma unroll
    for (int u = 0; u < kSweepLoads; ++u)
      if (2 * u < sh.nvalid) e[u] = gload128(sh.src + 2 * u);
  };
  auto entry = [](const u32x4 (&e)[kSweepLoads], int i) { return (i & 1) ? make_uint2(e[i >> 1].z, e[i >> 1].w) : make_uint2(e[i >> 1].x, e[i >> 1].y); };

  // ---- candidate count, overflow depth (and, on a threshold miss, the rescan) ---------------------------
  bool have_e0 = true;
  int n_sweeps = 0;
  for (int attempt = 0;; ++attempt) {
    if (tid == 0) { sh_total = 0u; sh_ovp = 0u; }
    __syncthreads();
    uint32_t tot = 0, ovp = 0;
    for (int r = 0; r < rounds; ++r) {
      const int s = kSweepEntries * (tid + NTHR * r), list = s / T;
      if (s % T == 0 && list < n_reg) {               // the thread that owns the head of a list counts it
        const uint32_t c = min((r == 0 && have_e0) ? c0 : ccount[list], cap_w);
        tot += c;
        if (c > (uint32_t)T) ovp = max(ovp, (c - T + T - 1) / T);
      }
    }
    if (tot) atomicAdd(&sh_total, tot);
    if (ovp) atomicMax(&sh_ovp, ovp);
    __syncthreads();
    max_passes = (int)sh_ovp;
    n_sweeps = rounds + rounds * max_passes;
    if (sh_total >= (uint32_t)Ksel || attempt > 0) break;
    __syncthreads();
    // (every workgroup of the head takes this branch, the counts it depends on being the score pass's, and writes
    // the same values to the rescan set: no ordering between them is needed)
    rescan_head<D, TPI, NTHR>(g, pr, blk, gq, n, n_chunks);
    ccount = (const uint32_t*)(blk + g.off_rescount) + (size_t)gq * n_reg_max;
    compact = (const uint2*)(blk + g.off_resc) + (size_t)gq * n_reg_max * T;
    sparse = (const uint2*)(blk + g.off_resf) + (size_t)gq * n_reg_max * cap_w;
    have_e0 = false;
    __syncthreads();
  }
  const uint32_t total = sh_total;
  TKPHI_PHASE(ws, 11);
  float* partial = (float*)(blk + g.off_part) + ((size_t)gq * (g.n_tiles + g.n_atiles) + part) * g.part_stride;
  auto empty_partial = [&]() {
    if (tid == 0) { store_agent(partial, -INFINITY); store_agent(partial + 1, 0.f); store_agent(partial + 2, 0.f); store_agent(partial + 3, 0.f); }
    if (tid < D) { store_agent(partial + 4 + tid, 0.f); store_agent(partial + 4 + D + tid, 0.f); }
  };
  if (total < (uint32_t)Ksel) {                     // cannot happen after a rescan (every mid token is a candidate)
    if (tid == 0 && part == 0) *plan = SelPlan{-1, 0, 0, 0, 0};
    empty_partial();
    return;
  }
  // Wk[h] for the gather phase: requested now (the first sweep has arrived, nothing else is in flight), stored
  // to LDS right before the gather (the barrier after the histogram pass orders LDS only, so it does not wait
  // for these loads)
  WkPieces<D, NTHR> wkp;
  wkp.request(pr.Wk, h);
  float bk_t = 0.f, pq_t = 0.f;
  if (tid < D) { bk_t = pr.bk[(size_t)h * D + tid]; pq_t = ((const float*)(blk + g.off_phiq))[(size_t)gq * D + tid]; }

  // (have_e0 is false exactly after a rescan: those lists were written without a bound)
  const SelBins bin_of{edge0, have_e0 && edge0 != 0u && edge0 != 0xffffffffu};
  // This workgroup's share of the gather: the winners of lists [l0, l1), in list order
  const int split = g.sg_split;
  const int per_part = (n_reg + split - 1) / split;
  const int l0 = part * per_part, l1 = min(n_reg, l0 + per_part);
  int my_base = 0, my_count = 0;                    // winners in earlier lists; winners of this workgroup
  // Common case: one sweep holds every candidate and there are at most kDense of them (about 2.5 K per head at a
  // 1 % budget, against 12 K list slots).  They are first packed, in list order, into an LDS array (64 KB that
  // is otherwise unused: a workgroup of 1024 threads has a CU to itself); histogram, threshold and winners then
  // walk 3-4 entries per thread instead of 12 slots.
  if (n_sweeps == 1 && have_e0 && total <= (uint32_t)kDense) {
    const int n_cand = (int)total;
    const Share sh0 = share_of(0, tid, (int)min(c0, cap_w));
    const int nv = sh0.nvalid;
    for (int i = tid; i < kFineBins; i += NTHR) sh_hist[i] = 0u;
    if (tid == 0) {
      sh_bstar = -1; sh_krem = 0; sh_chi = 0; sh_nb = 0; sh_nbc = 0; sh_thr = 0ull;
      sh_r0 = l0 < n_reg ? 0 : n_cand; sh_r1 = n_cand;
    }
    const int off = sel_scan_incl(nv, sh_scan) - nv;       // (its barriers also publish the initial values above)
#pragma unroll
    for (int i = 0; i < kSweepEntries; ++i)
      if (i < nv) dense[off + i] = entry(e0, i);
    {
      const int s0 = kSweepEntries * tid, list = s0 / T;
      if (s0 % T == 0 && list < n_reg) {               // first slot of a list: where the list starts in the packed array
        if (list == l0) sh_r0 = off;
        if (list == l1) sh_r1 = off;
      }
    }
    lds_barrier();
    const int r0 = sh_r0, r1 = sh_r1;
    // ---- histogram -> boundary bin ----------------------------------------------------------------------------
    for (int idx = tid; idx < n_cand; idx += NTHR) atomicAdd(&sh_hist[bin_of(score_key(__uint_as_float(dense[idx].x)))], 1u);
    lds_barrier();
    TKPHI_PHASE(ws, 12);
    {
      // thread t takes the BPT bins below kFineBins - BPT t, highest first: a prefix sum over the threads is a
      // suffix sum over the bins
      constexpr int BPT = kFineBins / NTHR;
      int cb[BPT], own = 0;
#pragma unroll
      for (int e = 0; e < BPT; ++e) { cb[e] = (int)sh_hist[kFineBins - 1 - BPT * tid - e]; own += cb[e]; }
      int gt = sel_scan_incl(own, sh_scan) - own;          // candidates in bins above this thread's
#pragma unroll
      for (int e = 0; e < BPT; ++e) {
        if (gt + cb[e] >= Ksel && gt < Ksel) { sh_bstar = kFineBins - 1 - BPT * tid - e; sh_krem = Ksel - gt; sh_chi = gt; sh_nb = cb[e]; }
        gt += cb[e];
      }
      lds_barrier();
    }
    const int bstar = sh_bstar, krem = sh_krem, c_hi = sh_chi, nb = sh_nb;
    if (bstar < 0) {                                  // cannot happen: total >= Ksel
      if (tid == 0 && part == 0) *plan = SelPlan{-1, 0, 0, 0, 0};
      empty_partial();
      return;
    }
    TKPHI_PHASE(ws, 13);
    // ---- thr: the K_rem-th best composite of the boundary bin -------------------------------------------------
    if (nb <= kBCap) {
      for (int idx = tid; idx < n_cand; idx += NTHR) {
        const uint2 en = dense[idx];
        const uint32_t key = score_key(__uint_as_float(en.x));
        if (bin_of(key) == bstar) {
          const int at = atomicAdd(&sh_nbc, 1);
          if (at < kBCap) bcand[at] = composite(key, en.y);
        }
      }
      lds_barrier();
      const int sub = tid & 7, slot = tid >> 3;
      for (int k0 = 0; k0 < nb; k0 += NTHR / 8) {
        const int j = k0 + slot;
        const bool valid = j < nb;
        const uint64_t mine = valid ? bcand[j] : ~0ull;
        int rank = 0;
        for (int i = sub; i < nb; i += 8) rank += bcand[i] > mine ? 1 : 0;
        rank += __shfl_xor(rank, 1);
        rank += __shfl_xor(rank, 2);
        rank += __shfl_xor(rank, 4);
        if (valid && sub == 0 && rank == krem - 1) sh_thr = mine;
      }
      lds_barrier();
    } else {                                          // (e.g. all scores equal) radix passes over the packed array
      auto get = [&](int j, uint64_t* v) {
        const uint2 en = dense[j];
        const uint32_t key = score_key(__uint_as_float(en.x));
        *v = composite(key, en.y);
        return bin_of(key) == bstar;
      };
      const uint64_t t = radix_select_desc(n_cand, krem, get, sh_hist, sh_scan, &sh_prefix, &sh_want);
      if (tid == 0) sh_thr = t;
      __syncthreads();
    }
    const uint64_t thr = sh_thr;
    TKPHI_PHASE(ws, 14);
    if (tid == 0 && part == 0) *plan = SelPlan{bstar, krem, c_hi, nb, Ksel};
    // ---- winners of the packed range [r0, r1) --------------------------------------------------------------------
    auto is_winner = [&](int idx, int lim, uint2* en) {
      if (idx >= lim) return false;
      *en = dense[idx];
      return composite(score_key(__uint_as_float(en->x)), en->y) >= thr;
    };
    {
      // thread t owns the `per` consecutive entries from r0 + t per: one prefix sum over the threads keeps list order
      const int per = (r1 - r0 + NTHR - 1) / NTHR, first = r0 + tid * per;
      int mine = 0;
      for (int e = 0; e < per; ++e) { uint2 en; mine += is_winner(first + e, r1, &en) ? 1 : 0; }
      const int incl = sel_scan_incl(mine, sh_scan);
      if (tid == NTHR - 1) sh_tot = incl;
      int at = incl - mine;
      for (int e = 0; e < per; ++e) {
        uint2 en;
        if (is_winner(first + e, r1, &en)) {
          if (at < kWinLds) { w_tok[at] = (int)en.y; w_s[at] = __uint_as_float(en.x); }
          ++at;
        }
      }
      lds_barrier();
      my_count = sh_tot;
    }
    // the retrieved list of the head, for the export of the merge and for winners beyond the LDS stage
    if (my_count > kWinLds || pr.topk_idx) {
      int before = 0;
      for (int idx = tid; idx < r0; idx += NTHR) { uint2 en; before += is_winner(idx, r0, &en) ? 1 : 0; }
      const int incl_b = sel_scan_incl(before, sh_scan);
      if (tid == NTHR - 1) sh_tot = incl_b;
      lds_barrier();
      my_base = sh_tot;
      lds_barrier();
      int seen = 0;
      for (int base = r0; base < r1; base += NTHR) {
        uint2 en = make_uint2(0u, 0u);
        const int flag = is_winner(base + tid, r1, &en) ? 1 : 0;
        const int incl = sel_scan_incl(flag, sh_scan);
        if (tid == NTHR - 1) sh_tot = incl;
        const int at = my_base + seen + incl - flag;
        if (flag && at < min(Ksel, g.max_K)) { sel_idx[at] = (int32_t)en.y; sel_score[at] = __uint_as_float(en.x); }
        __syncthreads();
        seen += sh_tot;
        __syncthreads();
      }
    }
  } else {
    // (the general path: several sweeps, more candidates than the packed array holds, or the lists of a rescan;
    // every phase reads its entries from the lists again)
    // ---- pass A: histogram of the candidates' fine bins ----------------------------------------------------------
    for (int i = tid; i < kFineBins; i += NTHR) sh_hist[i] = 0u;
    if (tid == 0) { sh_bstar = -1; sh_krem = 0; sh_chi = 0; sh_nb = 0; sh_nbc = 0; sh_thr = 0ull; }
    __syncthreads();
    for (int sw = 0; sw < n_sweeps; ++sw) {
      const Share sh = share_of(sw, tid);
      u32x4 e[kSweepLoads];
      load_share(sh, e);
#pragma unroll
      for (int i = 0; i < kSweepEntries; ++i)
        if (i < sh.nvalid) atomicAdd(&sh_hist[bin_of(score_key(__uint_as_float(entry(e, i).x)))], 1u);
    }
    lds_barrier();                                    // (the histogram is LDS traffic; the Wk loads stay in flight)
    TKPHI_PHASE(ws, 12);
    {
      // thread t takes the BPT bins below kFineBins - BPT t, highest first: a prefix sum over the threads is a
      // suffix sum over the bins
      constexpr int BPT = kFineBins / NTHR;
      int cb[BPT], own = 0;
#pragma unroll
      for (int e = 0; e < BPT; ++e) { cb[e] = (int)sh_hist[kFineBins - 1 - BPT * tid - e]; own += cb[e]; }
      int gt = sel_scan_incl(own, sh_scan) - own;          // candidates in bins above this thread's
#pragma unroll
      for (int e = 0; e < BPT; ++e) {
        if (gt + cb[e] >= Ksel && gt < Ksel) { sh_bstar = kFineBins - 1 - BPT * tid - e; sh_krem = Ksel - gt; sh_chi = gt; sh_nb = cb[e]; }
        gt += cb[e];
      }
      lds_barrier();
    }
    const int bstar = sh_bstar, krem = sh_krem, c_hi = sh_chi, nb = sh_nb;
    if (bstar < 0) {                                  // cannot happen: total >= Ksel
      if (tid == 0 && part == 0) *plan = SelPlan{-1, 0, 0, 0, 0};
      empty_partial();
      return;
    }
    TKPHI_PHASE(ws, 13);

    // ---- thr: the K_rem-th best composite of the boundary bin ------------------------------------------------
    if (nb <= kBCap) {
      // stage the boundary candidates (any order: ranks do not depend on it), then rank by counting the larger
      // composites, 8 lanes per candidate; the candidate of rank K_rem - 1 is the threshold
      for (int sw = 0; sw < n_sweeps; ++sw) {
        const Share sh = share_of(sw, tid);
        u32x4 e[kSweepLoads];
        load_share(sh, e);
#pragma unroll
        for (int i = 0; i < kSweepEntries; ++i) {
          if (i < sh.nvalid) {
            const uint2 en = entry(e, i);
            const uint32_t key = score_key(__uint_as_float(en.x));
            if (bin_of(key) == bstar) {
              const int at = atomicAdd(&sh_nbc, 1);
              if (at < kBCap) bcand[at] = composite(key, en.y);
            }
          }
        }
      }
      lds_barrier();
      const int sub = tid & 7, slot = tid >> 3;
      for (int k0 = 0; k0 < nb; k0 += NTHR / 8) {
        const int j = k0 + slot;
        const bool valid = j < nb;
        const uint64_t mine = valid ? bcand[j] : ~0ull;
        int rank = 0;
        int i = sub;
        for (; i + 24 < nb; i += 32) {
          const uint64_t x0 = bcand[i], x1 = bcand[i + 8], x2 = bcand[i + 16], x3 = bcand[i + 24];
          rank += (x0 > mine ? 1 : 0) + (x1 > mine ? 1 : 0) + (x2 > mine ? 1 : 0) + (x3 > mine ? 1 : 0);
        }
        for (; i < nb; i += 8) rank += bcand[i] > mine ? 1 : 0;
        rank += __shfl_xor(rank, 1);
        rank += __shfl_xor(rank, 2);
        rank += __shfl_xor(rank, 4);
        if (valid && sub == 0 && rank == krem - 1) sh_thr = mine;
      }
      lds_barrier();
    } else {
      // the slot (sweep, thread, entry) as one index for the radix passes (e.g. all scores equal)
      auto get = [&](int j, uint64_t* v) {
        const int sw = j / (NTHR * kSweepEntries), rem = j % (NTHR * kSweepEntries);
        const Share sh = share_of(sw, rem / kSweepEntries);
        const int i = rem % kSweepEntries;
        if (i >= sh.nvalid) return false;
        const uint2 e = sh.src[i];
        const uint32_t key = score_key(__uint_as_float(e.x));
        *v = composite(key, e.y);
        return bin_of(key) == bstar;
      };
      const uint64_t t = radix_select_desc(n_sweeps * NTHR * kSweepEntries, krem, get, sh_hist, sh_scan, &sh_prefix, &sh_want);
      if (tid == 0) sh_thr = t;
      __syncthreads();
    }
    const uint64_t thr = sh_thr;
    TKPHI_PHASE(ws, 14);
    if (tid == 0 && part == 0) *plan = SelPlan{bstar, krem, c_hi, nb, Ksel};

    // ---- this workgroup's winners: lists [l0, l1), in list order -----------------------------------------------
    for (int sw = 0; sw < n_sweeps; ++sw) {
      const Share sh = share_of(sw, tid);
      u32x4 e[kSweepLoads];
      load_share(sh, e);
      uint32_t fw = 0;                                // bit i: entry i is retrieved
#pragma unroll
      for (int i = 0; i < kSweepEntries; ++i) {
        if (i < sh.nvalid) {
          const uint2 en = entry(e, i);
          if (composite(score_key(__uint_as_float(en.x)), en.y) >= thr) fw |= 1u << i;
        }
      }
      const int nw = __popc(fw);
      const bool mine = sh.list >= l0 && sh.list < l1;
      // (winners of one sweep: <= 12288 mine, <= 12288 before: 16 bits each)
      const int packed = (mine ? nw : 0) | ((sh.list < l0 ? nw : 0) << 16);
      const int incl = sel_scan_incl(packed, sh_scan);
      if (tid == NTHR - 1) sh_tot = incl;
      int at = my_count + ((incl - packed) & 0xffff);   // rank among this workgroup's winners
      lds_barrier();
      const int tot = sh_tot;
      if (mine) {
#pragma unroll
        for (int i = 0; i < kSweepEntries; ++i) {
          if (fw & (1u << i)) {
            const uint2 en = entry(e, i);
            if (at < kWinLds) { w_tok[at] = (int)en.y; w_s[at] = __uint_as_float(en.x); }
            // (global position: filled in below, once the winners of earlier lists in later sweeps are known)
            ++at;
          }
        }
      }
      my_count += tot & 0xffff;
      my_base += tot >> 16;
      lds_barrier();
    }
    // the retrieved list of the head, for the exports of the merge kernel and for winners beyond the LDS stage:
    // a second pass writes this workgroup's winners at my_base + rank (list positions never leave [0, Ksel))
    {
      int seen = 0;
      const bool need_global = my_count > kWinLds;
      for (int sw = 0; sw < n_sweeps; ++sw) {
        const Share sh = share_of(sw, tid);
        const bool mine = sh.list >= l0 && sh.list < l1;
        if (n_sweeps == 1 && !need_global && !pr.topk_idx) break;     // (nothing reads the list)
        u32x4 e[kSweepLoads];
        load_share(sh, e);
        uint32_t fw = 0;
#pragma unroll
        for (int i = 0; i < kSweepEntries; ++i) {
          if (mine && i < sh.nvalid) {
            const uint2 en = entry(e, i);
            if (composite(score_key(__uint_as_float(en.x)), en.y) >= thr) fw |= 1u << i;
          }
        }
        const int nw = __popc(fw);
        const int incl = sel_scan_incl(nw, sh_scan);
        if (tid == NTHR - 1) sh_tot = incl;
        int at = my_base + seen + incl - nw;
#pragma unroll
        for (int i = 0; i < kSweepEntries; ++i) {
          if (fw & (1u << i)) {
            const uint2 en = entry(e, i);
            if (at < min(Ksel, g.max_K)) { sel_idx[at] = (int32_t)en.y; sel_score[at] = __uint_as_float(en.x); }
            ++at;
          }
        }
        __syncthreads();
        seen += sh_tot;
        __syncthreads();
      }
    }
  }
  TKPHI_PHASE(ws, 15);

  // ---- gather: kBatch winners per round, one or two 16-token tiles per wavefront -----------------------------
  const int r = lane & 15, kg = lane >> 4;
  const int64_t head_off = (int64_t)h * pr.stride_head;
  constexpr int LPR = D / 8;                        // lanes per value row (16 bytes each)
  constexpr int RPP = NTHR / LPR;            // rows per pass (64 or 128)
  constexpr int NPASS = kBatch / RPP;               // value rows per thread and round (4)
  constexpr int NTW = kBatch / (16 * NWV);    // 16-token tiles per wavefront and round
  const int seg = tid % LPR, rsub = tid / LPR;
  float run_m = -INFINITY, run_Z = 0.f, run_zs = 0.f, run_nu = 0.f, run_zv = 0.f;   // (nu, zv: channel tid < D)
  wkp.commit(wk_lds);                               // (requested before the histogram pass: long since arrived)
  if (tid < D) { sh_bk[tid] = bk_t; sh_pq[tid] = pq_t; }
  __syncthreads();                                  // lds_a changes hands; the staged Wk is complete
  // (inside the loop the wavefronts exchange data through LDS only: its barriers leave the key and value loads in flight)
  // winner j of the round that starts at b0 (thread t < kBatch <-> winner b0 + t)
  auto winner = [&](int b0, int j, int* tok, float* s) {
    const int i = b0 + min(j, min(kBatch, my_count - b0) - 1);
    if (i < kWinLds) { *tok = w_tok[i]; *s = w_s[i]; }
    else { *tok = sel_idx[min(my_base + i, g.max_K - 1)]; *s = sel_score[min(my_base + i, g.max_K - 1)]; }
    *tok = g.n_sink + min(max(*tok, 0), n - 1);
  };
  // The key rows of this wavefront's tiles and the value rows of all passes only need the token indices.  The rows
  // of round b + 1 are requested inside round b, each set into the registers round b has just finished with (keys
  // after the feature dots, values after the weighted sums): a round trip to memory per workgroup, not per round.
  GatherFrag a[NTW][KS];
  u32x4 vrow[NPASS];
  auto load_keys = [&](int b0) {
    const int cnt = min(kBatch, my_count - b0);
#pragma unroll
    for (int u = 0; u < NTW; ++u) {
      const int t16 = (wv + u * NWV) * 16;      // first token of this wavefront's u-th tile
      if (t16 < cnt) {
        int tk; float s;
        winner(b0, t16 + r, &tk, &s);
        const char* rp = (const char*)pr.K + (head_off + (int64_t)tk * pr.stride_tok) * 2 + kg * 16;
#pragma unroll
        for (int j = 0; j < KS; ++j) a[u][j].u = gload128(rp + j * 64);
      }
    }
  };
  auto load_values = [&](int b0) {
    const int cnt = min(kBatch, my_count - b0);
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
      if (ps * RPP < cnt) {
        int vtok; float vs;
        winner(b0, ps * RPP + rsub, &vtok, &vs);
        vrow[ps] = gload128((const char*)pr.V + (head_off + (int64_t)vtok * pr.stride_tok + seg * 8) * 2);
      }
    }
  };
  if (my_count > 0) { load_keys(0); load_values(0); }
  for (int b0 = 0; b0 < my_count; b0 += kBatch) {
    const int cnt = min(kBatch, my_count - b0);
    const bool more = b0 + kBatch < my_count;
    // batch maximum of the scores
    if (tid < kBatch) {
      int tk; float s;
      winner(b0, tid, &tk, &s);
      b_w[tid] = tid < cnt ? s : -INFINITY;         // (scores for now)
    }
    lds_barrier();
    if (wv == 0) {
      float mloc = -INFINITY;
#pragma unroll
      for (int k = 0; k < kBatch / 64; ++k) mloc = fmaxf(mloc, b_w[lane + 64 * k]);
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) mloc = fmaxf(mloc, __shfl_xor(mloc, o));
      if (lane == 0) sh_m = mloc;
    }
    // z_i of this wavefront's tokens
#pragma unroll
    for (int u = 0; u < NTW; ++u) {
      const int t16 = (wv + u * NWV) * 16;
      if (t16 < cnt) {
        float z[4];
        wave_feature_dots<D>(a[u], wk_lds, sh_bk, sh_pq, g.a, g.c, z);
        if (r == 0) {
#pragma unroll
          for (int i = 0; i < 4; ++i) b_z[t16 + 4 * kg + i] = (t16 + 4 * kg + i < cnt) ? z[i] : 0.f;
        }
      } else if (lane < 16) {
        b_z[t16 + lane] = 0.f;
      }
    }
    if (more) load_keys(b0 + kBatch);
    lds_barrier();
    const float mloc = sh_m;
    if (tid < kBatch) b_w[tid] = tid < cnt ? __expf(b_w[tid] - mloc) : 0.f;
    lds_barrier();
    // weighted value sums: rows of one wavefront that share a segment, then the 16 wavefronts
    float an[8], az[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { an[e] = 0.f; az[e] = 0.f; }
#pragma unroll
    for (int ps = 0; ps < NPASS; ++ps) {
      const int i = ps * RPP + rsub;
      if (ps * RPP < cnt && i < cnt) {
        float x[8];
        Elem<uint16_t>::unpack(make_uint4(vrow[ps].x, vrow[ps].y, vrow[ps].z, vrow[ps].w), x);
        const float wi = b_w[i], zi = b_z[i];
#pragma unroll
        for (int e = 0; e < 8; ++e) { an[e] = fmaf(wi, x[e], an[e]); az[e] = fmaf(zi, x[e], az[e]); }
      }
    }
    if (more) load_values(b0 + kBatch);
    for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { an[e] += __shfl_xor(an[e], o); az[e] += __shfl_xor(az[e], o); }
    }
    if (lane < LPR) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { red[(wv * 2 + 0) * 128 + lane * 8 + e] = an[e]; red[(wv * 2 + 1) * 128 + lane * 8 + e] = az[e]; }
    }
    if (wv == 1) {                                  // Z_loc and zsum of the batch, in a fixed order
      float Zb = (b_w[lane] + b_w[lane + 64]) + (b_w[lane + 128] + b_w[lane + 192]);
      float zb = (b_z[lane] + b_z[lane + 64]) + (b_z[lane + 128] + b_z[lane + 192]);
#pragma unroll
      for (int k = 4; k < kBatch / 64; k += 4) {    // (all zero in a round of at most 256 winners)
        Zb += (b_w[lane + 64 * k] + b_w[lane + 64 * (k + 1)]) + (b_w[lane + 64 * (k + 2)] + b_w[lane + 64 * (k + 3)]);
        zb += (b_z[lane + 64 * k] + b_z[lane + 64 * (k + 1)]) + (b_z[lane + 64 * (k + 2)] + b_z[lane + 64 * (k + 3)]);
      }
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) { Zb += __shfl_xor(Zb, o); zb += __shfl_xor(zb, o); }
      if (lane == 0) { sh_Z = Zb; sh_zs = zb; }
    }
    lds_barrier();
    {
      float nu_b = 0.f, zv_b = 0.f;
      if (tid < D) {
        for (int k = 0; k < NWV; ++k) { nu_b += red[(k * 2 + 0) * 128 + tid]; zv_b += red[(k * 2 + 1) * 128 + tid]; }
      }
      // running combination with the earlier batches (log-sum-exp rescaling)
      const float m_new = fmaxf(run_m, mloc);
      const float so = run_m > -INFINITY ? __expf(run_m - m_new) : 0.f, sb = __expf(mloc - m_new);
      run_nu = run_nu * so + nu_b * sb;
      run_Z = run_Z * so + sh_Z * sb;
      run_zv += zv_b;
      run_zs += sh_zs;
      run_m = m_new;
    }
    lds_barrier();                                // red, b_w, b_z are rewritten by the next batch
  }
  // (GPU-coherent stores: the workgroup that merges the head may run on another XCD)
  if (tid == 0) { store_agent(partial, run_m); store_agent(partial + 1, run_Z); store_agent(partial + 2, run_zs); store_agent(partial + 3, (float)my_count); }
  if (tid < D) { store_agent(partial + 4 + tid, run_nu); store_agent(partial + 4 + D + tid, run_zv); }
  TKPHI_PHASE(ws, 16);
}

// grid (sg_split, Hq, n_problems).  After its own share every workgroup of a head counts itself in (its partial made
// visible first); the one that arrives last finds all partials of the head complete and merges them (merge_head.h)
// with its first 256 threads: no separate merge launch.  The counters are cleared by the prep kernel of the same
// call.  (The other wavefronts of that workgroup end before the merge's barriers: a barrier waits only for the
// wavefronts of the workgroup that are still running.)
template <int D, int TPI, int NTHR>
__global__ __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(4, 4))) void select_gather_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                    char* __restrict__ ws, int mode) {
  __shared__ int sh_last;
  const int part = blockIdx.x, gq = blockIdx.y, p = blockIdx.z;
  select_gather_body<D, TPI, NTHR>(g, probs, ws, part, gq, p);
  const int L = probs[p].L;
  if (L < 1 || L > g.max_L) return;                 // (the merge writes nothing for such a problem either)
  // The partial went out with GPU-coherent stores and the merge reads the partials with GPU-coherent loads; the
  // barrier below waits for this workgroup's stores to complete before thread 0 counts it in.  Only the optional
  // export of the retrieved indices reads what ordinary stores of other workgroups wrote (the retrieved list): then,
  // and only then, device-wide fences (each writes back / invalidates a whole L2) bracket the count.
  const bool exports = probs[p].topk_idx != nullptr;
  if (exports) __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t* arrived = (uint32_t*)(problem_block(g, ws, p) + g.off_mcount) + gq;
    sh_last = atomicAdd(arrived, 1u) == (uint32_t)g.sg_split - 1u ? 1 : 0;
  }
  __syncthreads();
  if (!sh_last || threadIdx.x >= kThreads) return;
  if (exports) __threadfence();
  merge_head<true, true>(g, probs, ws, gq, p, mode);
}

void launch_select_gather(const Geom& g, const tkphi_problem* probs, char* ws, int mode, hipStream_t s) {
  dim3 grid(g.sg_split, g.Hq, g.n_problems);       // (Geom::n_tiles of this pipeline: one partial per workgroup)
  // Batches of short sequences at d = 64 (one workgroup per head, at least two heads per CU): 512-thread workgroups,
  // two per CU, so that one head's memory round trips hide behind the other's arithmetic
  const bool small_wg = g.d == 64 && g.sg_split == 1 && (long)g.Hq * g.n_problems >= 512 && g.max_K <= 1024;
  if (g.d == 128) TKPHI_LAUNCH(ST_SELECT, (select_gather_kernel<128, 4, 1024>), grid, dim3(1024), 0, s, g, probs, ws, mode);
  else if (small_wg) TKPHI_LAUNCH(ST_SELECT, (select_gather_kernel<64, 8, 512>), grid, dim3(512), 0, s, g, probs, ws, mode);
  else TKPHI_LAUNCH(ST_SELECT, (select_gather_kernel<64, 8, 1024>), grid, dim3(1024), 0, s, g, probs, ws, mode);
}

}  // namespace tkphi
