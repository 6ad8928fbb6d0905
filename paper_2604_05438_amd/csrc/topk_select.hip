// topk_select: exhaustive Top-K over the mid-region scores of one query head
// (Sec. "Models, tasks, and protocol": the K highest-scoring mid-region tokens), as a
// multi-workgroup radix select.
//
//   level 1  (done by score_mid)  histogram of a monotone bin of the score
//   this kernel, every workgroup  boundary bin b* = the bin holding the K-th largest
//                                 score; count, per slice, the tokens in bins above b*
//                                 and collect the tokens of bin b* as candidates
//   last workgroup of the head    exact K_rem-th largest candidate by (score descending,
//                                 index ascending) -> threshold (thr_key, thr_idx); per
//                                 slice output offsets so the gather pass can emit the
//                                 retrieved indices in ascending order
//
// The result is the selection predicate
//   retrieved(i)  <=>  key_i > thr_key  ||  (key_i == thr_key && i <= thr_idx)
// which is exact for any input (ties go to the lower index).  If the boundary bin holds
// more than kCandCap tokens the last workgroup falls back to radix passes over the
// head's score row in global memory: slower, same result.
#include "block_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

constexpr int kBinsPerThread = (kBins + kThreads - 1) / kThreads;   // 7

// K-th largest (1-based rank `want`) 64-bit composite among `count` elements delivered
// by get(j, &composite) -> bool (false: element does not take part).  8 radix passes of
// 8 bits.  All threads must call; returns the composite in every thread.
template <typename Get>
__device__ uint64_t radix_select_desc(int count, int want, Get get, uint32_t* sh_hist /*[256]*/,
                                      int* sh_scan /*[4]*/, uint64_t* sh_prefix, int* sh_want) {
  const int tid = threadIdx.x;
  if (tid == 0) { *sh_prefix = 0ull; *sh_want = want; }
  __syncthreads();
  for (int shift = 56; shift >= 0; shift -= 8) {
    sh_hist[tid] = 0u;
    __syncthreads();
    const uint64_t prefix = *sh_prefix;
    const int w = *sh_want;
    const uint64_t himask = shift == 56 ? 0ull : (~0ull << (shift + 8));
    for (int j = tid; j < count; j += kThreads) {
      uint64_t v;
      if (get(j, &v) && (v & himask) == prefix) atomicAdd(&sh_hist[(uint32_t)(v >> shift) & 255u], 1u);
    }
    __syncthreads();
    // thread t looks at digit 255 - t: prefix scan over t == suffix scan over digits
    const int digit = 255 - tid;
    const int c = (int)sh_hist[digit];
    const int incl = block_scan_incl(c, sh_scan);
    const int excl = incl - c;
    if (excl < w && w <= incl) {
      *sh_prefix = prefix | ((uint64_t)digit << shift);
      *sh_want = w - excl;
    }
    __syncthreads();
  }
  return *sh_prefix;
}

__device__ __forceinline__ uint64_t composite(uint32_t key, uint32_t row) {
  return ((uint64_t)key << 32) | (uint64_t)(0xffffffffu - row);
}

// grid (n_sel_slices, Hq, n_problems)
__global__ __launch_bounds__(kThreads) void select_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                          char* __restrict__ ws) {
  __shared__ uint32_t sh_hist[256];
  __shared__ int sh_scan[4];
  __shared__ uint64_t sh_prefix;
  __shared__ int sh_want, sh_bstar, sh_krem, sh_last;
  __shared__ int sh_slice[1024];
  extern __shared__ uint2 sh_cand[];     // [kCandCap] (key, row)

  const int sl = blockIdx.x, gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const int L = probs[p].L;
  if (L < 1 || L > g.max_L) return;
  const int n = mid_size(L, g.n_sink, g.n_tail);
  const int Ksel = max(0, min(min(probs[p].topk, n), g.max_K));
  const int n_slices = (n + g.sel_chunk - 1) / g.sel_chunk;
  const int n_wg = max(n_slices, 1);
  if (sl >= n_wg) return;

  char* blk = problem_block(g, ws, p);
  const uint32_t* hist = (const uint32_t*)(blk + g.off_hist) + (size_t)gq * kBins;
  HeadState* st = (HeadState*)(blk + g.off_state) + gq;
  const float* scores = (const float*)(blk + g.off_scores) + (size_t)gq * g.mid_stride;
  uint2* cand = (uint2*)(blk + g.off_cand) + (size_t)gq * kCandCap;
  int32_t* above = (int32_t*)(blk + g.off_above) + (size_t)gq * g.n_sel_slices;
  int32_t* offsets = (int32_t*)(blk + g.off_offsets) + (size_t)gq * g.n_sel_slices;

  // ---- boundary bin ----------------------------------------------------------------
  if (tid == 0) { sh_bstar = kBins; sh_krem = 0; }
  __syncthreads();
  {
    const int grp = kThreads - 1 - tid;            // thread t owns the bin group 255 - t
    const int lo = grp * kBinsPerThread;
    int c[kBinsPerThread];
    int tot = 0;
#pragma unroll
    for (int i = 0; i < kBinsPerThread; ++i) {
      const int b = lo + i;
      c[i] = b < kBins ? (int)hist[b] : 0;
      tot += c[i];
    }
    const int incl = block_scan_incl(tot, sh_scan);
    int run = incl - tot;                          // tokens in bins above this group
    if (Ksel > 0 && run < Ksel && Ksel <= incl) {
#pragma unroll
      for (int i = kBinsPerThread - 1; i >= 0; --i) {
        if (run < Ksel && Ksel <= run + c[i]) { sh_bstar = lo + i; sh_krem = Ksel - run; }
        run += c[i];
      }
    }
  }
  __syncthreads();
  const int bstar = sh_bstar, krem = sh_krem;

  // ---- filter pass over this slice -------------------------------------------------
  const int t0 = sl * g.sel_chunk, t1 = min(n, t0 + g.sel_chunk);
  int n_above = 0;
  for (int base = t0; base < t1; base += kThreads) {
    const int row = base + tid;
    bool is_cand = false;
    uint32_t key = 0;
    if (row < t1) {
      key = score_key(scores[row]);
      const int b = key_bin(key);
      n_above += (b > bstar) ? 1 : 0;
      is_cand = (b == bstar);
    }
    const uint64_t mask = __ballot(is_cand);
    if (mask) {
      const int lane = tid & 63;
      const int leader = __ffsll((long long)mask) - 1;
      uint32_t basepos = 0;
      if (lane == leader) basepos = atomicAdd(&st->cand_count, (uint32_t)__popcll(mask));
      basepos = __shfl(basepos, leader);
      if (is_cand) {
        const uint32_t slot = basepos + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
        if (slot < (uint32_t)kCandCap) cand[slot] = make_uint2(key, (uint32_t)row);
      }
    }
  }
  n_above = block_sum_int(n_above, sh_scan);
  if (tid == 0 && n_slices > 0) above[sl] = n_above;

  // ---- ticket: the last workgroup of this head resolves the boundary bin ------------
  __threadfence();          // every thread publishes its candidate / count stores device-wide
  __syncthreads();
  if (tid == 0) {
    const uint32_t t = atomicAdd(&st->ticket, 1u);
    sh_last = (t == (uint32_t)(n_wg - 1)) ? 1 : 0;
  }
  __syncthreads();
  if (!sh_last) return;
  __threadfence();

  uint32_t thr_key = 0xffffffffu;
  int32_t thr_idx = -1;
  for (int i = tid; i < 1024; i += kThreads) sh_slice[i] = 0;
  __syncthreads();
  const bool have_thr = Ksel > 0 && bstar < kBins;
  if (have_thr) {
    const int nb = (int)hist[bstar];
    uint64_t T;
    if (nb <= kCandCap) {
      for (int j = tid; j < nb; j += kThreads) sh_cand[j] = cand[j];
      __syncthreads();
      auto get = [&](int j, uint64_t* v) { const uint2 e = sh_cand[j]; *v = composite(e.x, e.y); return true; };
      T = radix_select_desc(nb, krem, get, sh_hist, sh_scan, &sh_prefix, &sh_want);
      for (int j = tid; j < nb; j += kThreads) {
        const uint2 e = sh_cand[j];
        if (composite(e.x, e.y) >= T) atomicAdd(&sh_slice[e.y / g.sel_chunk], 1);
      }
    } else {
      auto get = [&](int j, uint64_t* v) {
        const uint32_t key = score_key(scores[j]);
        *v = composite(key, (uint32_t)j);
        return key_bin(key) == bstar;
      };
      T = radix_select_desc(n, krem, get, sh_hist, sh_scan, &sh_prefix, &sh_want);
      for (int j = tid; j < n; j += kThreads) {
        const uint32_t key = score_key(scores[j]);
        if (key_bin(key) == bstar && composite(key, (uint32_t)j) >= T) atomicAdd(&sh_slice[j / g.sel_chunk], 1);
      }
    }
    thr_key = (uint32_t)(T >> 32);
    thr_idx = (int32_t)(0xffffffffu - (uint32_t)(T & 0xffffffffull));
  }
  __syncthreads();
  // per-slice output offsets: exclusive prefix over slices of (above + selected in bin b*)
  {
    constexpr int PER = 1024 / kThreads;   // 4
    int v[PER], tot = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int s = tid * PER + i;
      v[i] = s < n_slices ? (sh_slice[s] + (have_thr ? above[s] : 0)) : 0;
      tot += v[i];
    }
    const int incl = block_scan_incl(tot, sh_scan);
    int run = incl - tot;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int s = tid * PER + i;
      if (s < n_slices) offsets[s] = run;
      run += v[i];
    }
  }
  if (tid == 0) {
    st->thr_key = thr_key;
    st->thr_idx = thr_idx;
    st->bstar = bstar;
    st->krem = krem;
    st->n_sel = Ksel;
  }
}

void launch_select(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  dim3 grid(g.n_sel_slices, g.Hq, g.n_problems);
  hipLaunchKernelGGL(select_kernel, grid, dim3(kThreads), (size_t)kCandCap * sizeof(uint2), s, g, probs, ws);
}

}  // namespace tkphi
