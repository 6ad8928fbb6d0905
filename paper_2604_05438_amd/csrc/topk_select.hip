// topk_select: exhaustive Top-K over the mid-region scores of every query head
// (Sec. "Models, tasks, and protocol": the K highest-scoring mid-region tokens), plus the
// query feature map phi_q (App. "Head-wise phi architecture": one map per query head, run once
// per decode step).
//
// A two-level radix select in three small kernels, with no atomics and a fixed output order:
//   plan     one workgroup per query head: sums the per-chunk (suffix-count) histograms written
//            by score_mid -> boundary bin b* (the bin holding the K-th largest score; every token
//            in a higher bin is retrieved); per chunk, the output offsets of its tokens above
//            b* and of its tokens in b* (exclusive prefix sums of the chunk counts)
//   emit     one wavefront per chunk, all heads in parallel: one ordered pass over the chunk's
//            scores; tokens above b* go straight to the retrieved list, tokens in b* become
//            candidates, both at the offsets computed by `plan`
//   resolve  a few workgroups per query head: the K_rem best candidates by (score descending,
//            index ascending) are appended to the list
// The list holds (mid index, score): first the tokens above b* chunk by chunk (ascending
// index order when chunks are contiguous), then the boundary-bin winners (by rank, or in
// ascending index order on the radix paths).
// Ties go to the lower index.  If the boundary bin holds more than kCandCap tokens (e.g. all
// scores equal) `resolve` falls back to radix passes over the score row in global memory:
// slower, same result.  The ascending export of the retrieved set is written by the merge kernel.
#include "select_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

// the 8 uint16 counts a lane holds after a 16-byte load of a chunk histogram row
__device__ __forceinline__ void unpack_counts(const u32x4& v, uint32_t* c) {
  c[0] = v.x & 0xffffu; c[1] = v.x >> 16; c[2] = v.y & 0xffffu; c[3] = v.y >> 16;
  c[4] = v.z & 0xffffu; c[5] = v.z >> 16; c[6] = v.w & 0xffffu; c[7] = v.w >> 16;
}

// ------------------------------------------------------------------------------------
// plan: grid (Hq or 2 Hq, n_problems), 1024 threads.  Workgroup x < Hq plans query head x; with
// 2 Hq workgroups (few heads in flight) workgroup Hq + x evaluates phi_q of head x at the same
// time, otherwise workgroup x does it first.  One workgroup also writes the device status word.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void select_plan_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                  char* __restrict__ ws) {
  __shared__ uint32_t sh_tot[kBins];
  __shared__ int sh_scan[kSelWaves];
  __shared__ int sh_bstar, sh_krem, sh_chi, sh_nb;
  __shared__ int sh_ca[kMaxScanChunks], sh_cc[kMaxScanChunks];

  const int p = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  char* blk = problem_block(g, ws, p);
  // few heads in flight (gridDim.x == 2 Hq): phi_q has workgroups of its own and leaves the
  // critical path; many heads: every planning workgroup evaluates phi_q of its head first
  const bool split = (int)gridDim.x > g.Hq;
  const bool side_job = (int)blockIdx.x >= g.Hq;
  const int gq = side_job ? (int)blockIdx.x - g.Hq : (int)blockIdx.x;
  if ((side_job || !split) && gq == 0 && p == 0) write_device_status(g, probs, ws, true);

  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  if (side_job || !split) {
    if (g.phi_kind == TKPHI_PHI_MLP) { if (side_job) return; }    // phi_q came from the MLP launches
    else if (g.dtype == TKPHI_BF16) phi_q_head<uint16_t>(g, pr, blk, gq, (float*)sh_tot);
    else phi_q_head<float>(g, pr, blk, gq, (float*)sh_tot);
    if (side_job) return;
    __syncthreads();                     // sh_tot served as scratch
  }
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int Ksel = max(0, min(min(pr.topk, n), g.max_K));
  SelPlan* plan = (SelPlan*)(blk + g.off_plan) + gq;

  if (Ksel == 0) {
    if (tid == 0) *plan = SelPlan{-1, 0, 0, 0, 0};
    return;
  }

  const int n_chunks = (n + g.scan_chunk - 1) / g.scan_chunk;
  const uint16_t* hist = (const uint16_t*)(blk + g.off_hist) + (size_t)gq * kBins;   // + chunk * Hq * kBins
  const size_t hstep = (size_t)g.Hq * kBins;

  // ---- total histogram: lane owns bins 8*lane .. 8*lane+7 (one 16-byte load per chunk),
  // wavefront wv takes chunks wv, wv + 16, ...; the 16 wavefront sums meet in LDS ---------------
  if (tid < kBins) sh_tot[tid] = 0u;
  if (tid == 0) { sh_bstar = -1; sh_krem = 0; sh_chi = 0; }
  __syncthreads();
  {
    uint32_t t[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    constexpr int UH = 8;                // row loads in flight per lane
    for (int c0 = wv; c0 < n_chunks; c0 += kSelWaves * UH) {
      u32x4 v[UH];
#pragma unroll
      for (int k = 0; k < UH; ++k) {
        const int c = c0 + k * kSelWaves;
        // unconditional load from a clamped row (a predicated load would be waited for on its own)
        v[k] = gload128((const char*)(hist + (size_t)min(c, n_chunks - 1) * hstep) + lane * 16);
        if (c >= n_chunks) v[k] = (u32x4){0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int k = 0; k < UH; ++k) {
        uint32_t c8[8];
        unpack_counts(v[k], c8);
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] += c8[e];
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) if (t[e]) atomicAdd(&sh_tot[lane * 8 + e], t[e]);
  }
  __syncthreads();
  // the rows are suffix sums, so sh_tot[b] = tokens of this head in bins >= b: the boundary bin
  // is the highest b with sh_tot[b] >= K
  if (tid < kBins) {
    const int ge = (int)sh_tot[tid];
    const int gt = tid + 1 < kBins ? (int)sh_tot[tid + 1] : 0;
    if (ge >= Ksel && gt < Ksel) { sh_bstar = tid; sh_krem = Ksel - gt; sh_chi = gt; sh_nb = ge - gt; }
  }
  __syncthreads();
  const int bstar = sh_bstar;
  if (bstar < 0) {                       // cannot happen for consistent histograms
    if (tid == 0) *plan = SelPlan{-1, 0, 0, 0, 0};
    return;
  }

  // ---- per chunk: tokens above b*, tokens in b* (two suffix counts per chunk) ----------------------
  for (int c = tid; c < n_chunks; c += kSelThreads) {
    const uint16_t* row = hist + (size_t)c * hstep;
    const int ge = row[bstar];
    const int gt = bstar + 1 < kBins ? row[bstar + 1] : 0;
    sh_ca[c] = gt; sh_cc[c] = ge - gt;
  }
  __syncthreads();
  {
    constexpr int PER = kMaxScanChunks / kSelThreads;      // 2 chunks per thread
    int va[PER], vc[PER], ta = 0, tc = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid * PER + i;
      va[i] = c < n_chunks ? sh_ca[c] : 0;
      vc[i] = c < n_chunks ? sh_cc[c] : 0;
      ta += va[i]; tc += vc[i];
    }
    // both sums fit 2 x 20 bits? no: scan them separately (|M| can exceed 2^20)
    const int ia = sel_scan_incl(ta, sh_scan);
    const int ic = sel_scan_incl(tc, sh_scan);
    int ra = ia - ta, rc = ic - tc;
    int32_t* choff = (int32_t*)(blk + g.off_chunkoff) + (size_t)gq * g.n_scan_chunks * 2;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid * PER + i;
      if (c < n_chunks) { choff[2 * c] = ra; choff[2 * c + 1] = rc; }
      ra += va[i]; rc += vc[i];
    }
  }
  if (tid == 0) *plan = SelPlan{bstar, sh_krem, sh_chi, sh_nb, Ksel};
}

// ------------------------------------------------------------------------------------
// emit: grid (ceil(n_scan_chunks / 4), Hq, n_problems), 256 threads; wavefront w <-> one chunk
// ------------------------------------------------------------------------------------
template <bool IL, int U, bool DIAG>   // IL: interleaved chunks (Geom::interleave); U: loads in flight per
                                       // lane; DIAG: also reduce (max, sum e^(s-max), sum (s-max) e^(s-max))
__global__ __launch_bounds__(kThreads) void select_emit_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                               char* __restrict__ ws) {
  const int gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const int lane = tid & 63, wv = tid >> 6;
  const int L = probs[p].L;
  if (L < 1 || L > g.max_L) return;
  const int n = mid_size(L, g.n_sink, g.n_tail);
  char* blk = problem_block(g, ws, p);
  const SelPlan plan = ((const SelPlan*)(blk + g.off_plan))[gq];
  int bstar = plan.bstar;
  if (bstar < 0) {
    if (!DIAG) return;
    bstar = kBins;                       // nothing to retrieve: the pass only reduces the diagnostics
  }
  // (rotated per head and problem: in a ragged batch late chunks are rare, and workgroups go to
  // the XCDs round-robin by linear index)
  const int chunk = (((int)blockIdx.x + gq + p * g.Hq) % (int)gridDim.x) * 4 + wv;
  const int n_chunks = (n + g.scan_chunk - 1) / g.scan_chunk;
  if (chunk >= n_chunks) return;
  // the chunk's tokens in blocks of 256, in the order score_mid took them: block s lies in unit
  // s / (scan_unit / 256) of the chunk (contiguous chunks: simply t0 + 256 s)
  const int bpu = IL ? g.scan_unit / 256 : 1;
  const int n_blocks = g.scan_chunk / 256;
  const int t1 = IL ? n : min(n, (chunk + 1) * g.scan_chunk);
  auto block_token = [&](int s) {
    if (IL) return s < n_blocks ? (chunk + (s / bpu) * n_chunks) * g.scan_unit + (s % bpu) * 256 : t1;
    return chunk * g.scan_chunk + s * 256;
  };
  const bool keep_cand = plan.nb <= kCandCap;
  // the histogram fixed how many tokens lie above / inside the threshold bin; the writes are
  // bounded by those counts so that scores that disagree with it cannot leave the buffers
  const int a_cap = min(plan.c_hi, g.max_K), c_cap = min(plan.nb, kCandCap);
  const float* scores = (const float*)(blk + g.off_scores) + (size_t)gq * g.mid_stride;
  int32_t* sel_idx = (int32_t*)(blk + g.off_selidx) + (size_t)gq * g.max_K;
  float* sel_score = (float*)(blk + g.off_selscore) + (size_t)gq * g.max_K;
  uint2* cand = (uint2*)(blk + g.off_cand) + (size_t)gq * kCandCap;
  const int32_t* choff = (const int32_t*)(blk + g.off_chunkoff) + ((size_t)gq * g.n_scan_chunks + chunk) * 2;
  int a_pos = choff[0], c_pos = choff[1];

  // 4 consecutive tokens per lane, 256 per wavefront instruction
  float dm = -INFINITY, dz = 0.f, dw = 0.f;        // this lane's share of the chunk record (DIAG)
  for (int s0 = 0; s0 < n_blocks; s0 += U) {
    if (block_token(s0) >= t1) break;
    float4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = block_token(s0 + u) + lane * 4;
      v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (tok + 3 < t1) v[u] = *(const float4*)(scores + tok);     // rows are 16-byte aligned (mid_stride % 64 == 0)
      else {
        if (tok < t1) v[u].x = scores[tok];
        if (tok + 1 < t1) v[u].y = scores[tok + 1];
        if (tok + 2 < t1) v[u].z = scores[tok + 2];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tok = block_token(s0 + u) + lane * 4;
      const float sv[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
      if (DIAG) {
        float mx = dm;
#pragma unroll
        for (int e = 0; e < 4; ++e) if (tok + e < t1) mx = fmaxf(mx, sv[e]);
        if (mx > dm) {                               // new shift: rescale what has been summed
          if (dz > 0.f) { const float r = __expf(dm - mx); dw = (dw + (dm - mx) * dz) * r; dz *= r; }
          dm = mx;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (tok + e < t1) { const float x = sv[e] - dm, ex = __expf(x); dz += ex; dw = fmaf(x, ex, dw); }
        }
      }
      int fa[4], fc[4], na = 0, nc = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int b = (tok + e < t1) ? key_bin(score_key(sv[e])) : -1;
        fa[e] = b > bstar ? 1 : 0;
        fc[e] = b == bstar ? 1 : 0;
        na += fa[e]; nc += fc[e];
      }
      // exclusive prefix over lanes of (na, nc) packed in one int (each <= 256)
      const int packed = na | (nc << 16);
      int x = packed;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(x, o);
        if (lane >= o) x += y;
      }
      const int total = __shfl(x, 63);
      int pa = a_pos + ((x - packed) & 0xffff), pc = c_pos + ((x - packed) >> 16);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (fa[e]) { if (pa < a_cap) { sel_idx[pa] = tok + e; sel_score[pa] = sv[e]; } ++pa; }
        if (fc[e]) { if (keep_cand && pc < c_cap) cand[pc] = make_uint2(score_key(sv[e]), (uint32_t)(tok + e)); ++pc; }
      }
      a_pos += total & 0xffff;
      c_pos += total >> 16;
    }
  }
  if (DIAG) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      const float m2 = __shfl_xor(dm, o), z2 = __shfl_xor(dz, o), w2 = __shfl_xor(dw, o);
      const float mm = fmaxf(dm, m2);
      float za = 0.f, wa = 0.f, zb = 0.f, wb = 0.f;
      if (dz > 0.f) { const float r = __expf(dm - mm); za = dz * r; wa = (dw + (dm - mm) * dz) * r; }
      if (z2 > 0.f) { const float r = __expf(m2 - mm); zb = z2 * r; wb = (w2 + (m2 - mm) * z2) * r; }
      dm = mm; dz = za + zb; dw = wa + wb;
    }
    if (lane == 0) ((float4*)(blk + g.off_diag))[(size_t)chunk * g.Hq + gq] = make_float4(dm, dz, dw, 0.f);
  }
}

// ------------------------------------------------------------------------------------
// resolve: grid (split, Hq, n_problems), 1024 threads; dynamic LDS: kCandCap x 8 bytes
//
// Boundary-bin candidates that fit the LDS stage and whose rank counting is short enough for the
// workgroups at hand (rounds of 128 candidates x nb <= kCountWork: 1024 candidates for one workgroup
// per head, all kCandCap = 4096 for 16): the `split` workgroups of a head share the work.  Each one stages all candidates (as 64-bit composites) in LDS and ranks
// its own slice by counting the larger ones, 8 lanes per candidate; a candidate of rank
// r < K_rem goes to list position c_hi + r, so the winners follow the tokens above b* in
// descending (score, then ascending index) order and no scan is needed.  More candidates:
// workgroup 0 alone runs radix passes (over the staged candidates, or over the score row if
// they exceeded kCandCap) and appends the winners in ascending index order.
// ------------------------------------------------------------------------------------
constexpr int kResolveSplitMax = 16;      // workgroups per head when few heads are in flight
constexpr int kCountWork = 16384;

__global__ __launch_bounds__(kSelThreads) void select_resolve_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                     char* __restrict__ ws) {
  __shared__ uint32_t sh_hist[256];
  __shared__ int sh_scan[kSelWaves];
  __shared__ uint64_t sh_prefix;
  __shared__ int sh_want;
  extern __shared__ uint64_t sh_comp[];  // [kCandCap] composites of the candidates, ascending row

  const int part = blockIdx.x, gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  char* blk = problem_block(g, ws, p);
  const SelPlan plan = ((const SelPlan*)(blk + g.off_plan))[gq];
  const int bstar = plan.bstar, krem = plan.krem, c_hi = plan.c_hi, nb = plan.nb, Ksel = plan.n_sel;
  if (bstar < 0 || Ksel == 0) return;
  const int per = (nb + (int)gridDim.x - 1) / (int)gridDim.x;         // candidates per workgroup when they are counted
  const bool count_path = nb <= kCandCap && ((per + kSelThreads / 8 - 1) / (kSelThreads / 8)) * nb <= kCountWork;
  if (!count_path && part != 0) return;
  const float* scores = (const float*)(blk + g.off_scores) + (size_t)gq * g.mid_stride;
  int32_t* sel_idx = (int32_t*)(blk + g.off_selidx) + (size_t)gq * g.max_K;
  float* sel_score = (float*)(blk + g.off_selscore) + (size_t)gq * g.max_K;
  // list positions never leave [c_hi, Ksel) <= max_K whatever the candidates hold
  const int k_cap = min(krem, max(0, min(Ksel, g.max_K) - c_hi));

  if (nb <= kCandCap) {
    const uint2* cand = (const uint2*)(blk + g.off_cand) + (size_t)gq * kCandCap;
    for (int j = tid; j < nb; j += kSelThreads) { const uint2 e = cand[j]; sh_comp[j] = composite(e.x, e.y); }
    __syncthreads();
    if (count_path) {
      const int sub = tid & 7, slot = tid >> 3;                       // 8 lanes per candidate, 128 slots
      for (int k0 = 0; k0 < per; k0 += kSelThreads / 8) {
        const int k = k0 + slot, j = part * per + k;
        const bool valid = k < per && j < nb;
        const uint64_t mine = valid ? sh_comp[j] : ~0ull;
        int rank = 0;
        int i = sub;
        for (; i + 24 < nb; i += 32) {
          const uint64_t c0 = sh_comp[i], c1 = sh_comp[i + 8], c2 = sh_comp[i + 16], c3 = sh_comp[i + 24];
          rank += (c0 > mine ? 1 : 0) + (c1 > mine ? 1 : 0) + (c2 > mine ? 1 : 0) + (c3 > mine ? 1 : 0);
        }
        for (; i < nb; i += 8) rank += sh_comp[i] > mine ? 1 : 0;
        rank += __shfl_xor(rank, 1);
        rank += __shfl_xor(rank, 2);
        rank += __shfl_xor(rank, 4);
        if (valid && sub == 0 && rank < k_cap) {
          sel_idx[c_hi + rank] = (int)(0xffffffffu - (uint32_t)mine);
          sel_score[c_hi + rank] = key_score((uint32_t)(mine >> 32));
        }
      }
      return;
    }
    auto get = [&](int j, uint64_t* v) { *v = sh_comp[j]; return true; };
    const uint64_t thr = radix_select_desc(nb, krem, get, sh_hist, sh_scan, &sh_prefix, &sh_want);
    // ordered append of the winners: thread t owns candidates [t*R, (t+1)*R)
    const int R = (nb + kSelThreads - 1) / kSelThreads;
    int cnt = 0;
    for (int j = tid * R; j < min(nb, (tid + 1) * R); ++j) cnt += sh_comp[j] >= thr ? 1 : 0;
    int pos = sel_scan_incl(cnt, sh_scan) - cnt;
    for (int j = tid * R; j < min(nb, (tid + 1) * R); ++j) {
      const uint64_t e = sh_comp[j];
      if (e >= thr) {
        if (pos < k_cap) { sel_idx[c_hi + pos] = (int)(0xffffffffu - (uint32_t)e); sel_score[c_hi + pos] = key_score((uint32_t)(e >> 32)); }
        ++pos;
      }
    }
  } else {
    auto get = [&](int j, uint64_t* v) {
      const uint32_t key = score_key(scores[j]);
      *v = composite(key, (uint32_t)j);
      return key_bin(key) == bstar;
    };
    const uint64_t thr = radix_select_desc(n, krem, get, sh_hist, sh_scan, &sh_prefix, &sh_want);
    int pos0 = 0;
    for (int base = 0; base < n; base += kSelThreads) {
      const int j = base + tid;
      int f = 0;
      float s = 0.f;
      if (j < n) {
        s = scores[j];
        const uint32_t key = score_key(s);
        f = (key_bin(key) == bstar && composite(key, (uint32_t)j) >= thr) ? 1 : 0;
      }
      const int incl = sel_scan_incl(f, sh_scan);
      if (f && pos0 + incl - 1 < k_cap) { sel_idx[c_hi + pos0 + incl - 1] = j; sel_score[c_hi + pos0 + incl - 1] = s; }
      if (tid == kSelThreads - 1) sh_want = incl;
      __syncthreads();
      pos0 += sh_want;
      __syncthreads();
    }
  }
}

void launch_select(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  dim3 pgrid((g.Hq * g.n_problems <= 128 && g.phi_kind != TKPHI_PHI_MLP ? 2 : 1) * g.Hq, g.n_problems);
  TKPHI_LAUNCH(ST_PLAN, select_plan_kernel, pgrid, dim3(kSelThreads), 0, s, g, probs, ws);
  const bool selecting = g.max_mid > 0 && g.max_K > 0;
  if (!selecting && !(g.diag && g.max_mid > 0)) return;
  dim3 egrid((g.n_scan_chunks + 3) / 4, g.Hq, g.n_problems);
  if (g.diag) {
    if (g.interleave) TKPHI_LAUNCH(ST_EMIT, (select_emit_kernel<true, 2, true>), egrid, dim3(kThreads), 0, s, g, probs, ws);
    else TKPHI_LAUNCH(ST_EMIT, (select_emit_kernel<false, 2, true>), egrid, dim3(kThreads), 0, s, g, probs, ws);
  } else if (g.interleave) {
    TKPHI_LAUNCH(ST_EMIT, (select_emit_kernel<true, 2, false>), egrid, dim3(kThreads), 0, s, g, probs, ws);
  } else if (g.scan_chunk >= 2048) {
    TKPHI_LAUNCH(ST_EMIT, (select_emit_kernel<false, 4, false>), egrid, dim3(kThreads), 0, s, g, probs, ws);
  } else {
    TKPHI_LAUNCH(ST_EMIT, (select_emit_kernel<false, 2, false>), egrid, dim3(kThreads), 0, s, g, probs, ws);
  }
  if (!selecting) return;
  // enough workgroups to spread the rank counting of one layer over the chip, one per head in big batches
  const int split = std::clamp(512 / std::max(1, g.Hq * g.n_problems), 1, kResolveSplitMax);
  dim3 rgrid(split, g.Hq, g.n_problems);
  TKPHI_LAUNCH(ST_RESOLVE, select_resolve_kernel, rgrid, dim3(kSelThreads), (size_t)kCandCap * sizeof(uint64_t), s, g, probs, ws);
}

}  // namespace tkphi
