// Decode back end.
//
// gather (exact_branch + residual_correct): for every slice of the mid-region and for the
// anchors, accumulates per query head
//     m_loc = max s_i,  Z_loc = sum exp(s_i - m_loc),  nu_loc = sum exp(s_i - m_loc) v_i
// over the retrieved tokens of the slice (eq. (exact_terms)), and the feature-space
// contributions to subtract from the summaries (eq. (subtraction)), kept as the already
// contracted sums  zsum = sum_i z_i,  zv = sum_i z_i v_i  with
// z_i = phi_q(q) . phi_k(k_i)  and phi_k(k_i) recomputed from the gathered key, so that S_R
// is never materialised:  S_R^T phi_q = S_M^T phi_q - zv,  phi_q . u_R = phi_q . u_M - zsum.
//
// merge: combines the slice partials in a fixed order (log-sum-exp rescaling), evaluates
// the summary terms and applies the single-normalisation merge (eq. (hybrid_merge)) with
// the exact branch's max shift applied to the residual branch.
#include "block_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

constexpr int kPairCap = 3072;    // (query head, token) pairs queued in LDS before a flush

struct Pair {
  int32_t tok;     // absolute token index
  float s;         // score (mid tokens); anchors: filled in before processing
  int32_t gl;      // query head within the group
};

// Generic (any storage type) pair processing: one pair at a time, whole workgroup.
// Threads c < d own value channel c of the accumulators; threads j < dphi evaluate
// feature j of the gathered key.
template <typename T>
struct GatherAcc {
  float nu[kMaxGroup];     // per query head of the group, this thread's channel
  float zv[kMaxGroup];
  float m[kMaxGroup], Z[kMaxGroup], zsum[kMaxGroup];   // uniform across threads
  int cnt[kMaxGroup];
};

// grid (n_sel_slices + 1, Hkv, n_problems); slice index n_sel_slices is the anchor set
template <typename T>
__global__ __launch_bounds__(kThreads) void gather_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                          char* __restrict__ ws) {
  __shared__ Pair queue[kPairCap];
  __shared__ float kf[kMaxDim];
  __shared__ float qf[kMaxGroup][kMaxDim];
  __shared__ float red_f[4];
  __shared__ int red_i[4];
  __shared__ int sh_fill;
  __shared__ int sh_emitted[kMaxGroup];

  const int sl = blockIdx.x, h = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int n_slices = (n + g.sel_chunk - 1) / g.sel_chunk;
  const bool is_anchor = (sl == g.n_sel_slices);
  if (!is_anchor && sl >= n_slices) return;
  const int G = g.G, d = g.d, dphi = g.dphi;
  char* blk = problem_block(g, ws, p);

  GatherAcc<T> acc;
#pragma unroll
  for (int gl = 0; gl < kMaxGroup; ++gl) {
    acc.nu[gl] = 0.f; acc.zv[gl] = 0.f; acc.m[gl] = -INFINITY; acc.Z[gl] = 0.f; acc.zsum[gl] = 0.f; acc.cnt[gl] = 0;
  }
  if (tid == 0) sh_fill = 0;
  if (tid < kMaxGroup) sh_emitted[tid] = 0;
  for (int i = tid; i < G * d; i += kThreads)
    qf[i / d][i % d] = Elem<T>::load1(pr.q, (int64_t)(h * G + i / d) * d + (i % d));
  __syncthreads();

  const int64_t head_off = (int64_t)h * pr.stride_head;
  const float* phiq = (const float*)(blk + g.off_phiq);

  // processes queue[0 .. fill): one pair at a time
  auto flush = [&](int fill) {
    for (int e = 0; e < fill; ++e) {
      const Pair pe = queue[e];
      const int64_t row_off = head_off + (int64_t)pe.tok * pr.stride_tok;
      __syncthreads();                       // previous pair's readers of kf are done
      if (tid < d) kf[tid] = Elem<T>::load1(pr.K, row_off + tid);
      const float vc = tid < d ? Elem<T>::load1(pr.V, row_off + tid) : 0.f;
      __syncthreads();
      float s = pe.s;
      float z = 0.f;
      if (is_anchor) {
        float part = 0.f;
        if (tid < d) part = kf[tid] * qf[pe.gl][tid];
        s = block_sum(part, red_f) * g.score_scale + 0.0f;
      } else {
        float zj = 0.f;
        if (tid < dphi) {
          float dot = 0.f, nrm = 0.f;
          const int64_t wbase = ((int64_t)h * dphi + tid) * d;
          for (int c = 0; c < d; ++c) {
            const float x = kf[c];
            dot = fmaf(Elem<T>::load1(pr.Wk, wbase + c), x, dot);
            nrm = fmaf(x, x, nrm);
          }
          const float f = expf(g.a * dot - g.c * nrm + pr.bk[(int64_t)h * dphi + tid]);
          zj = f * phiq[(size_t)(h * G + pe.gl) * dphi + tid];
        }
        z = block_sum(zj, red_f);
      }
#pragma unroll
      for (int gl = 0; gl < kMaxGroup; ++gl) {
        if (gl == pe.gl) {
          const float m_new = fmaxf(acc.m[gl], s);
          const float r = __expf(acc.m[gl] - m_new);     // exp(-inf) = 0 on the first pair
          const float w = __expf(s - m_new);
          acc.nu[gl] = acc.nu[gl] * r + w * vc;
          acc.Z[gl] = acc.Z[gl] * r + w;
          acc.m[gl] = m_new;
          acc.zsum[gl] += z;
          acc.zv[gl] = fmaf(z, vc, acc.zv[gl]);
          acc.cnt[gl] += 1;
        }
      }
    }
    __syncthreads();
  };

  if (is_anchor) {
    // anchors: [0, n_sink) and [L - n_tail, L), or every token when the mid-region is empty
    const int n_anchor = n > 0 ? g.n_sink + g.n_tail : pr.L;
    const int total = n_anchor * G;
    for (int base = 0; base < total; base += kPairCap) {
      const int cnt = min(kPairCap, total - base);
      for (int i = tid; i < cnt; i += kThreads) {
        const int e = base + i;
        const int a = e / G;
        const int tok = (n > 0 && a >= g.n_sink) ? (pr.L - g.n_tail + (a - g.n_sink)) : a;
        queue[i].tok = tok; queue[i].s = 0.f; queue[i].gl = e % G;
      }
      __syncthreads();
      flush(cnt);
    }
  } else {
    const int t0 = sl * g.sel_chunk, t1 = min(n, t0 + g.sel_chunk);
    const float* scores = (const float*)(blk + g.off_scores);
    const HeadState* st = (const HeadState*)(blk + g.off_state);
    const int32_t* offsets = (const int32_t*)(blk + g.off_offsets);
    for (int base = t0; base < t1; base += kThreads) {
      if (sh_fill + kThreads * G > kPairCap) {
        const int fill = sh_fill;
        flush(fill);
        if (tid == 0) sh_fill = 0;
        __syncthreads();
      }
      const int row = base + tid;
      for (int gl = 0; gl < G; ++gl) {
        const int gq = h * G + gl;
        bool sel = false;
        float s = 0.f;
        if (row < t1) {
          s = scores[(size_t)gq * g.mid_stride + row];
          const uint32_t key = score_key(s);
          const uint32_t tk = st[gq].thr_key;
          sel = key > tk || (key == tk && row <= st[gq].thr_idx);
        }
        const int incl = block_scan_incl(sel ? 1 : 0, red_i);
        const int fill = sh_fill;
        const int emitted = sh_emitted[gl];
        if (sel) {
          const int pos = fill + incl - 1;
          queue[pos].tok = g.n_sink + row; queue[pos].s = s; queue[pos].gl = gl;
          if (pr.topk_idx)
            pr.topk_idx[(size_t)gq * g.max_K + offsets[(size_t)gq * g.n_sel_slices + sl] + emitted + incl - 1] = g.n_sink + row;
        }
        __syncthreads();
        if (tid == kThreads - 1) { sh_fill = fill + incl; sh_emitted[gl] = emitted + incl; }
        __syncthreads();
      }
    }
    const int fill = sh_fill;
    flush(fill);
  }

  // write the partial: [m, Z, zsum, count, nu[d], zv[d]] per query head of the group
  float* part = (float*)(blk + g.off_part) + ((size_t)(h * (g.n_sel_slices + 1) + sl) * G) * g.part_stride;
#pragma unroll
  for (int gl = 0; gl < kMaxGroup; ++gl) {
    if (gl < G) {
      float* pp = part + (size_t)gl * g.part_stride;
      if (tid == 0) { pp[0] = acc.m[gl]; pp[1] = acc.Z[gl]; pp[2] = acc.zsum[gl]; pp[3] = (float)acc.cnt[gl]; }
      if (tid < d) { pp[4 + tid] = acc.nu[gl]; pp[4 + d + tid] = acc.zv[gl]; }
    }
  }
}

// grid (Hq, n_problems)
__global__ __launch_bounds__(kThreads) void merge_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                         char* __restrict__ ws, int mode) {
  const int gq = blockIdx.x, p = blockIdx.y, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int n_slices = (n + g.sel_chunk - 1) / g.sel_chunk;
  const int Ksel = max(0, min(min(pr.topk, n), g.max_K));
  const int G = g.G, d = g.d, dphi = g.dphi;
  const int h = gq / G, gl = gq % G;
  char* blk = problem_block(g, ws, p);
  const float* part0 = (const float*)(blk + g.off_part) + ((size_t)(h * (g.n_sel_slices + 1)) * G + gl) * g.part_stride;
  const size_t slice_step = (size_t)G * g.part_stride;

  // shift m = max over the exact support (anchor partial + slice partials)
  float m = part0[(size_t)g.n_sel_slices * slice_step];
  for (int s = 0; s < n_slices; ++s) m = fmaxf(m, part0[s * slice_step]);
  const bool empty_E = !(m > -INFINITY);
  if (empty_E) m = 0.f;

  float nu = 0.f, zv = 0.f, Z = 0.f, zsum = 0.f;
  const int c = tid;
  auto add_part = [&](const float* pp) {
    const float ml = pp[0];
    if (ml > -INFINITY) {
      const float r = __expf(ml - m);
      Z = fmaf(r, pp[1], Z);
      if (c < d) nu = fmaf(r, pp[4 + c], nu);
    }
    zsum += pp[2];
    if (c < d) zv += pp[4 + d + c];
  };
  add_part(part0 + (size_t)g.n_sel_slices * slice_step);      // anchors first
  for (int s = 0; s < n_slices; ++s) add_part(part0 + s * slice_step);

  // residual branch from the summaries
  float nuR = 0.f, ZR = 0.f;
  bool clamped = false;
  // (with every mid token retrieved in SUB mode the residual set is empty: exactly zero)
  if (mode != TKPHI_MODE_TOPK_ONLY && n > 0 && !(mode == TKPHI_MODE_SUB && Ksel == n)) {
    const float* phiq = (const float*)(blk + g.off_phiq) + (size_t)gq * dphi;
    const float* S = pr.S + (size_t)h * dphi * d;
    const float* u = pr.u + (size_t)h * dphi;
    float accn = 0.f, accz = 0.f;
    for (int j = 0; j < dphi; ++j) {
      const float pj = phiq[j];
      accz = fmaf(pj, u[j], accz);
      if (c < d) accn = fmaf(pj, S[(size_t)j * d + c], accn);
    }
    if (mode == TKPHI_MODE_SUB) { accn -= zv; accz -= zsum; }
    nuR = accn; ZR = accz;
    if (!(ZR > 0.f)) {                     // numerical clamp: drop the residual branch
      clamped = true;
      nuR = 0.f; ZR = 0.f;
    }
  }
  // y = (nu_E + exp(-m) nu_R) / (Z_E + exp(-m) Z_R), evaluated with the common shift max(m, 0)
  const float ms = fmaxf(m, 0.f);
  const float eE = __expf(m - ms), eR = __expf(-ms);
  const float den = eE * Z + eR * ZR;
  if (c < d) pr.out[(size_t)gq * d + c] = (eE * nu + eR * nuR) / den;
  if (pr.aux) {
    float* ax = pr.aux + (size_t)gq * TKPHI_AUX_STRIDE(d);
    if (tid == 0) { ax[0] = m; ax[1] = Z; ax[2] = ZR; ax[3] = clamped ? 1.f : 0.f; }
    if (c < d) { ax[4 + c] = nu; ax[4 + d + c] = nuR; }
  }
  if (clamped && tid == 0) atomicOr((uint32_t*)(ws + g.off_status), TKPHI_DEV_CLAMPED);
}

void launch_gather(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  dim3 grid(g.n_sel_slices + 1, g.Hkv, g.n_problems);
  if (g.dtype == TKPHI_BF16)
    hipLaunchKernelGGL(gather_kernel<uint16_t>, grid, dim3(kThreads), 0, s, g, probs, ws);
  else
    hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(kThreads), 0, s, g, probs, ws);
}

void launch_merge(const Geom& g, const tkphi_problem* probs, char* ws, int mode, hipStream_t s) {
  dim3 grid(g.Hq, g.n_problems);
  hipLaunchKernelGGL(merge_kernel, grid, dim3(kThreads), 0, s, g, probs, ws, mode);
}

}  // namespace tkphi
