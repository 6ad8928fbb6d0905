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
#include "block_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
union Frag {
  u32x4 u;
  bf16x8 v;
};

// ---- anchors: exact terms over [0, n_sink) u [L - n_tail, L) (or every token if M is empty) --------
// Whole workgroup; thread c < d owns value channel c.  Writes the partial of the anchor slot.
template <typename T>
__device__ void anchor_partial(const Geom& g, const tkphi_problem& pr, int gq, int n, float* part) {
  __shared__ float a_q[kMaxDim];
  __shared__ float a_s[kThreads];
  __shared__ float a_red[4];
  const int tid = threadIdx.x, d = g.d;
  const int h = gq / g.G;
  const int n_anchor = n > 0 ? g.n_sink + g.n_tail : pr.L;
  const int64_t head_off = (int64_t)h * pr.stride_head;
  for (int c = tid; c < d; c += kThreads) a_q[c] = Elem<T>::load1(pr.q, (int64_t)gq * d + c);
  __syncthreads();
  float m = -INFINITY, Z = 0.f, nu = 0.f;
  for (int base = 0; base < n_anchor; base += kThreads) {
    const int cnt = min(kThreads, n_anchor - base);
    // one anchor score per thread
    float s = -INFINITY;
    if (tid < cnt) {
      const int a = base + tid;
      const int tok = (n > 0 && a >= g.n_sink) ? (pr.L - g.n_tail + (a - g.n_sink)) : a;
      float dot = 0.f;
      const int64_t off = head_off + (int64_t)tok * pr.stride_tok;
      for (int c = 0; c < d; ++c) dot = fmaf(Elem<T>::load1(pr.K, off + c), a_q[c], dot);
      s = dot * g.score_scale + 0.0f;
    }
    a_s[tid] = s;
    const float mb = block_max(s, a_red);          // barriers inside: a_s is visible afterwards
    const float m_new = fmaxf(m, mb);
    const float r = __expf(m - m_new);             // exp(-inf) = 0 on the first batch
    nu *= r; Z *= r; m = m_new;
    for (int i = 0; i < cnt; ++i) {
      const int a = base + i;
      const int tok = (n > 0 && a >= g.n_sink) ? (pr.L - g.n_tail + (a - g.n_sink)) : a;
      const float w = __expf(a_s[i] - m);
      Z += w;
      if (tid < d) nu = fmaf(w, Elem<T>::load1(pr.V, head_off + (int64_t)tok * pr.stride_tok + tid), nu);
    }
    __syncthreads();
  }
  if (tid == 0) { part[0] = m; part[1] = Z; part[2] = 0.f; part[3] = (float)n_anchor; }
  if (tid < d) { part[4 + tid] = nu; part[4 + d + tid] = 0.f; }
}

// ------------------------------------------------------------------------------------
// gather, bf16 on the matrix cores: grid (n_tiles + 1, Hq, n_problems); D == d_head == d_phi.
// Wavefront w owns 16 retrieved tokens: their key rows are the A operand (lane (r, kg): token
// r, 8 consecutive channels per k-step), Wk of the KV head is staged once per workgroup in
// LDS (rows padded by 16 B: conflict-free ds_read_b128) and provides the B operand per
// 16-feature tile.
// ------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kThreads) void gather_mfma_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                               char* __restrict__ ws) {
  constexpr int KS = D / 32, NT = D / 16;
  constexpr int WROW = D * 2 + 16;                 // bytes per staged Wk row
  __shared__ __attribute__((aligned(16))) char wk_lds[D * WROW];
  __shared__ int p_tok[kPairsPerWG];
  __shared__ float p_s[kPairsPerWG], p_w[kPairsPerWG], p_z[kPairsPerWG];
  __shared__ float red[kThreads / D][2 * D];
  __shared__ float sh_m;

  const int tile = blockIdx.x, gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  char* blk = problem_block(g, ws, p);
  float* part = (float*)(blk + g.off_part) + ((size_t)gq * (g.n_tiles + 1) + tile) * g.part_stride;
  if (tile == g.n_tiles) { anchor_partial<uint16_t>(g, pr, gq, n, part); return; }
  const int Ksel = ((const int32_t*)(blk + g.off_nsel))[gq];
  const int i0 = tile * kPairsPerWG;
  if (i0 >= Ksel) return;
  const int cnt = min(kPairsPerWG, Ksel - i0);
  const int h = gq / g.G;
  const int lane = tid & 63, wv = tid >> 6, r = lane & 15, kg = lane >> 4;

  // the tile's retrieved tokens
  if (tid < kPairsPerWG) {
    const int i = i0 + min(tid, cnt - 1);
    p_tok[tid] = g.n_sink + ((const int32_t*)(blk + g.off_selidx))[(size_t)gq * g.max_K + i];
    p_s[tid] = tid < cnt ? ((const float*)(blk + g.off_selscore))[(size_t)gq * g.max_K + i] : -INFINITY;
  }
  // stage Wk[h] ([D features][D channels] bf16) with padded rows
  {
    const char* wsrc = (const char*)pr.Wk + (size_t)h * D * D * 2;
    constexpr int SEGS = D * 2 / 16;               // 16-byte segments per row
    for (int i = tid; i < D * SEGS; i += kThreads) {
      const int row = i / SEGS, seg = i % SEGS;
      *(u32x4*)(wk_lds + row * WROW + seg * 16) = *(const u32x4*)(wsrc + (size_t)row * D * 2 + seg * 16);
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
    for (int j = 0; j < KS; ++j) a[j].u = *(const u32x4*)(rp + j * 64);
    // |k|^2 of token r: this lane's 8*KS channels, then the 4 lanes of the row
    float nrm = 0.f;
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      float x[8];
      Elem<uint16_t>::unpack(*(const uint4*)&a[j].u, x);
#pragma unroll
      for (int e = 0; e < 8; ++e) nrm = fmaf(x[e], x[e], nrm);
    }
    nrm += __shfl_xor(nrm, 16);
    nrm += __shfl_xor(nrm, 32);
    float nr[4];                                   // |k|^2 of tokens 4kg + i
#pragma unroll
    for (int i = 0; i < 4; ++i) nr[i] = __shfl(nrm, 4 * kg + i);

    const float* phiq = (const float*)(blk + g.off_phiq) + (size_t)gq * D;
    const float* bk = pr.bk + (size_t)h * D;
    float zacc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
    for (int nt = 0; nt < NT; ++nt) {
      floatx4 acc = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < KS; ++j) {
        Frag b;
        b.u = *(const u32x4*)(wk_lds + (nt * 16 + r) * WROW + j * 64 + kg * 16);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j].v, b.v, acc, 0, 0, 0);
      }
      // acc[i] = Wk[feature nt*16 + r] . k(token 4kg + i)
      const float bj = bk[nt * 16 + r], pj = phiq[nt * 16 + r];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float f = __expf(g.a * acc[i] - g.c * nr[i] + bj);
        uint32_t hi, lo;
        split_bf16(f, &hi, &lo);             // the 16 bits the summary build contracted
        zacc[i] = fmaf(join_bf16(hi, lo), pj, zacc[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int o = 8; o >= 1; o >>= 1) zacc[i] += __shfl_xor(zacc[i], o);
    }
    if (r == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) p_z[wv * 16 + 4 * kg + i] = zacc[i];
    }
  }
  __syncthreads();
  if (tid < kPairsPerWG) p_w[tid] = tid < cnt ? __expf(p_s[tid] - sh_m) : 0.f;
  __syncthreads();

  // value accumulation: thread (c = tid % D, grp = tid / D) takes tokens grp, grp + NG, ...
  constexpr int NG = kThreads / D;
  const int c = tid % D, grp = tid / D;
  float nu = 0.f, zv = 0.f;
  for (int i = grp; i < cnt; i += NG) {
    const float v = bf16_bits_to_float(((const uint16_t*)pr.V)[head_off + (int64_t)p_tok[i] * pr.stride_tok + c]);
    nu = fmaf(p_w[i], v, nu);
    zv = fmaf(p_z[i], v, zv);
  }
  red[grp][c] = nu; red[grp][D + c] = zv;
  __syncthreads();
  if (tid < D) {
    float a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int k = 0; k < NG; ++k) { a0 += red[k][tid]; a1 += red[k][D + tid]; }
    part[4 + tid] = a0; part[4 + D + tid] = a1;
  }
  if (tid == 0) {
    float Z = 0.f, zs = 0.f;
    for (int i = 0; i < cnt; ++i) { Z += p_w[i]; zs += p_z[i]; }
    part[0] = sh_m; part[1] = Z; part[2] = zs; part[3] = (float)cnt;
  }
}

// ------------------------------------------------------------------------------------
// gather, generic (any storage type, fp32 arithmetic): same grid; one retrieved token at a
// time, threads j < dphi evaluate feature j, threads c < d own value channel c.
// ------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void gather_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                          char* __restrict__ ws) {
  __shared__ float kf[kMaxDim];
  __shared__ float red_f[4];
  const int tile = blockIdx.x, gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  char* blk = problem_block(g, ws, p);
  float* part = (float*)(blk + g.off_part) + ((size_t)gq * (g.n_tiles + 1) + tile) * g.part_stride;
  if (tile == g.n_tiles) { anchor_partial<T>(g, pr, gq, n, part); return; }
  const int Ksel = ((const int32_t*)(blk + g.off_nsel))[gq];
  const int i0 = tile * kPairsPerWG;
  if (i0 >= Ksel) return;
  const int cnt = min(kPairsPerWG, Ksel - i0);
  const int h = gq / g.G, d = g.d, dphi = g.dphi;
  const int32_t* sel_idx = (const int32_t*)(blk + g.off_selidx) + (size_t)gq * g.max_K + i0;
  const float* sel_s = (const float*)(blk + g.off_selscore) + (size_t)gq * g.max_K + i0;
  const float* phiq = (const float*)(blk + g.off_phiq) + (size_t)gq * dphi;
  const int64_t head_off = (int64_t)h * pr.stride_head;

  float m = -INFINITY;
  for (int i = 0; i < cnt; ++i) m = fmaxf(m, sel_s[i]);
  float nu = 0.f, zv = 0.f, Z = 0.f, zsum = 0.f;
  for (int i = 0; i < cnt; ++i) {
    const int64_t row_off = head_off + (int64_t)(g.n_sink + sel_idx[i]) * pr.stride_tok;
    __syncthreads();                       // the previous token's readers of kf are done
    if (tid < d) kf[tid] = Elem<T>::load1(pr.K, row_off + tid);
    const float vc = tid < d ? Elem<T>::load1(pr.V, row_off + tid) : 0.f;
    __syncthreads();
    float zj = 0.f;
    if (tid < dphi) {
      float dot = 0.f, nrm = 0.f;
      const int64_t wbase = ((int64_t)h * dphi + tid) * d;
      for (int c = 0; c < d; ++c) {
        const float x = kf[c];
        dot = fmaf(Elem<T>::load1(pr.Wk, wbase + c), x, dot);
        nrm = fmaf(x, x, nrm);
      }
      zj = expf(g.a * dot - g.c * nrm + pr.bk[(int64_t)h * dphi + tid]) * phiq[tid];
    }
    const float z = block_sum(zj, red_f);
    const float w = __expf(sel_s[i] - m);
    nu = fmaf(w, vc, nu); Z += w;
    zv = fmaf(z, vc, zv); zsum += z;
  }
  if (tid == 0) { part[0] = m; part[1] = Z; part[2] = zsum; part[3] = (float)cnt; }
  if (tid < d) { part[4 + tid] = nu; part[4 + d + tid] = zv; }
}

// ------------------------------------------------------------------------------------
// merge: grid (Hq, n_problems)
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void merge_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                         char* __restrict__ ws, int mode) {
  __shared__ float red_f[4];
  const int gq = blockIdx.x, p = blockIdx.y, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int Ksel = max(0, min(min(pr.topk, n), g.max_K));
  const int n_used = (Ksel + kPairsPerWG - 1) / kPairsPerWG;     // tiles holding retrieved tokens
  const int d = g.d, dphi = g.dphi;
  const int h = gq / g.G;
  char* blk = problem_block(g, ws, p);
  const float* part0 = (const float*)(blk + g.off_part) + (size_t)gq * (g.n_tiles + 1) * g.part_stride;
  const float* anchor = part0 + (size_t)g.n_tiles * g.part_stride;

  // shift m = max over the exact support (anchor partial + tile partials)
  float ml = tid == 0 ? anchor[0] : -INFINITY;
  for (int t = tid; t < n_used; t += kThreads) ml = fmaxf(ml, part0[(size_t)t * g.part_stride]);
  float m = block_max(ml, red_f);
  const bool empty_E = !(m > -INFINITY);
  if (empty_E) m = 0.f;

  float nu = 0.f, zv = 0.f, Z = 0.f, zsum = 0.f;
  const int c = tid;
  auto add_part = [&](const float* pp) {
    const float mp = pp[0];
    if (mp > -INFINITY) {
      const float r = __expf(mp - m);
      Z = fmaf(r, pp[1], Z);
      if (c < d) nu = fmaf(r, pp[4 + c], nu);
    }
    zsum += pp[2];
    if (c < d) zv += pp[4 + d + c];
  };
  add_part(anchor);                                    // anchors first, then the tiles in order
  for (int t = 0; t < n_used; ++t) add_part(part0 + (size_t)t * g.part_stride);

  // residual branch from the summaries
  // (with every mid token retrieved in SUB mode the residual set is empty: exactly zero)
  float nuR = 0.f, ZR = 0.f;
  bool clamped = false;
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
  dim3 grid(g.n_tiles + 1, g.Hq, g.n_problems);
  if (g.use_mfma) {
    if (g.d == 128) hipLaunchKernelGGL(gather_mfma_kernel<128>, grid, dim3(kThreads), 0, s, g, probs, ws);
    else hipLaunchKernelGGL(gather_mfma_kernel<64>, grid, dim3(kThreads), 0, s, g, probs, ws);
  } else if (g.dtype == TKPHI_BF16) {
    hipLaunchKernelGGL(gather_kernel<uint16_t>, grid, dim3(kThreads), 0, s, g, probs, ws);
  } else {
    hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(kThreads), 0, s, g, probs, ws);
  }
}

void launch_merge(const Geom& g, const tkphi_problem* probs, char* ws, int mode, hipStream_t s) {
  dim3 grid(g.Hq, g.n_problems);
  hipLaunchKernelGGL(merge_kernel, grid, dim3(kThreads), 0, s, g, probs, ws, mode);
}

}  // namespace tkphi
