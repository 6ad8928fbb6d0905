// The phi and anchor jobs of the filtered pipeline's prep stage as 256-thread workgroups, for batches: with many
// (problem, head) pairs in a call the jobs are throughput work, and small workgroups (eight per CU) run them four
// times as densely as the 1024-thread ones that a single layer uses for the shortest latency.
//   phi job     phi_q(q) of a query head (App. "Head-wise phi architecture": per query head, once per step)
//               and the summary terms S_M^T phi_q, phi_q . u_M that eq. (subtraction) and eq. (hybrid_merge)
//               start from
//   anchor job  the exact terms of eq. (exact_terms) over a tile of 64 anchors (sink, tail, generated tokens
//               of eq. (implemented_decode))
#pragma once

#include "tkphi_internal.h"

namespace tkphi {

// ---- phi job: one workgroup per query head ----------------------------------------------------------------
// phi_q -> workspace; sphi[c] = sum_j phi_q[j] S[h][j][c]; uphi = sum_j phi_q[j] u[h][j].  Sums run in a fixed
// order.    LDS: sh_phiq, pu [kMaxDim], red [1024]
__device__ __forceinline__ void side_phi(const Geom& g, const tkphi_problem& pr, char* blk, int gq, float* sh_phiq, float* pu,
                                         float* red) {
  const int tid = threadIdx.x, d = g.d, dphi = g.dphi, h = gq / g.G;
  const bool act = tid < kThreads;
  // rows of Wq: LPR lanes per row (16 bytes each), rows_pp rows per pass, 8 passes in flight
  const int LPR = d / 8, seg = tid % LPR, row_in = tid / LPR, rows_pp = kThreads / LPR;
  const u32x4 qv = gload128((const char*)pr.q + ((size_t)gq * d + seg * 8) * 2);
  float qx[8];
  Elem<uint16_t>::unpack(make_uint4(qv.x, qv.y, qv.z, qv.w), qx);
  float nrm = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) nrm = fmaf(qx[e], qx[e], nrm);
  for (int o = LPR >> 1; o >= 1; o >>= 1) nrm += __shfl_xor(nrm, o);
  float* phiq = (float*)(blk + g.off_phiq) + (size_t)gq * dphi;
  constexpr int MAXP = 8;
  for (int j0 = 0; j0 < dphi; j0 += rows_pp * MAXP) {
    u32x4 wv[MAXP];
    float bj[MAXP];
#pragma unroll
    for (int k = 0; k < MAXP; ++k) {
      if (j0 + k * rows_pp >= dphi) break;            // (uniform)
      const int j = min(j0 + k * rows_pp + row_in, dphi - 1);
      wv[k] = gload128((const char*)pr.Wq + (((size_t)gq * dphi + j) * d + seg * 8) * 2);
      bj[k] = pr.bq[(size_t)gq * dphi + j];
    }
#pragma unroll
    for (int k = 0; k < MAXP; ++k) {
      if (j0 + k * rows_pp >= dphi) break;
      const int jr = j0 + k * rows_pp + row_in;
      float x[8];
      Elem<uint16_t>::unpack(make_uint4(wv[k].x, wv[k].y, wv[k].z, wv[k].w), x);
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(x[e], qx[e], dot);
      for (int o = LPR >> 1; o >= 1; o >>= 1) dot += __shfl_xor(dot, o);
      if (act && jr < dphi && seg == 0) {
        const float f = expf(g.a * dot - g.c * nrm + bj[k]);
        phiq[jr] = f;
        sh_phiq[jr] = f;
      }
    }
  }
  __syncthreads();
  // S^T phi_q: thread (jg, c4) takes the features of group jg for 4 value channels, 8 rows of S in flight
  const int QPR = d / 4, NG = kThreads / QPR;         // float4 per row of S; feature groups (8 for d = 128, 16 for d = 64)
  const int jg = tid / QPR, c4 = tid % QPR;
  const int per = (dphi + NG - 1) / NG, j0 = jg * per, j1 = min(dphi, j0 + per);
  const float* __restrict__ S = pr.S + (size_t)h * dphi * d;
  float4 sacc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int jb = j0; jb < j1; jb += 8) {
    u32x4 sv[8];
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (jb + k < j1) sv[k] = gload128(S + (size_t)(jb + k) * d + c4 * 4);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if (jb + k < j1) {
        const float pj = sh_phiq[jb + k];
        sacc.x = fmaf(pj, __uint_as_float(sv[k].x), sacc.x); sacc.y = fmaf(pj, __uint_as_float(sv[k].y), sacc.y);
        sacc.z = fmaf(pj, __uint_as_float(sv[k].z), sacc.z); sacc.w = fmaf(pj, __uint_as_float(sv[k].w), sacc.w);
      }
    }
  }
  if (act) *(float4*)(red + jg * d + c4 * 4) = sacc;  // NG d = 1024 floats
  for (int j = tid; j < dphi && act; j += kThreads) pu[j] = sh_phiq[j] * pr.u[(size_t)h * dphi + j];
  __syncthreads();
  if (tid < d) {
    float a = 0.f;
    for (int k = 0; k < NG; ++k) a += red[k * d + tid];
    ((float*)(blk + g.off_sphi))[(size_t)gq * d + tid] = a;
  } else if (tid == kThreads - 64) {
    float a = 0.f;
    for (int j = 0; j < dphi; ++j) a += pu[j];      // feature order
    ((float*)(blk + g.off_uphi))[gq] = a;
  }
}

// ---- anchor job: one workgroup per (query head, tile of 64 anchors) -------------------------------------------
// Anchors are the rows [0, n_sink) u [L - n_tail, L) (every row if the mid-region is empty) followed by the
// generated tokens [L, L + n_gen).  Writes the tile's partial in the layout of the gather kernels:
// [m_loc, Z_loc, 0, count, nu_loc[d], 0[d]].  LDS: a_s, a_w [64], red [4][128]
__device__ __forceinline__ void side_anchor(const Geom& g, const tkphi_problem& pr, char* blk, int gq, int batch, float* a_s,
                                            float* a_w, float* red) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, d = g.d, h = gq / g.G;
  const bool act = tid < kThreads;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int n_prefill = n > 0 ? g.n_sink + g.n_tail : pr.L;
  const int n_anchor = n_prefill + min(max(pr.n_gen, 0), g.max_gen);
  const int base = batch * 64;
  if (base >= n_anchor) return;
  const int cnt = min(64, n_anchor - base);
  float* part = (float*)(blk + g.off_part) + ((size_t)gq * (g.n_tiles + g.n_atiles) + g.n_tiles + batch) * g.part_stride;
  const int LPR = d / 8, seg = tid % LPR, rsub = tid / LPR, RPP = kThreads / LPR;   // rows per pass: 16 (d = 128) or 32
  constexpr int MAXPS = 4;                           // 64 rows / 16
  const int n_pass = 64 / RPP;
  u32x4 kv[MAXPS], vv[MAXPS];
  const u32x4 qv = gload128((const char*)pr.q + ((size_t)gq * d + seg * 8) * 2);
#pragma unroll
  for (int ps = 0; ps < MAXPS; ++ps) {
    if (ps < n_pass) {
      const int a = base + min(ps * RPP + rsub, cnt - 1);
      const int tok = a >= n_prefill ? pr.L + (a - n_prefill) : (n > 0 && a >= g.n_sink) ? (pr.L - g.n_tail + (a - g.n_sink)) : a;
      const size_t off = ((size_t)h * pr.stride_head + (size_t)tok * pr.stride_tok + seg * 8) * 2;
      kv[ps] = gload128((const char*)pr.K + off);
      vv[ps] = gload128((const char*)pr.V + off);
    }
  }
  float qx[8];
  Elem<uint16_t>::unpack(make_uint4(qv.x, qv.y, qv.z, qv.w), qx);
#pragma unroll
  for (int ps = 0; ps < MAXPS; ++ps) {
    if (ps < n_pass) {
      float kx[8];
      Elem<uint16_t>::unpack(make_uint4(kv[ps].x, kv[ps].y, kv[ps].z, kv[ps].w), kx);
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s = fmaf(kx[e], qx[e], s);
      for (int o = LPR >> 1; o >= 1; o >>= 1) s += __shfl_xor(s, o);
      const int row = ps * RPP + rsub;
      if (act && seg == 0) a_s[row] = row < cnt ? s * g.score_scale + 0.0f : -INFINITY;
    }
  }
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
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
  for (int ps = 0; ps < MAXPS; ++ps) {
    if (ps < n_pass) {
      const int row = ps * RPP + rsub;
      const float w = row < cnt ? a_w[row] : 0.f;
      float vx[8];
      Elem<uint16_t>::unpack(make_uint4(vv[ps].x, vv[ps].y, vv[ps].z, vv[ps].w), vx);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(w, vx[e], acc[e]);
    }
  }
  // rows of one wavefront that share a segment: lanes seg, seg + LPR, ...
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], o);
  }
  if (act && lane < LPR) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wv * 128 + lane * 8 + e] = acc[e];
  }
  __syncthreads();
  if (tid < d) {
    part[4 + tid] = (red[tid] + red[128 + tid]) + (red[256 + tid] + red[384 + tid]);
    part[4 + d + tid] = 0.f;
  }
}

}  // namespace tkphi
