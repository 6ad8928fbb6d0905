// The merge of one query head (eq. (hybrid_merge)): the partials of the exact branch (anchor tiles, retrieved
// tiles) are combined under one max shift, the residual branch phi_q^T S_M, phi_q . u_M minus the retrieved
// tokens' share (eq. (subtraction)) is added under the same normalisation, with the numerical clamp of the
// residual denominator; optional exports (aux, diagnostics, the retrieved indices in ascending order).
// Written for kThreads = 256 threads, all of which must call it together (it contains workgroup barriers).
// Called by the merge kernel (one workgroup per head) and by the workgroup of the fused select + gather kernel
// that finishes a head last.
#pragma once

#include "block_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

// COHERENT: the retrieved-token partials were written (store_agent) by other workgroups of the running launch
template <bool PRE, bool COHERENT = false>   // PRE: S_M^T phi_q and phi_q . u_M come from the prep kernel (workspace), not from S, u
__device__ __forceinline__ void merge_head(const Geom& g, const tkphi_problem* __restrict__ probs, char* __restrict__ ws, int gq,
                                           int p, int mode) {
  __shared__ float red_f[4];
  __shared__ float sh_phiq[kMaxDim], sh_u[kMaxDim];
  __shared__ float sh_grp[9][128];                 // [feature group][value channel]; row 8: scalars of the partial combine
  const int tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int Ksel = max(0, min(min(pr.topk, n), g.max_K));
  const int n_anchor = (n > 0 ? g.n_sink + g.n_tail : pr.L) + min(max(pr.n_gen, 0), g.max_gen);   // anchors + generated tokens
  // partials holding retrieved tokens: tiles of 64, or (PRE) one per workgroup of the fused select + gather kernel
  const int n_used = PRE ? (Ksel > 0 ? g.n_tiles : 0) : (Ksel + kPairsPerWG - 1) / kPairsPerWG;
  const int na_used = (n_anchor + 63) / 64;                      // tiles holding anchors
  const int d = g.d, dphi = g.dphi;
  const int h = gq / g.G;
  char* blk = problem_block(g, ws, p);
  const float* part0 = (const float*)(blk + g.off_part) + (size_t)gq * (g.n_tiles + g.n_atiles) * g.part_stride;
  const bool use_res = mode != TKPHI_MODE_TOPK_ONLY && n > 0 && !(mode == TKPHI_MODE_SUB && Ksel == n);
  // partial k of this head, in combination order: anchor tiles first, then the retrieved tiles
  const int n_parts = na_used + n_used;
  auto ldp = [](const float* q) { return COHERENT ? load_agent(q) : *q; };
  auto part_ptr = [&](int k) { return part0 + (size_t)(k < na_used ? g.n_tiles + k : k - na_used) * g.part_stride; };

  // ---- residual branch: S^T phi_q and u . phi_q, all loads of S issued together --------------
  // thread (jg = tid / (d/4), c4 = tid % (d/4)) takes the features of group jg for 4 value channels
  float4 sacc = make_float4(0.f, 0.f, 0.f, 0.f);
  const int QPR = d / 4, NG = kThreads / QPR;      // float4 per row; feature groups (8 for d=128, 16 for d=64)
  const int jg = tid / QPR, c4 = tid % QPR;
  float pre_n = 0.f, pre_z = 0.f;
  if (PRE && use_res) {
    pre_z = ((const float*)(blk + g.off_uphi))[gq];
    if (tid < d) pre_n = ((const float*)(blk + g.off_sphi))[(size_t)gq * d + tid];
  }
  if (!PRE && use_res) {
    const float* phiq = (const float*)(blk + g.off_phiq) + (size_t)gq * dphi;
    for (int j = tid; j < dphi; j += kThreads) { sh_phiq[j] = phiq[j]; sh_u[j] = pr.u[(size_t)h * dphi + j]; }
    const float* __restrict__ S = pr.S + (size_t)h * dphi * d;
    const int per = (dphi + NG - 1) / NG;          // features per group (<= 32)
    const int j0 = jg * per, j1 = min(dphi, j0 + per);
    constexpr int MAXF = 32;
    float4 sv[MAXF];
#pragma unroll
    for (int k = 0; k < MAXF; ++k)
      if (j0 + k < j1) sv[k] = *(const float4*)(S + (size_t)(j0 + k) * d + c4 * 4);
    __syncthreads();                               // phi_q staged
#pragma unroll
    for (int k = 0; k < MAXF; ++k) {
      if (j0 + k < j1) {
        const float pj = sh_phiq[j0 + k];
        sacc.x = fmaf(pj, sv[k].x, sacc.x); sacc.y = fmaf(pj, sv[k].y, sacc.y);
        sacc.z = fmaf(pj, sv[k].z, sacc.z); sacc.w = fmaf(pj, sv[k].w, sacc.w);
      }
    }
  }

  // ---- shift m = max over the exact support (all partial headers) ------------------------------
  // kThreads / d thread groups (2 for d = 128, 4 for d = 64) take the batches of UN partials round-robin,
  // thread c of a group one value channel; the group sums are then added in group order.  The first batch
  // of every group is requested before the shift is worked out: one memory round trip for both.
  const int NGRP = kThreads / d, grp = tid / d, c = tid % d;
  constexpr int UN = 16;
  float hm[UN], hz[UN], hs[UN], vn[UN], vz[UN];
  auto load_batch = [&](int t0) {
#pragma unroll
    for (int k = 0; k < UN; ++k) {
      const float* pp = part_ptr(min(t0 + k, n_parts - 1));
      hm[k] = ldp(pp); hz[k] = ldp(pp + 1); hs[k] = ldp(pp + 2);
      vn[k] = ldp(pp + 4 + c);
      vz[k] = ldp(pp + 4 + d + c);
    }
  };
  // At most UN partials (the usual case: a dozen): every thread takes all of them, finds the shift itself and
  // needs no exchange with other threads; the sums are those of group 0 of the general scheme, bit for bit.
  const bool few = n_parts <= UN;
  float m = -INFINITY;
  if (few) {
    load_batch(0);
#pragma unroll
    for (int k = 0; k < UN; ++k)
      if (k < n_parts) m = fmaxf(m, hm[k]);
  } else {
    if (grp * UN < n_parts) load_batch(grp * UN);
    float ml = -INFINITY;
    for (int k = tid; k < n_parts; k += kThreads) ml = fmaxf(ml, ldp(part_ptr(k)));
    m = block_max(ml, red_f);
  }
  const bool empty_E = !(m > -INFINITY);
  if (empty_E) m = 0.f;

  // ---- combine the partials in a fixed order ---------------------------------------------------
  float nu = 0.f, zv = 0.f, Z = 0.f, zsum = 0.f;
  float ZA = 0.f;                        // anchor share of Z (diagnostics only)
  const int first = few ? 0 : grp * UN;
  for (int t0 = first; t0 < n_parts; t0 += NGRP * UN) {
    if (t0 != first) load_batch(t0);
#pragma unroll
    for (int k = 0; k < UN; ++k) {
      if (t0 + k < n_parts) {
        const float r = __expf(hm[k] - m);
        Z = fmaf(r, hz[k], Z);
        if (t0 + k < na_used) ZA = fmaf(r, hz[k], ZA);
        nu = fmaf(r, vn[k], nu);
        zsum += hs[k];
        zv += vz[k];
      }
    }
  }
  if (!few) {
    // sh_grp is free until the residual sums below: [0] nu, [1] zv per (group, channel); [2] Z, zsum, ZA per group
    float* cmb = &sh_grp[0][0];
    __syncthreads();
    cmb[grp * 128 + c] = nu;
    cmb[512 + grp * 128 + c] = zv;
    if (c == 0) { cmb[1024 + grp * 4 + 0] = Z; cmb[1024 + grp * 4 + 1] = zsum; cmb[1024 + grp * 4 + 2] = ZA; }
    __syncthreads();
    nu = 0.f; zv = 0.f; Z = 0.f; zsum = 0.f; ZA = 0.f;
    for (int q = 0; q < NGRP; ++q) {
      nu += cmb[q * 128 + c]; zv += cmb[512 + q * 128 + c];
      Z += cmb[1024 + q * 4 + 0]; zsum += cmb[1024 + q * 4 + 1]; ZA += cmb[1024 + q * 4 + 2];
    }
    __syncthreads();                               // before sh_grp is reused
  }

  // (with every mid token retrieved in SUB mode the residual set is empty: exactly zero)
  float nuR = 0.f, ZR = 0.f;
  bool clamped = false;
  if (PRE && use_res) {
    float accn = pre_n, accz = pre_z;
    if (mode == TKPHI_MODE_SUB) { accn -= zv; accz -= zsum; }
    nuR = accn; ZR = accz;
    if (!(ZR > 0.f)) {                     // numerical clamp: drop the residual branch
      clamped = true;
      nuR = 0.f; ZR = 0.f;
    }
  }
  if (!PRE && use_res) {
    // fixed-order sum over the feature groups
    float* row = &sh_grp[0][0];
    if (jg < 8) { row[jg * 128 + c4 * 4 + 0] = sacc.x; row[jg * 128 + c4 * 4 + 1] = sacc.y;
                  row[jg * 128 + c4 * 4 + 2] = sacc.z; row[jg * 128 + c4 * 4 + 3] = sacc.w; }
    __syncthreads();
    if (jg >= 8) {                                 // d = 64: groups 8..15 add onto groups 0..7
      row[(jg - 8) * 128 + 64 + c4 * 4 + 0] = sacc.x; row[(jg - 8) * 128 + 64 + c4 * 4 + 1] = sacc.y;
      row[(jg - 8) * 128 + 64 + c4 * 4 + 2] = sacc.z; row[(jg - 8) * 128 + 64 + c4 * 4 + 3] = sacc.w;
    }
    float accz = 0.f;
    for (int j = 0; j < dphi; ++j) accz = fmaf(sh_phiq[j], sh_u[j], accz);
    __syncthreads();
    float accn = 0.f;
    if (c < d) {
      for (int k = 0; k < 8; ++k) accn += row[k * 128 + c];
      if (NG == 16) for (int k = 0; k < 8; ++k) accn += row[k * 128 + 64 + c];
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
  if (tid < d) pr.out[(size_t)gq * d + c] = (eE * nu + eR * nuR) / den;
  if (pr.aux) {
    float* ax = pr.aux + (size_t)gq * TKPHI_AUX_STRIDE(d);
    if (tid == 0) { ax[0] = m; ax[1] = Z; ax[2] = ZR; ax[3] = clamped ? 1.f : 0.f; }
    if (tid < d) { ax[4 + c] = nu; ax[4 + d + c] = nuR; }
  }
  if (clamped && tid == 0) atomicOr((uint32_t*)(ws + g.off_status), TKPHI_DEV_CLAMPED);

  // ---- optional diagnostics (Sec. "Analysis: entropy and completion gains"; App. "Entropy, mass
  // recovery, and residual-denominator diagnostics") from the per-chunk (max, sum e^(s-max),
  // sum (s-max) e^(s-max)) records written by the select emit pass ---------------------------------
  if (g.diag && pr.diag) {
    float* dg = pr.diag + (size_t)gq * TKPHI_DIAG_STRIDE;
    if (n == 0) {
      if (tid < TKPHI_DIAG_STRIDE) dg[tid] = 0.f;
    } else {
      const float4* rec = (const float4*)(blk + g.off_diag) + gq;          // + chunk * Hq
      const int n_chunks = (n + g.scan_chunk - 1) / g.scan_chunk;
      float lm = -INFINITY;
      for (int k = tid; k < n_chunks; k += kThreads) lm = fmaxf(lm, rec[(size_t)k * g.Hq].x);
      const float mM = block_max(lm, red_f);
      float lz = 0.f, lw = 0.f;
      for (int k = tid; k < n_chunks; k += kThreads) {
        const float4 rc = rec[(size_t)k * g.Hq];
        if (rc.y > 0.f) {
          const float r = __expf(rc.x - mM);
          lz = fmaf(r, rc.y, lz);
          lw = fmaf(r, rc.z + (rc.x - mM) * rc.y, lw);
        }
      }
      __syncthreads();
      const float ZM = block_sum(lz, red_f);
      __syncthreads();
      const float WM = block_sum(lw, red_f);
      if (tid == 0) {
        // masses relative to exp(mM): Z_M = ZM, Z_A = ZA e^(m-mM), Z_K = (Z - ZA) e^(m-mM)
        const float sh = empty_E ? 0.f : __expf(m - mM);
        const float zA = ZA * sh, zK = fmaxf(Z - ZA, 0.f) * sh;
        const float zR = ZM - zK;
        const float zRhat = ZR * __expf(-mM);                              // Z_R^ is unshifted
        dg[0] = n > 1 ? (__logf(ZM) - WM / ZM) / __logf((float)n) : 0.f;
        dg[1] = __logf(ZM) + mM;
        dg[2] = zK / ZM;
        dg[3] = den > 0.f ? eR * ZR / den : 0.f;
        dg[4] = zR / (zA + ZM);
        dg[5] = (ZR > 0.f && zR > 0.f) ? (__logf(ZR) - (__logf(zR) + mM)) : NAN;
        dg[6] = zA > 0.f ? __logf(zA) + mM : -INFINITY;
        dg[7] = 0.f;
        (void)zRhat;
      }
    }
  }

  // ---- optional export: retrieved token indices, ascending ---------------------------------------
  // The list is in emission order (chunk by chunk, then the boundary-bin winners): rank every
  // entry by counting the smaller ones, the list going through LDS in tiles.
  if (pr.topk_idx && Ksel > 0) {
    __shared__ int sh_win[1024];
    const int32_t* sel_idx = (const int32_t*)(blk + g.off_selidx) + (size_t)gq * g.max_K;
    int32_t* out = pr.topk_idx + (size_t)gq * g.max_K;
    for (int base = 0; base < Ksel; base += kThreads) {
      const int i = base + tid;
      const bool active = i < Ksel;
      const int v = active ? sel_idx[i] : 0;
      int r = 0;
      for (int t0 = 0; t0 < Ksel; t0 += 1024) {
        const int cnt = min(1024, Ksel - t0);
        __syncthreads();
        for (int j = tid; j < cnt; j += kThreads) sh_win[j] = sel_idx[t0 + j];
        __syncthreads();
        if (active)
          for (int j = 0; j < cnt; ++j) r += sh_win[j] < v ? 1 : 0;
      }
      if (active) out[min(r, Ksel - 1)] = g.n_sink + v;
    }
  }
}

}  // namespace tkphi
