// The retrieved-token side of eq. (subtraction) on the matrix cores, for one wavefront and 16 tokens:
// z_i = phi_q . phi_k(k_i) with phi_k(k_i) recomputed from the gathered key through the same arithmetic
// as the summary build (bf16 MFMA with fp32 accumulation, one exp2 per feature, the result kept as a bf16
// hi + lo pair), so that what is subtracted is what was added.  Shared by the gather kernel of the spill
// pipeline and the fused select + gather kernel of the filtered one.
#pragma once

#include "tkphi_internal.h"

namespace tkphi {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 gt_bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float gt_floatx4;
union GatherFrag {
  u32x4 u;
  gt_bf16x8 v;
};

constexpr int wk_row_bytes(int D) { return D * 2 + 16; }   // staged Wk rows are padded by 16 B: conflict-free 16-byte reads

// Stages Wk[h] ([D features][D channels] bf16) into LDS with padded rows in two steps, so that a caller with NT
// threads can put other work between the request and the LDS stores: wk_request loads the thread's pieces
// (piece i of the matrix = 16 bytes; thread t holds pieces t, t + NT, ...), wk_commit stores them; a barrier
// before the first use.
template <int D, int NT>
struct WkPieces {
  static constexpr int SEGS = D * 2 / 16, N = (D * SEGS + NT - 1) / NT;
  u32x4 t[N];
  __device__ __forceinline__ void request(const void* Wk, int h) {
    const char* wsrc = (const char*)Wk + (size_t)h * D * D * 2;
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const int i = min((int)threadIdx.x + k * NT, D * SEGS - 1);
      t[k] = gload128(wsrc + (size_t)(i / SEGS) * D * 2 + (i % SEGS) * 16);
    }
  }
  __device__ __forceinline__ void commit(char* wk_lds) const {
    constexpr int WROW = wk_row_bytes(D);
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const int i = (int)threadIdx.x + k * NT;
      if (i < D * SEGS) *(u32x4*)(wk_lds + (i / SEGS) * WROW + (i % SEGS) * 16) = t[k];
    }
  }
};

// The same in one step; every thread of the workgroup takes part; the caller puts a barrier before the first use.
template <int D>
__device__ __forceinline__ void stage_wk(const void* Wk, int h, char* wk_lds) {
  constexpr int WROW = wk_row_bytes(D), SEGS = D * 2 / 16;
  const char* wsrc = (const char*)Wk + (size_t)h * D * D * 2;
  for (int i0 = threadIdx.x; i0 < D * SEGS; i0 += 4 * blockDim.x) {
    u32x4 t[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = min(i0 + k * (int)blockDim.x, D * SEGS - 1);
      t[k] = gload128(wsrc + (size_t)(i / SEGS) * D * 2 + (i % SEGS) * 16);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + k * (int)blockDim.x;
      if (i < D * SEGS) *(u32x4*)(wk_lds + (i / SEGS) * WROW + (i % SEGS) * 16) = t[k];
    }
  }
}

// a[j]: key row of this lane's token r = lane & 15, channels j 32 + kg 8 .. + 8 (kg = lane >> 4).
// On return z[i] = phi_q . phi_k(k) of token 4 kg + i, in every lane of the kg group.
template <int D>
__device__ __forceinline__ void wave_feature_dots(const GatherFrag (&a)[D / 32], const char* wk_lds, const float* bk_h,
                                                  const float* phiq, float fa, float fc, float (&z)[4]) {
  constexpr int KS = D / 32, NT = D / 16, WROW = wk_row_bytes(D);
  const int lane = threadIdx.x & 63, r = lane & 15, kg = lane >> 4;
  float bj[NT], pj[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) { bj[nt] = bk_h[nt * 16 + r] * kLog2e; pj[nt] = phiq[nt * 16 + r]; }
  const float a2 = fa * kLog2e, c2 = fc * kLog2e;
  // |k|^2 of token r: this lane's 8 KS channels, then the 4 lanes of the row
  float nrm = 0.f;
#pragma unroll
  for (int j = 0; j < KS; ++j) {
    float x[8];
    Elem<uint16_t>::unpack(make_uint4(a[j].u.x, a[j].u.y, a[j].u.z, a[j].u.w), x);
#pragma unroll
    for (int e = 0; e < 8; ++e) nrm = fmaf(x[e], x[e], nrm);
  }
  nrm += __shfl_xor(nrm, 16);
  nrm += __shfl_xor(nrm, 32);
  float cn[4];                                   // c |k|^2 log2(e) of tokens 4 kg + i
#pragma unroll
  for (int i = 0; i < 4; ++i) cn[i] = c2 * __shfl(nrm, 4 * kg + i);
#pragma unroll
  for (int i = 0; i < 4; ++i) z[i] = 0.f;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    gt_floatx4 acc = (gt_floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      GatherFrag b;
      b.u = *(const u32x4*)(wk_lds + (nt * 16 + r) * WROW + j * 64 + kg * 16);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j].v, b.v, acc, 0, 0, 0);
    }
    // acc[i] = Wk[feature nt 16 + r] . k(token 4 kg + i)
    float f[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = phi_exp2(acc[i], a2, bj[nt] - cn[i]);
    uint32_t h01, l01, h23, l23;                 // the 16 bits per feature that the summary build contracted
    split_bf16_pair(f[0], f[1], &h01, &l01);
    split_bf16_pair(f[2], f[3], &h23, &l23);
    z[0] = fmaf(join_bf16_lo(h01, l01), pj[nt], z[0]);
    z[1] = fmaf(join_bf16_hi(h01, l01), pj[nt], z[1]);
    z[2] = fmaf(join_bf16_lo(h23, l23), pj[nt], z[2]);
    z[3] = fmaf(join_bf16_hi(h23, l23), pj[nt], z[3]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) z[i] += __shfl_xor(z[i], o);
  }
}

}  // namespace tkphi
