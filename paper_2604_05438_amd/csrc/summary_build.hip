// Prefill summary build (eq. (natural_cache)):
//   S[h][j][c] = sum_{i in M} phi_k(k_i)[j] v_i[c],   u[h][j] = sum_{i in M} phi_k(k_i)[j]
// with phi_k(k)[j] = exp(a * Wk[h][j] . k - c |k|^2 + bk[h][j]).
//
// The mid-region of each (problem, KV head) is split into chunks; one workgroup reduces a
// chunk into a partial [dphi][d] + [dphi], and a second kernel sums the partials of a head
// in chunk order, so the result does not depend on scheduling.
//
// bf16 caches use the matrix cores for both contractions (features = K Wk^T, then
// S = Phi^T [V | 1]); other storage types use a generic fp32 kernel.
#include "block_utils.h"
#include "tkphi_internal.h"

namespace tkphi {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
union Frag {
  u32x4 u;
  bf16x8 v;
};

// Sum over the N (power of two, <= 16) consecutive lanes that hold one row, by data-parallel-primitive
// moves inside a row of 16 lanes: the same butterfly as xor-shuffles by 1, 2, 4, 8 (lanes that mirror
// each other across a quad pair / a half row hold equal partial sums after the earlier steps), every
// lane ends with the total.
template <int N>
__device__ __forceinline__ float row_lanes_sum(float s) {
  auto dpp = [](float v, auto ctrl) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, false));
  };
  if (N >= 2) s += dpp(s, std::integral_constant<int, 0xB1>{});    // quad_perm [1, 0, 3, 2]
  if (N >= 4) s += dpp(s, std::integral_constant<int, 0x4E>{});    // quad_perm [2, 3, 0, 1]
  if (N >= 8) s += dpp(s, std::integral_constant<int, 0x141>{});   // row_half_mirror
  if (N >= 16) s += dpp(s, std::integral_constant<int, 0x140>{});  // row_mirror
  return s;
}

// ------------------------------------------------------------------------------------
// bf16 on the matrix cores: grid (n_build_chunks, Hkv, n_problems); D == d_head == d_phi.
//
// Tiles of 64 tokens; the key and value tiles are staged in LDS once per workgroup (keys
// row-major, values transposed in registers - 4 tokens x 8 channels per lane - and stored
// channel-major), |k|^2 is reduced while staging.  Wavefront w owns the features
// [w*D/NW, (w+1)*D/NW): its slice of Wk stays in registers for the whole chunk.
//   GEMM1  P[64 tokens][own features] = K Wk^T : A = key rows from LDS, B = Wk slice
//          -> exp -> bf16 hi + lo; the result registers (4 consecutive tokens per lane and
//          16-token tile) are already the A operand of GEMM2 over a fixed permutation of
//          the 32 tokens of a k-step, so the features never touch LDS
//   GEMM2  S[own features][all channels] += Phi^T V : B = transposed value tile from LDS
//          (two 8-byte reads per operand, same token permutation), hi and lo as two MFMAs
// u is summed from the same features.  Two LDS tile buffers: tile t+1 is staged (and the
// global loads of tile t+2 are issued) before tile t is contracted: one barrier per tile.
// ------------------------------------------------------------------------------------
// NW wavefronts per workgroup (4 or 8), each owning D / NW features.  The LDS tiles allow two workgroups per CU
// at D = 128 and four at D = 64, so NW = 8 resp. 4 puts four wavefronts on a SIMD: one's exponentials and staging
// hide behind another's MFMAs.
template <int D, bool CACHE, int NW>  // CACHE: also store the contracted features in pr.phi_cache
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(D == 64 ? 4 : NW / 2, D == 64 ? 4 : NW / 2))) void build_mfma_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                 char* __restrict__ ws) {
  constexpr int KS = D / 32;            // k-steps of GEMM1 (over channels)
  constexpr int NT = 64 * NW;           // threads
  constexpr int FT = D / (16 * NW);     // feature tiles per wavefront
  static_assert(FT >= 1, "at least 16 features per wavefront");
  constexpr int CT = D / 16;            // channel tiles of S
  constexpr int SEGS = D / 8;           // 16-byte segments per row
  constexpr int KLD = 64 * SEGS / NT;   // key-row loads per thread and tile (4 or 2)
  constexpr int KROW = D * 2 + 16;      // bytes per staged key row
  constexpr int TROW = 64 * 2 + 16;     // bytes per staged value-channel row (64 tokens)
  // two tile buffers: tile t+1 is staged while tile t is contracted, one barrier per tile
  __shared__ __attribute__((aligned(16))) char k_tb[2][64 * KROW];    // [token][channel]
  __shared__ __attribute__((aligned(16))) char v_tb[2][D * TROW];     // [channel][token]
  __shared__ __attribute__((aligned(16))) float nrm_tb[2][64];        // c |k|^2 log2(e); +inf past the chunk end

  const int ch = blockIdx.x, h = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int c0 = ch * g.build_chunk;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + g.build_chunk);
  const int lane = tid & 63, wv = tid >> 6, r = lane & 15, kg = lane >> 4;
  const float a2 = g.a * kLog2e, c2 = g.c * kLog2e;

  // Wk slice: wk[ft][j] = Wk[h][feature wv*D/4 + ft*16 + r][channels j*32 + kg*8 .. +8]
  Frag wk[FT][KS];
  float bias[FT];
  {
    const uint16_t* wsrc = (const uint16_t*)pr.Wk + (size_t)h * D * D;
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) {
      const int feat = wv * (D / NW) + ft * 16 + r;
#pragma unroll
      for (int j = 0; j < KS; ++j) wk[ft][j].u = gload128(wsrc + (size_t)feat * D + j * 32 + kg * 8);
      bias[ft] = pr.bk[(size_t)h * D + feat] * kLog2e;
    }
  }
  floatx4 sacc[FT][CT];
#pragma unroll
  for (int ft = 0; ft < FT; ++ft)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) sacc[ft][ct] = (floatx4){0.f, 0.f, 0.f, 0.f};
  float uacc[FT];
#pragma unroll
  for (int ft = 0; ft < FT; ++ft) uacc[ft] = 0.f;

  const size_t row_bytes = (size_t)pr.stride_tok * 2;
  const size_t base_off = ((size_t)h * pr.stride_head + (size_t)g.n_sink * pr.stride_tok) * 2;
  // key loads: thread (krow = tid / SEGS, seg = tid % SEGS) takes rows krow + i * (256 / SEGS)
  const int kseg = tid % SEGS, krow = tid / SEGS;
  constexpr int KRP = NT / SEGS;  // key rows per pass
  // value loads: thread (tq, sg) takes tokens 4*tq .. 4*tq+3 of the tile, 16-byte segment sg
  const bool v_active = tid < 16 * SEGS;
  const int tq = tid % 16, sg = tid / 16;
  // A tile's rows start at a uniform address; a thread's byte offsets inside a full tile never change
  // (32 bits: a tile spans 64 rows), so the loads of a full tile are base + offset with no per-row arithmetic.
  const char* Kt = (const char*)pr.K + base_off;
  const char* Vt = (const char*)pr.V + base_off;
  uint32_t koff[KLD], voff[4];
#pragma unroll
  for (int i = 0; i < KLD; ++i) koff[i] = (uint32_t)((krow + i * KRP) * row_bytes) + kseg * 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) voff[i] = (uint32_t)((tq * 4 + i) * row_bytes) + sg * 16;

  u32x4 kk[KLD], vv[4];
  auto issue_loads = [&](int t0) {
    const char* kt = Kt + (size_t)t0 * row_bytes;
    const char* vt = Vt + (size_t)t0 * row_bytes;
    if (t0 + 64 <= c1) {                 // full tile
#pragma unroll
      for (int i = 0; i < KLD; ++i) kk[i] = gload128_stream(kt + koff[i]);
      if (v_active) {
#pragma unroll
        for (int i = 0; i < 4; ++i) vv[i] = gload128_stream(vt + voff[i]);
      }
    } else {                             // last tile of the mid-region: rows past the end re-read the last row
#pragma unroll
      for (int i = 0; i < KLD; ++i) {
        const int row = min(krow + i * KRP, c1 - 1 - t0);
        kk[i] = gload128_stream(kt + (size_t)row * row_bytes + kseg * 16);
      }
      if (v_active) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int vrow = min(tq * 4 + i, c1 - 1 - t0);
          vv[i] = gload128_stream(vt + (size_t)vrow * row_bytes + sg * 16);
        }
      }
    }
  };

  auto stage = [&](int t0, char* k_t, char* v_t, float* nrm_t) {
    const bool full = t0 + 64 <= c1;     // (uniform) no row of the tile lies past the end
    // ---- stage the tile: keys row-major (+ norms), values channel-major ---------------------
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
      const int row = krow + i * KRP;
      *(u32x4*)(k_t + row * KROW + kseg * 16) = kk[i];
      float x[8];
      Elem<uint16_t>::unpack(make_uint4(kk[i].x, kk[i].y, kk[i].z, kk[i].w), x);
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) s = fmaf(x[e], x[e], s);
      s = row_lanes_sum<SEGS>(s);        // over the SEGS lanes that share the row
      if (kseg == 0) nrm_t[row] = (full || t0 + row < c1) ? c2 * s : INFINITY;
    }
    if (v_active) {
      uint32_t w[4][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool ok = full || t0 + tq * 4 + i < c1;
        w[i][0] = ok ? vv[i].x : 0u; w[i][1] = ok ? vv[i].y : 0u;
        w[i][2] = ok ? vv[i].z : 0u; w[i][3] = ok ? vv[i].w : 0u;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {      // dword q of a token holds channels 2q (low half) and 2q+1 (high half)
        const u32x2 even = (u32x2){__builtin_amdgcn_perm(w[1][q], w[0][q], 0x05040100u), __builtin_amdgcn_perm(w[3][q], w[2][q], 0x05040100u)};
        const u32x2 odd = (u32x2){__builtin_amdgcn_perm(w[1][q], w[0][q], 0x07060302u), __builtin_amdgcn_perm(w[3][q], w[2][q], 0x07060302u)};
        *(u32x2*)(v_t + (sg * 8 + 2 * q) * TROW + tq * 8) = even;
        *(u32x2*)(v_t + (sg * 8 + 2 * q + 1) * TROW + tq * 8) = odd;
      }
    }
  };
  float* cache_h = CACHE ? pr.phi_cache + (size_t)h * n * D : nullptr;   // [token of M][feature]
  auto contract = [&](int t0, const char* k_t, const char* v_t, const float* nrm_t) {
    // ---- GEMM1 + exponent: all 64 tokens x this wavefront's features --------------------------
    u32x2 phi_hi[4][FT], phi_lo[4][FT];            // [16-token tile][feature tile]: tokens 4kg .. 4kg+3
    float ut[FT];                                  // this tile's share of u, added to the running sum once
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) ut[ft] = 0.f;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      Frag a[KS];
#pragma unroll
      for (int j = 0; j < KS; ++j) a[j].u = *(const u32x4*)(k_t + (mt * 16 + r) * KROW + j * 64 + kg * 16);
      const floatx4 cn = *(const floatx4*)(nrm_t + mt * 16 + 4 * kg);
#pragma unroll
      for (int ft = 0; ft < FT; ++ft) {
        floatx4 acc = (floatx4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KS; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j].v, wk[ft][j].v, acc, 0, 0, 0);
        float f[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = phi_exp2(acc[i], a2, bias[ft] - cn[i]);
        ut[ft] += (f[0] + f[1]) + (f[2] + f[3]);
        uint32_t h01, l01, h23, l23;
        split_bf16_pair(f[0], f[1], &h01, &l01);
        split_bf16_pair(f[2], f[3], &h23, &l23);
        phi_hi[mt][ft] = (u32x2){h01, h23};
        phi_lo[mt][ft] = (u32x2){l01, l23};
        if (CACHE) {                     // the 16-bit values GEMM2 contracts, as fp32
          const int tok = t0 + mt * 16 + 4 * kg;
          float* cp = cache_h + (size_t)tok * D + wv * (D / NW) + ft * 16 + r;
          if (tok + 0 < c1) cp[0] = join_bf16_lo(h01, l01);
          if (tok + 1 < c1) cp[D] = join_bf16_hi(h01, l01);
          if (tok + 2 < c1) cp[2 * D] = join_bf16_lo(h23, l23);
          if (tok + 3 < c1) cp[3 * D] = join_bf16_hi(h23, l23);
        }
      }
    }

#pragma unroll
    for (int ft = 0; ft < FT; ++ft) uacc[ft] += ut[ft];

    // ---- GEMM2: S[own features][all channels] += Phi^T V ------------------------------------------
    // k-step ks contracts the 32 tokens of tiles 2ks and 2ks+1; lane (., kg) holds tokens
    // 32ks + 4kg + {0..3} and 32ks + 16 + 4kg + {0..3} in both operands
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      Frag ahi[FT], alo[FT];
#pragma unroll
      for (int ft = 0; ft < FT; ++ft) {
        ahi[ft].u = (u32x4){phi_hi[2 * ks][ft].x, phi_hi[2 * ks][ft].y, phi_hi[2 * ks + 1][ft].x, phi_hi[2 * ks + 1][ft].y};
        alo[ft].u = (u32x4){phi_lo[2 * ks][ft].x, phi_lo[2 * ks][ft].y, phi_lo[2 * ks + 1][ft].x, phi_lo[2 * ks + 1][ft].y};
      }
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const char* vp = v_t + (ct * 16 + r) * TROW + (32 * ks + 4 * kg) * 2;
        const u32x2 b0 = *(const u32x2*)vp, b1 = *(const u32x2*)(vp + 32);
        Frag vb;
        vb.u = (u32x4){b0.x, b0.y, b1.x, b1.y};
#pragma unroll
        for (int ft = 0; ft < FT; ++ft) {
          sacc[ft][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo[ft].v, vb.v, sacc[ft][ct], 0, 0, 0);
          sacc[ft][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi[ft].v, vb.v, sacc[ft][ct], 0, 0, 0);
        }
      }
    }
  };

  issue_loads(c0);
  stage(c0, k_tb[0], v_tb[0], nrm_tb[0]);
  if (c0 + 64 < c1) issue_loads(c0 + 64);
  lds_barrier();                         // (LDS only: the loads of the next tile stay in flight)
  int cur = 0;
  for (int t0 = c0; t0 < c1; t0 += 64) {
    if (t0 + 64 < c1) {                  // next tile: registers -> the other buffer, then refill the registers
      stage(t0 + 64, k_tb[cur ^ 1], v_tb[cur ^ 1], nrm_tb[cur ^ 1]);
      if (t0 + 128 < c1) issue_loads(t0 + 128);
    }
    contract(t0, k_tb[cur], v_tb[cur], nrm_tb[cur]);
    lds_barrier();                       // the other buffer is complete, this one is free
    cur ^= 1;
  }

  // ---- write the chunk partial: S part [D][D] then u part [D] ----------------------------------
  float* bp = (float*)(ws + g.off_bpart) + ((size_t)(p * g.Hkv + h) * g.n_build_chunks + ch) * ((size_t)D * (D + 1));
#pragma unroll
  for (int ft = 0; ft < FT; ++ft) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        bp[(size_t)(wv * (D / NW) + ft * 16 + 4 * kg + i) * D + ct * 16 + r] = sacc[ft][ct][i];
    float x = uacc[ft];
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    if (kg == 0) bp[(size_t)D * D + wv * (D / NW) + ft * 16 + r] = x;
  }
}

// ------------------------------------------------------------------------------------
// generic kernel (any storage type, fp32 arithmetic): grid (n_build_chunks, Hkv, n_problems)
// threads form a 16 x 16 grid over (feature block, channel block).
// ------------------------------------------------------------------------------------
constexpr int kTB = 16;   // tokens per batch

template <typename T>
__global__ __launch_bounds__(kThreads) void build_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                         char* __restrict__ ws) {
  __shared__ float kf[kTB][kMaxDim];
  __shared__ float vf[kTB][kMaxDim];
  __shared__ float ph[kTB][kMaxDim];
  constexpr int FJmax = kMaxDim / 16, FCmax = 128 / 16;

  const int ch = blockIdx.x, h = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int c0 = ch * g.build_chunk;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + g.build_chunk);
  const int d = g.d, dphi = g.dphi;
  const int FJ = dphi / 16, FC = d / 16;
  const int tj = tid / 16, tc = tid % 16;

  float acc[FJmax][FCmax];
  float uacc[FJmax];
#pragma unroll
  for (int a = 0; a < FJmax; ++a) {
    uacc[a] = 0.f;
#pragma unroll
    for (int b = 0; b < FCmax; ++b) acc[a][b] = 0.f;
  }
  const int64_t head_off = (int64_t)h * pr.stride_head;

  for (int base = c0; base < c1; base += kTB) {
    const int nt = min(kTB, c1 - base);
    __syncthreads();
    for (int i = tid; i < kTB * d; i += kThreads) {
      const int t = i / d, c = i % d;
      float kv = 0.f, vv = 0.f;
      if (t < nt) {
        const int64_t off = head_off + (int64_t)(g.n_sink + base + t) * pr.stride_tok + c;
        kv = Elem<T>::load1(pr.K, off);
        vv = Elem<T>::load1(pr.V, off);
      }
      kf[t][c] = kv; vf[t][c] = vv;
    }
    __syncthreads();
    // features: thread (t = tid / 16, j = tid % 16 + 16 * i)
    {
      const int t = tid / 16;
      float nrm = 0.f;
      for (int c = 0; c < d; ++c) nrm = fmaf(kf[t][c], kf[t][c], nrm);
      for (int i = 0; i < FJ; ++i) {
        const int j = (tid % 16) + 16 * i;
        const int64_t wbase = ((int64_t)h * dphi + j) * d;
        float dot = 0.f;
        constexpr int EPL = Elem<T>::per16;
        for (int c = 0; c < d; c += EPL) {       // 16-byte pieces of the Wk row
          const u32x4 wv4 = gload128((const char*)pr.Wk + (wbase + c) * sizeof(T));
          float wx[EPL];
          Elem<T>::unpack(make_uint4(wv4.x, wv4.y, wv4.z, wv4.w), wx);
#pragma unroll
          for (int e = 0; e < EPL; ++e) dot = fmaf(wx[e], kf[t][c + e], dot);
        }
        const float f = expf(g.a * dot - g.c * nrm + pr.bk[(int64_t)h * dphi + j]);
        ph[t][j] = t < nt ? f : 0.f;
        if (g.cache && t < nt) pr.phi_cache[((size_t)h * n + base + t) * dphi + j] = f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int a = 0; a < FJmax; ++a) {
      if (a < FJ) {
        const int j = tj * FJ + a;
        float ub = 0.f;                    // this batch's share of u
        for (int t = 0; t < kTB; ++t) {
          const float f = ph[t][j];
          ub += f;
#pragma unroll
          for (int b = 0; b < FCmax; ++b)
            if (b < FC) acc[a][b] = fmaf(f, vf[t][tc * FC + b], acc[a][b]);
        }
        uacc[a] += ub;
      }
    }
  }

  float* bp = (float*)(ws + g.off_bpart) +
              ((size_t)(p * g.Hkv + h) * g.n_build_chunks + ch) * ((size_t)dphi * (d + 1));
#pragma unroll
  for (int a = 0; a < FJmax; ++a) {
    if (a < FJ) {
      const int j = tj * FJ + a;
#pragma unroll
      for (int b = 0; b < FCmax; ++b)
        if (b < FC) bp[(size_t)j * d + tc * FC + b] = acc[a][b];
      if (tc == 0) bp[(size_t)dphi * d + j] = uacc[a];
    }
  }
}

// sums the chunk partials of each (problem, KV head) in a fixed order.
// grid (ceil(dphi*(d+1)/4 / 64), Hkv, n_problems), 256 threads = 64 float4 elements x 4 chunk
// groups: group q sums chunks q*16 .. q*16+15 of every 64 (16 loads in flight), then the four
// group sums are added in group order.
__global__ __launch_bounds__(kThreads) void build_reduce_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                char* __restrict__ ws) {
  __shared__ float4 sh[4][64];
  const int h = blockIdx.y, p = blockIdx.z;
  if (blockIdx.x == 0 && h == 0 && p == 0) write_device_status(g, probs, ws, false);
  const int L = probs[p].L;
  if (L < 1 || L > g.max_L) return;
  const int n = mid_size(L, g.n_sink, g.n_tail);
  const int n_chunks = (n + g.build_chunk - 1) / g.build_chunk;
  const int d = g.d, dphi = g.dphi;
  const size_t per = (size_t)dphi * (d + 1);          // floats per partial (a multiple of 4)
  const int el = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const size_t e4 = (size_t)blockIdx.x * 64 + el;     // float4 index inside a partial
  const bool live = e4 * 4 < per;
  const float4* bp = (const float4*)((const float*)(ws + g.off_bpart) + ((size_t)(p * g.Hkv + h) * g.n_build_chunks) * per) +
                     (live ? e4 : 0);
  const size_t per4 = per / 4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int c0 = 0; c0 < n_chunks; c0 += 64) {
    float4 v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int c = c0 + grp * 16 + k;
      v[k] = bp[(size_t)min(c, n_chunks - 1) * per4];
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      if (c0 + grp * 16 + k < n_chunks) { acc.x += v[k].x; acc.y += v[k].y; acc.z += v[k].z; acc.w += v[k].w; }
    }
  }
  sh[grp][el] = acc;
  __syncthreads();
  if (grp != 0 || !live) return;
  float4 s = sh[0][el];
#pragma unroll
  for (int q = 1; q < 4; ++q) { s.x += sh[q][el].x; s.y += sh[q][el].y; s.z += sh[q][el].z; s.w += sh[q][el].w; }
  const size_t e = e4 * 4;
  if (e < (size_t)dphi * d) *(float4*)(probs[p].S + (size_t)h * dphi * d + e) = s;
  else *(float4*)(probs[p].u + (size_t)h * dphi + (e - (size_t)dphi * d)) = s;
}

void launch_build(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  if (g.max_mid > 0) {
    dim3 grid(g.n_build_chunks, g.Hkv, g.n_problems);
    if (g.phi_kind == TKPHI_PHI_MLP) {
      launch_mlp_build(g, probs, ws, s);            // phi_k of the mid-region, then S, u chunk partials from the features
    } else if (g.use_mfma) {
      if (g.d == 128 && g.cache) TKPHI_LAUNCH(ST_UNTIMED, (build_mfma_kernel<128, true, 4>), grid, dim3(kThreads), 0, s, g, probs, ws);
      else if (g.d == 128) TKPHI_LAUNCH(ST_UNTIMED, (build_mfma_kernel<128, false, 4>), grid, dim3(kThreads), 0, s, g, probs, ws);
      else if (g.cache) TKPHI_LAUNCH(ST_UNTIMED, (build_mfma_kernel<64, true, 4>), grid, dim3(kThreads), 0, s, g, probs, ws);
      else TKPHI_LAUNCH(ST_UNTIMED, (build_mfma_kernel<64, false, 4>), grid, dim3(kThreads), 0, s, g, probs, ws);
    } else if (g.dtype == TKPHI_BF16) {
      TKPHI_LAUNCH(ST_UNTIMED, build_kernel<uint16_t>, grid, dim3(kThreads), 0, s, g, probs, ws);
    } else {
      TKPHI_LAUNCH(ST_UNTIMED, build_kernel<float>, grid, dim3(kThreads), 0, s, g, probs, ws);
    }
  }
  const int per4 = g.dphi * (g.d + 1) / 4;
  dim3 rgrid((per4 + 63) / 64, g.Hkv, g.n_problems);
  TKPHI_LAUNCH(ST_UNTIMED, build_reduce_kernel, rgrid, dim3(kThreads), 0, s, g, probs, ws);
}

}  // namespace tkphi
