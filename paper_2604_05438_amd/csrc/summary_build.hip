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
// bf16 on the matrix cores: grid (n_build_chunks, Hkv, n_problems), 4 wavefronts,
// D == d_head == d_phi.  Wavefront w owns the features [w D/4, (w+1) D/4): its slice of Wk
// stays in registers for the whole chunk.
//
// The chunk is cut into tiles of 32 tokens.  A stage of LDS holds one tile of keys and one of
// values, both row-major as they lie in the cache, brought in by loads that write LDS
// directly; NS stages form a ring, so NS - 1 tiles are on their way from HBM while one is
// contracted, and no register is spent on data in flight.  Per tile:
//   GEMM1  P[32 tokens][own features] = K Wk^T : A = key rows from LDS, B = Wk slice
//          -> exp -> bf16 hi + lo; the result registers (4 consecutive tokens per lane and
//          16-token tile) are already the A operand of GEMM2 over a fixed permutation of
//          the 32 tokens, so the features never touch LDS
//   GEMM2  S[own features][all channels] += Phi^T V : B = value tile read through the
//          transposing LDS read (same token permutation), hi and lo as two MFMAs
// u is summed from the same features.
//
// Each load instruction moves 64 x 16 bytes into 1 KB of consecutive LDS (lane l -> bytes
// 16 l ..), so a lane picks WHICH 16-byte granule of its row it fetches: granule slot s of row
// r holds granule s ^ f(r) of that row, with f chosen per tensor so that the reads spread
// over all banks:
//   keys    read as the A operand of GEMM1 (16 lanes = 16 rows, same granule): f = row mod 16
//           (rows of 256 bytes), (row / 2) mod 8 (rows of 128 bytes)
//   values  read by the transposing LDS read (16 lanes take 8 bytes each of 4 rows x 16
//           channels; lane j receives the 4 tokens of channel j): f = 2 (row mod 8) resp.
//           2 ((row / 2) mod 4)
// |k|^2: a wavefront reads back the rows its own loads brought (its own wait covers them), sums
// the squares with 16-bit dot products and leaves c |k|^2 per row in LDS before the tile's
// barrier: one barrier per tile.
// ------------------------------------------------------------------------------------
typedef short short4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {   // a.lo b.lo + a.hi b.hi + c
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  union { uint32_t u; bf16x2 v; } x, y;
  x.u = a; y.u = b;
  return __builtin_amdgcn_fdot2_f32_bf16(x.v, y.v, c, false);
}

template <int D, bool CACHE, int NS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 4 : 2, D == 64 ? 4 : 2)))
void build_mfma_kernel(Geom g, const tkphi_problem* __restrict__ probs, char* __restrict__ ws) {
  constexpr int NW = 4;
  constexpr int KS = D / 32;            // k-steps of GEMM1 (over channels)
  constexpr int FT = D / (16 * NW);     // feature tiles per wavefront
  constexpr int CT = D / 16;            // channel tiles of S
  constexpr int GR = D / 8;             // 16-byte granules per row
  constexpr int TT = 32;                // tokens per tile
  constexpr int ROWB = D * 2;           // bytes per row
  constexpr int TILEB = TT * ROWB;      // bytes per key (or value) tile
  constexpr int RPI = 64 / GR;          // rows one load instruction covers
  constexpr int NLD = TT / (RPI * NW);  // load instructions per wavefront, tile and tensor
  static_assert(NLD >= 1 && NS >= 3 && NS <= 6, "ring shape");
  extern __shared__ __attribute__((aligned(1024))) char ring[];   // [NS][keys, values][TT][ROWB], then norms [NS][TT]
  float* nrm_all = (float*)(ring + NS * 2 * TILEB);               // c |k|^2 log2(e); +inf past the chunk end

  const int ch = blockIdx.x, h = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int c0 = ch * g.build_chunk;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + g.build_chunk);
  const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), r = lane & 15, kg = lane >> 4;
  const float a2 = g.a * kLog2e, c2 = g.c * kLog2e;

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
  wait_vm_loads<0>();                    // (the tile loads below are counted by hand)
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
  const char* Kt = (const char*)pr.K + base_off;
  const char* Vt = (const char*)pr.V + base_off;
  const uint32_t ring_addr = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)ring;

  auto f_key = [](int row) { return GR == 16 ? (row & 15) : ((row >> 1) & 7); };
  auto f_val = [](int row) { return GR == 16 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1); };
  // loads: instruction i of wavefront wv fills rows (wv * NLD + i) * RPI .. + RPI of a tile
  int ld_row[NLD], ld_kg[NLD], ld_vg[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    ld_row[i] = (wv * NLD + i) * RPI + lane / GR;
    ld_kg[i] = ((lane % GR) ^ f_key(ld_row[i])) * 16;
    ld_vg[i] = ((lane % GR) ^ f_val(ld_row[i])) * 16;
  }
  const int n_tiles = (c1 - c0 + TT - 1) / TT;
  // a full tile is fetched as uniform tile base + a lane's constant 32-bit offset (when a tile's rows span < 2 GiB)
  const bool near = (uint64_t)TT * row_bytes < (1ull << 31);
  uint32_t ld_ko[NLD], ld_vo[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    ld_ko[i] = near ? (uint32_t)(ld_row[i] * row_bytes) + ld_kg[i] : 0u;
    ld_vo[i] = near ? (uint32_t)(ld_row[i] * row_bytes) + ld_vg[i] : 0u;
  }
  auto issue = [&](int ti) {             // tile ti of the chunk -> stage ti % NS
    const int t0 = c0 + ti * TT;
    const uint32_t st = ring_addr + (uint32_t)(ti % NS) * (2 * TILEB) + (uint32_t)(wv * NLD) * 1024;
    if (near && t0 + TT <= c1) {
      const char* kb = Kt + (size_t)t0 * row_bytes;
      const char* vb = Vt + (size_t)t0 * row_bytes;
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        load_to_lds16_stream(kb, ld_ko[i], st + i * 1024);
        load_to_lds16_stream(vb, ld_vo[i], st + TILEB + i * 1024);
      }
    } else {                             // rows past the end re-read the last row
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const size_t ro = (size_t)min(t0 + ld_row[i], c1 - 1) * row_bytes;
        load_to_lds16_stream(Kt + ro + ld_kg[i], st + i * 1024);
        load_to_lds16_stream(Vt + ro + ld_vg[i], st + TILEB + i * 1024);
      }
    }
  };
  // |k|^2 of the rows this wavefront loaded (lane l holds 16 bytes of row l / GR of each of its blocks)
  auto own_norms = [&](int ti) {
    const int t0 = c0 + ti * TT;
    const char* k_t = ring + (size_t)(ti % NS) * (2 * TILEB);
    float* nrm_t = nrm_all + (ti % NS) * TT;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const u32x4 w = *(const u32x4*)(k_t + (wv * NLD + i) * 1024 + lane * 16);
      float sq = dot2_bf16(w.x, w.x, 0.f);
      sq = dot2_bf16(w.y, w.y, sq);
      sq = dot2_bf16(w.z, w.z, sq);
      sq = dot2_bf16(w.w, w.w, sq);
      sq = row_lanes_sum<GR>(sq);
      if (lane % GR == 0) nrm_t[ld_row[i]] = t0 + ld_row[i] < c1 ? c2 * sq : INFINITY;
    }
  };
  // reads: per-lane byte offsets inside a key tile (A operand of GEMM1, row r of a 16-token tile) and
  // inside a value tile (8 bytes of row 4 kg + s / 4, channels 16 ct + 4 (s mod 4) .., s = lane mod 16)
  uint32_t a_off[KS], v_off[CT];
#pragma unroll
  for (int j = 0; j < KS; ++j) a_off[j] = (uint32_t)(r * ROWB + (((j * 4 + kg) ^ f_key(r)) * 16));
  {
    const int vrow = 4 * kg + (r >> 2), b = r & 3, fv2 = f_val(vrow) >> 1;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) v_off[ct] = (uint32_t)(vrow * ROWB + ((ct ^ fv2) << 5) + b * 8);
  }
  float* cache_h = CACHE ? pr.phi_cache + (size_t)h * n * D : nullptr;   // [token of M][feature]

  auto contract = [&](int ti) {
    const int t0 = c0 + ti * TT;
    const char* k_t = ring + (size_t)(ti % NS) * (2 * TILEB);
    const char* v_t = k_t + TILEB;
    const float* nrm_t = nrm_all + (ti % NS) * TT;
    u32x2 phi_hi[2][FT], phi_lo[2][FT];
    float ut[FT];
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) ut[ft] = 0.f;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      Frag a[KS];
#pragma unroll
      for (int j = 0; j < KS; ++j) a[j].u = *(const u32x4*)(k_t + mt * 16 * ROWB + a_off[j]);
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

    // GEMM2, one k-step: lane (., kg) holds tokens 4 kg + {0..3} and 16 + 4 kg + {0..3} in both operands
    Frag ahi[FT], alo[FT];
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) {
      ahi[ft].u = (u32x4){phi_hi[0][ft].x, phi_hi[0][ft].y, phi_hi[1][ft].x, phi_hi[1][ft].y};
      alo[ft].u = (u32x4){phi_lo[0][ft].x, phi_lo[0][ft].y, phi_lo[1][ft].x, phi_lo[1][ft].y};
    }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      typedef short4v __attribute__((address_space(3)))* lds_s4;
      union { short4v s; u32x2 u; } b0, b1;
      b0.s = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(v_t + v_off[ct]));
      b1.s = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(v_t + 16 * ROWB + v_off[ct]));
      Frag vb;
      vb.u = (u32x4){b0.u.x, b0.u.y, b1.u.x, b1.u.y};
#pragma unroll
      for (int ft = 0; ft < FT; ++ft) {
        sacc[ft][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo[ft].v, vb.v, sacc[ft][ct], 0, 0, 0);
        sacc[ft][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi[ft].v, vb.v, sacc[ft][ct], 0, 0, 0);
      }
    }
  };

#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < n_tiles) issue(s);
  constexpr int PER = 2 * NLD;           // load instructions per wavefront and tile
  for (int ti = 0; ti < n_tiles; ++ti) {
    // this wavefront's share of tile ti has landed once at most min(NS - 2, tiles issued after ti) tiles are in flight
    const int after = min(NS - 2, n_tiles - 1 - ti);
    if (after >= NS - 2) wait_vm_loads<(NS - 2) * PER>();
    else if (after == 3) wait_vm_loads<3 * PER>();
    else if (after == 2) wait_vm_loads<2 * PER>();
    else if (after == 1) wait_vm_loads<PER>();
    else wait_vm_loads<0>();
    own_norms(ti);
    lds_barrier();                       // every share of tile ti is in LDS; stage (ti - 1) % NS is free
    if (ti + NS - 1 < n_tiles) issue(ti + NS - 1);
    contract(ti);
  }

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

template <int D, bool CACHE, int NS>
static void launch_build_mfma_as(const Geom& g, const tkphi_problem* probs, char* ws, dim3 grid, hipStream_t s) {
  const size_t lds = (size_t)NS * (2 * 32 * D * 2 + 32 * 4);
  const hipError_t e = hipFuncSetAttribute((const void*)build_mfma_kernel<D, CACHE, NS>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) { set_error("hipFuncSetAttribute(%zu bytes of LDS): %s", lds, hipGetErrorString(e)); return; }
  TKPHI_LAUNCH(ST_UNTIMED, (build_mfma_kernel<D, CACHE, NS>), grid, dim3(256), lds, s, g, probs, ws);
}
static void launch_build_mfma(const Geom& g, const tkphi_problem* probs, char* ws, dim3 grid, hipStream_t s) {
  constexpr int NS = 4;                  // ring stages: three tiles on their way while one is contracted
  if (g.d == 128 && g.cache) launch_build_mfma_as<128, true, NS>(g, probs, ws, grid, s);
  else if (g.d == 128) launch_build_mfma_as<128, false, NS>(g, probs, ws, grid, s);
  else if (g.cache) launch_build_mfma_as<64, true, NS>(g, probs, ws, grid, s);
  else launch_build_mfma_as<64, false, NS>(g, probs, ws, grid, s);
}

void launch_build(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  if (g.max_mid > 0) {
    dim3 grid(g.n_build_chunks, g.Hkv, g.n_problems);
    if (g.phi_kind == TKPHI_PHI_MLP) {
      launch_mlp_build(g, probs, ws, s);            // phi_k of the mid-region, then S, u chunk partials from the features
    } else if (g.use_mfma) {
      launch_build_mfma(g, probs, ws, grid, s);
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
