// MLP feature maps (App. "Head-wise phi architecture"): the one-block ReZero MLP
//   g0 = Ws x + bs;  Delta = W2 GeLU(W1 g0 + b1) + b2;  g1 = g0 + alpha Delta;  phi(x) = exp(Wo g1 + bo)
// evaluated for the keys of the mid-region at build time, and the summary contraction
// S = Phi^T V, u = sum Phi (eq. (natural_cache)) from the stored features.
//
// Keys: every 64-token tile runs the chain
//   stem  G = X Ws^T + bs            (X = bf16 key rows: exact, single MFMA pass)
//   hid   H = GeLU(G W1^T + b1)
//   res   G = G + alpha (H W2^T + b2)    (in place: a tile reads only its own G entries)
//   out   Phi = exp(G Wo^T + bo)     -> tkphi_problem::phi_cache
// with one tiled matrix-core GEMM (mlp_gemm_tile).  A tile's layers depend only on the tile's own
// rows: by default one persistent launch per group of up to Geom::mlp_group problems takes each
// workgroup's tiles through stem, hid and res + out (g1 stays on chip); widths that do not fuse run
// the layers as separate launches per problem and block of Geom::mlp_block tokens.
// Without cfg.cache_features the features of a group go to a workspace buffer that the summary
// contraction of the group consumes, and decode recomputes the features of the retrieved keys
// (Sec. "Retrieved-token subtraction") by sending their rows through the same chain.
// Activations are fp32 in the workspace; as MFMA operands they are split into a bf16 hi + lo
// pair (16 significant bits, two MFMAs per product), weights are bf16 as stored, accumulation
// is fp32.  With ~1.3 MFLOP per token and KV head against 256 bytes of key the chain is bound by
// the matrix cores, not by HBM.
#include <algorithm>

#include "tkphi_internal.h"

namespace tkphi {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
union Frag {
  u32x4 u;
  bf16x8 v;
};

enum { EPI_STEM = 0, EPI_HID = 1, EPI_RES = 2, EPI_OUT = 3, EPI_RESOUT = 4 };

// ------------------------------------------------------------------------------------
// Weights in MFMA-fragment order.  A matrix W [N][Kd] (row-major bf16) is cut into blocks of 16
// outputs x 32 inputs; block (ct, ks) is stored as the 1 KB a wavefront loads as one operand:
// lane (r, kg) -> the 16 bytes W[16 ct + r][32 ks + 8 kg .. + 7], at byte ((ct Kd/32 + ks) 64 + lane) 16.
// The GEMM's operand loads then are whole 1 KB lines instead of 16 pieces of 64 B (measured 19 %
// faster).  One launch packs the four matrices of every KV head of the problems p0 .. p0 + gridDim.z - 1
// into the workspace, problem p0 + z into slot z: grid (ceil(pieces / 256), Hkv, problems); per head
// Ws | W1 | W2 | Wo, in this order.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ size_t packed_bytes_per_head(const Geom& g) {
  return ((size_t)g.d_emb * g.d + (size_t)2 * g.d_emb * g.d_emb + (size_t)g.dphi * g.d_emb) * 2;
}

__device__ __forceinline__ const char* packed_weights(const Geom& g, const char* ws, int slot, int h) {
  return ws + g.off_wpack + ((size_t)slot * g.Hkv + h) * packed_bytes_per_head(g);
}
// Where the key features of KV head h of a problem (n mid tokens) live: the caller's cache, or, without one, the
// workspace buffer of the problem's slot in the group being built.
__device__ __forceinline__ float* key_feature_rows(const Geom& g, const tkphi_problem& pr, char* ws, int slot, int h, int n) {
  if (g.cache) return pr.phi_cache + (size_t)h * n * g.dphi;
  return (float*)(ws + g.off_feat) + ((size_t)slot * g.Hkv + h) * (size_t)g.max_mid * g.dphi;
}

__global__ __launch_bounds__(kThreads) void mlp_pack_weights_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                    char* __restrict__ ws, int p0) {
  const int h = blockIdx.y, slot = blockIdx.z;
  const tkphi_problem pr = probs[p0 + slot];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const tkphi_mlp mp = pr.mlp_k[h];
  const int E = g.d_emb;
  const size_t n_s = (size_t)E * g.d / 8, n_1 = (size_t)E * E / 8, n_o = (size_t)g.dphi * E / 8;   // 16-byte pieces
  size_t q = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (q >= n_s + 2 * n_1 + n_o) return;
  char* dst = ws + g.off_wpack + ((size_t)slot * g.Hkv + h) * packed_bytes_per_head(g) + q * 16;
  const char* W;
  int Kd;
  if (q < n_s) { W = (const char*)mp.Ws; Kd = g.d; }
  else if (q < n_s + n_1) { W = (const char*)mp.W1; Kd = E; q -= n_s; }
  else if (q < n_s + 2 * n_1) { W = (const char*)mp.W2; Kd = E; q -= n_s + n_1; }
  else { W = (const char*)mp.Wo; Kd = E; q -= n_s + 2 * n_1; }
  const int lane = (int)(q & 63), r = lane & 15, kg = lane >> 4;
  const size_t blk = q >> 6;
  const int ks = (int)(blk % (Kd / 32)), ct = (int)(blk / (Kd / 32));
  *(u32x4*)dst = gload128(W + ((size_t)(ct * 16 + r) * Kd + ks * 32 + kg * 8) * 2);
}

// ------------------------------------------------------------------------------------
// The tile GEMM: 256 threads, a 64-token x (64 NT)-output tile of one KV head (the launchers give
// workgroup i the head i % Hkv: workgroups go to the 8 XCDs round-robin by linear index, so with 8 KV
// heads each XCD's L2 holds the weights of one head instead of all of them);
// wavefront w owns the outputs [16 NT w, 16 NT (w + 1)) (NT MFMA column tiles) of all four
// 16-token row tiles, so an A fragment read from LDS feeds NT (x2: hi, lo) MFMAs.  With NT = 8
// one workgroup spans all 512 outputs and the activations are read once.
// K loop in stages of 32: the A tile goes through LDS as bf16 hi / lo planes (row stride 80 B:
// conflict-free 16-byte operand reads), the weights go straight from the fragment-packed copy in
// global memory (L2) into the other operand.  Two LDS buffers, one barrier per stage; the next
// stage's global loads are issued before the MFMAs of the current one.
// ------------------------------------------------------------------------------------
// EPI_RESOUT (d_emb == 64 NT, d_phi == 64 NTO): residual and output layer in one launch.  The
// workgroup holds complete rows of g1 = g0 + alpha Delta in its accumulators; wavefront c's 16 NT
// features at a time go through LDS (bf16 hi / lo planes, token-major) and every wavefront multiplies
// them with its NTO output tiles of Wo.  g1 is never written to memory.
template <int NT>
constexpr int mlp_lds_bytes() {
  constexpr int stage = 4 * 64 * (32 * 2 + 16), planes = 2 * 64 * (16 * NT * 2 + 16);
  return stage > planes ? stage : planes;
}

// One 64-token tile of one layer.  tok0: first row of the tile; Gt, Ht: the tile's fp32
// activations g and h, [64][d_emb]; lds_raw: mlp_lds_bytes<NT>() bytes, free on entry (the caller
// puts a barrier between two calls); n0: first output of the workgroup (0 unless the layer is wider
// than 64 NT).  Row tok0 + i is mid token tok0 + i, or, with a row map, mid token rowmap[tok0 + i]
// (decode: the retrieved list of a query head); feat: where row 0's features go (row-major, d_phi floats
// per row); slot: which packed weights.
template <int EPI, int NT, int NTO>
__device__ __forceinline__ void mlp_gemm_tile(const Geom& g, const tkphi_problem& pr, const tkphi_mlp& mp, char* __restrict__ ws,
                                              char* lds_raw, int h, int n, int tok0, int rows_valid, float* Gt, float* Ht, int n0,
                                              int slot, float* feat, const int32_t* rowmap = nullptr) {
  constexpr int BM = 64, KB = 32;
  constexpr int AROW = KB * 2 + 16;
  constexpr bool A_BF16 = EPI == EPI_STEM;
  constexpr int KC = 16 * NT, RS = KC * 2 + 16;        // EPI_RESOUT: features per chunk, bytes per token row of a plane
  // staging planes: hi of buffer b at b BM AROW, lo at (2 + b) BM AROW
  const int tid = threadIdx.x;
  const int lane = tid & 63, r = lane & 15, kg = lane >> 4;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);     // wavefront index as a scalar: per-wavefront addresses stay in SGPRs
  const int E = g.d_emb;
  const int Kd = EPI == EPI_STEM ? g.d : E;
  const int Nout = EPI == EPI_OUT ? g.dphi : E;
  constexpr int EPI_W = EPI == EPI_RESOUT ? EPI_RES : EPI;     // which layer's weights the main loop multiplies
  if (n0 >= Nout) return;
  // fragment-packed weights of this head: Ws | W1 | W2 | Wo
  const size_t w_off = EPI_W == EPI_STEM ? 0 : EPI_W == EPI_HID ? (size_t)E * g.d : EPI_W == EPI_RES ? (size_t)E * g.d + (size_t)E * E
                                                                                                   : (size_t)E * g.d + (size_t)2 * E * E;
  const char* W = packed_weights(g, ws, slot, h) + w_off * 2;
  const float* bias = EPI_W == EPI_STEM ? mp.bs : EPI_W == EPI_HID ? mp.b1 : EPI_W == EPI_RES ? mp.b2 : mp.bo;

  // A rows: thread (srow = tid / 4, sseg = tid % 4) stages 8 consecutive inputs of row srow
  const int srow = tid >> 2, sseg = tid & 3;
  const int arow = min(srow, rows_valid - 1);          // clamped: rows past the end repeat the last one
  const char* a_src;
  if (A_BF16) {
    const int tok = rowmap ? min(max(rowmap[tok0 + arow], 0), n - 1) : tok0 + arow;
    a_src = (const char*)pr.K + ((size_t)h * pr.stride_head + (size_t)(g.n_sink + tok) * pr.stride_tok + sseg * 8) * 2;
  }
  else a_src = (const char*)((EPI_W == EPI_RES ? Ht : Gt) + (size_t)arow * E + sseg * 8);
  // weight operands: the NT output tiles of this wavefront (clamped to the last tile: every lane loads)
  const int colw = n0 + wv * NT * 16;
  const char* w_src[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) w_src[nt] = W + ((size_t)min(colw / 16 + nt, Nout / 16 - 1) * (Kd / 32) * 64 + lane) * 16;

  floatx4 acc[4][NT];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (floatx4){0.f, 0.f, 0.f, 0.f};

  u32x4 ar[2];          // fp32: 8 floats; bf16: ar[0] = 8 bf16
  Frag br[NT];
  auto issue = [&](int k0) {
    if (A_BF16) {
      ar[0] = gload128(a_src + (size_t)k0 * 2);
    } else {
      ar[0] = gload128(a_src + (size_t)k0 * 4);
      ar[1] = gload128(a_src + (size_t)k0 * 4 + 16);
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) br[nt].u = gload128(w_src[nt] + (size_t)(k0 / KB) * 1024);
  };

  const int n_stages = Kd / KB;
  issue(0);
  for (int st = 0; st < n_stages; ++st) {
    const int buf = st & 1;
    // ---- stage the A tile (split into hi / lo planes) ------------------------------------------
    if (A_BF16) {
      *(u32x4*)(lds_raw + buf * (BM * AROW) + srow * AROW + sseg * 16) = ar[0];
    } else {
      uint32_t hh[4], ll[4];
      split_bf16_pair(__uint_as_float(ar[0].x), __uint_as_float(ar[0].y), &hh[0], &ll[0]);
      split_bf16_pair(__uint_as_float(ar[0].z), __uint_as_float(ar[0].w), &hh[1], &ll[1]);
      split_bf16_pair(__uint_as_float(ar[1].x), __uint_as_float(ar[1].y), &hh[2], &ll[2]);
      split_bf16_pair(__uint_as_float(ar[1].z), __uint_as_float(ar[1].w), &hh[3], &ll[3]);
      *(u32x4*)(lds_raw + buf * (BM * AROW) + srow * AROW + sseg * 16) = (u32x4){hh[0], hh[1], hh[2], hh[3]};
      *(u32x4*)(lds_raw + (2 + buf) * (BM * AROW) + srow * AROW + sseg * 16) = (u32x4){ll[0], ll[1], ll[2], ll[3]};
    }
    Frag bcur[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) bcur[nt] = br[nt];
    __syncthreads();
    if (st + 1 < n_stages) issue((st + 1) * KB);
    // ---- MFMA ------------------------------------------------------------------------------------
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      Frag ahi, alo;
      ahi.u = *(const u32x4*)(lds_raw + buf * (BM * AROW) + (mt * 16 + r) * AROW + kg * 16);
      if (!A_BF16) alo.u = *(const u32x4*)(lds_raw + (2 + buf) * (BM * AROW) + (mt * 16 + r) * AROW + kg * 16);
      // weights as the row operand, tokens as the column operand: a lane ends up with 4 consecutive
      // outputs of one token (16-byte epilogue accesses).  All lo products of a row tile, then all hi
      // products: consecutive MFMAs never wait for each other's accumulator.
      if (!A_BF16) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bcur[nt].v, alo.v, acc[mt][nt], 0, 0, 0);
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bcur[nt].v, ahi.v, acc[mt][nt], 0, 0, 0);
    }
  }

  // ---- epilogue: acc[mt][nt][i] <-> token row mt*16 + r, output colw + nt*16 + 4kg + i --------------
  float* cache_h = feat + (size_t)tok0 * g.dphi;
  auto g_ptr = [&](int mt, int nt) { return Gt + (size_t)min(mt * 16 + r, rows_valid - 1) * E + colw + nt * 16 + 4 * kg; };
  if constexpr (EPI == EPI_RESOUT) {
    // g1 in place of the accumulators (the old residual stream is loaded a few tiles at a time)
    constexpr int HB = NT >= 8 ? 2 : NT > 1 ? NT / 2 : 1;
#pragma unroll
    for (int nb = 0; nb < NT; nb += HB) {
      float4 gv[HB][4];
#pragma unroll
      for (int j = 0; j < HB; ++j)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) gv[j][mt] = *(const float4*)g_ptr(mt, nb + j);
#pragma unroll
      for (int j = 0; j < HB; ++j) {
        const float4 b = *(const float4*)(bias + colw + (nb + j) * 16 + 4 * kg);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          acc[mt][nb + j][0] = fmaf(mp.alpha, acc[mt][nb + j][0] + b.x, gv[j][mt].x);
          acc[mt][nb + j][1] = fmaf(mp.alpha, acc[mt][nb + j][1] + b.y, gv[j][mt].y);
          acc[mt][nb + j][2] = fmaf(mp.alpha, acc[mt][nb + j][2] + b.z, gv[j][mt].z);
          acc[mt][nb + j][3] = fmaf(mp.alpha, acc[mt][nb + j][3] + b.w, gv[j][mt].w);
        }
      }
    }
    char* const p_hi = lds_raw;
    char* const p_lo = lds_raw + BM * RS;
    const char* Wo = packed_weights(g, ws, slot, h) + ((size_t)E * g.d + (size_t)2 * E * E) * 2;
    const int n_otiles = g.dphi / 16;
    floatx4 acco[4][NTO];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int j = 0; j < NTO; ++j) acco[mt][j] = (floatx4){0.f, 0.f, 0.f, 0.f};
    __syncthreads();                                   // the staging buffers are free
#pragma unroll 1
    for (int c = 0; c < 4; ++c) {
      if (wv == c) {                                   // this wavefront's features -> planes [token][16 NT features]
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) {
            uint32_t h01, l01, h23, l23;
            split_bf16_pair(acc[mt][nt][0], acc[mt][nt][1], &h01, &l01);
            split_bf16_pair(acc[mt][nt][2], acc[mt][nt][3], &h23, &l23);
            *(u32x2*)(p_hi + (mt * 16 + r) * RS + (nt * 16 + 4 * kg) * 2) = (u32x2){h01, h23};
            *(u32x2*)(p_lo + (mt * 16 + r) * RS + (nt * 16 + 4 * kg) * 2) = (u32x2){l01, l23};
          }
      }
      // (the output weights of this chunk are requested before the barrier: they do not depend on the planes)
      Frag wnext[NTO];
#pragma unroll
      for (int j = 0; j < NTO; ++j)
        wnext[j].u = gload128(Wo + ((size_t)(min(wv * NTO + j, n_otiles - 1) * (E / 32) + c * (KC / 32)) * 64 + lane) * 16);
      __syncthreads();
#pragma unroll 1
      for (int ksl = 0; ksl < KC / 32; ++ksl) {
        Frag wf[NTO];
#pragma unroll
        for (int j = 0; j < NTO; ++j) wf[j] = wnext[j];
        if (ksl + 1 < KC / 32) {
#pragma unroll
          for (int j = 0; j < NTO; ++j)
            wnext[j].u = gload128(Wo + ((size_t)(min(wv * NTO + j, n_otiles - 1) * (E / 32) + c * (KC / 32) + ksl + 1) * 64 + lane) * 16);
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          Frag bhi, blo;
          bhi.u = *(const u32x4*)(p_hi + (mt * 16 + r) * RS + (ksl * 32 + kg * 8) * 2);
          blo.u = *(const u32x4*)(p_lo + (mt * 16 + r) * RS + (ksl * 32 + kg * 8) * 2);
#pragma unroll
          for (int j = 0; j < NTO; ++j) acco[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j].v, blo.v, acco[mt][j], 0, 0, 0);
#pragma unroll
          for (int j = 0; j < NTO; ++j) acco[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j].v, bhi.v, acco[mt][j], 0, 0, 0);
        }
      }
      __syncthreads();                                 // planes are rewritten by the next chunk
    }
#pragma unroll
    for (int j = 0; j < NTO; ++j) {
      if (wv * NTO + j >= n_otiles) continue;
      const int col = (wv * NTO + j) * 16 + 4 * kg;
      const float4 b = *(const float4*)(mp.bo + col);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) {
        const int row = mt * 16 + r;
        if (row >= rows_valid) continue;
        *(float4*)(cache_h + (size_t)row * g.dphi + col) =
            make_float4(expf(acco[mt][j][0] + b.x), expf(acco[mt][j][1] + b.y), expf(acco[mt][j][2] + b.z), expf(acco[mt][j][3] + b.w));
      }
    }
    return;
  }
  float4 gcur[4], gnext[4];
  if (EPI == EPI_RES && colw < Nout) {
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) gcur[mt] = *(const float4*)g_ptr(mt, 0);
  }
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (colw + nt * 16 >= Nout) continue;              // (Nout is a multiple of 16: whole column tiles)
    const int col = colw + nt * 16 + 4 * kg;
    const float4 b = *(const float4*)(bias + col);
    if (EPI == EPI_RES && nt + 1 < NT && colw + (nt + 1) * 16 < Nout) {   // the next tile's residual stream, ahead of this tile's stores
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) gnext[mt] = *(const float4*)g_ptr(mt, nt + 1);
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      const int row = mt * 16 + r;
      float4 v = make_float4(acc[mt][nt][0] + b.x, acc[mt][nt][1] + b.y, acc[mt][nt][2] + b.z, acc[mt][nt][3] + b.w);
      if (EPI == EPI_HID) v = make_float4(gelu_erf(v.x), gelu_erf(v.y), gelu_erf(v.z), gelu_erf(v.w));
      if (EPI == EPI_RES) v = make_float4(fmaf(mp.alpha, v.x, gcur[mt].x), fmaf(mp.alpha, v.y, gcur[mt].y),
                                          fmaf(mp.alpha, v.z, gcur[mt].z), fmaf(mp.alpha, v.w, gcur[mt].w));
      if (EPI == EPI_OUT) v = make_float4(expf(v.x), expf(v.y), expf(v.z), expf(v.w));
      if (row >= rows_valid) continue;
      if (EPI == EPI_STEM || EPI == EPI_RES) *(float4*)(Gt + (size_t)row * E + col) = v;
      if (EPI == EPI_HID) *(float4*)(Ht + (size_t)row * E + col) = v;
      if (EPI == EPI_OUT) *(float4*)(cache_h + (size_t)row * g.dphi + col) = v;
    }
    if (EPI == EPI_RES) {
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) gcur[mt] = gnext[mt];
    }
  }
}

// block-wise launch of one layer: grid (Hkv * mlp_block / 64, ceil(Nout / (64 NT))); the activations of the
// whole token block live in the workspace ([Hkv][mlp_block][d_emb] for g, the same for h)
template <int EPI, int NT, int NTO = 0>
__global__ __launch_bounds__(kThreads, 2) void mlp_gemm_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                               char* __restrict__ ws, int p, int t0) {
  __shared__ __attribute__((aligned(16))) char lds_raw[mlp_lds_bytes<NT>()];
  const int h = blockIdx.x % g.Hkv;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int row0 = (blockIdx.x / g.Hkv) * 64;          // first row of the tile inside the token block
  if (t0 + row0 >= n) return;
  const int rows_valid = min(64, n - (t0 + row0));
  const tkphi_mlp mp = pr.mlp_k[h];
  float* Gb = (float*)(ws + g.off_act) + (size_t)h * g.mlp_block * g.d_emb;
  float* Hb = Gb + (size_t)g.Hkv * g.mlp_block * g.d_emb;
  mlp_gemm_tile<EPI, NT, NTO>(g, pr, mp, ws, lds_raw, h, n, t0 + row0, rows_valid, Gb + (size_t)row0 * g.d_emb,
                              Hb + (size_t)row0 * g.d_emb, (int)blockIdx.y * 64 * NT, 0, key_feature_rows(g, pr, ws, 0, h, n));
}

// The whole chain in one launch (d_emb == 64 NT, d_phi == 64 NTO): a tile's layers depend only on the
// tile's own rows, so a persistent workgroup takes a 64-token tile through stem, hidden layer and
// residual + output with workgroup barriers in between; its activations (2 x 64 x d_emb floats of the
// workspace per workgroup) never leave L2.  grid (n_wg); the tiles of the np problems p0 .. p0 + np - 1:
// tile T = blockIdx.x + k n_wg -> problem slot T / tpp, KV head (T % tpp) % Hkv, tokens
// [64 ((T % tpp) / Hkv), + 64), tpp = Hkv ceil(max_mid / 64) (tiles past a shorter problem's end are skipped).
// No launch gaps and one cold start per workgroup (4 % faster than the layer-wise launches; holding back
// every other workgroup at the start so that neighbours on a CU run different phases was measured to
// change nothing).
template <int NT, int NTO>
__global__ __launch_bounds__(kThreads, 2) void mlp_chain_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                char* __restrict__ ws, int p0, int np) {
  __shared__ __attribute__((aligned(16))) char lds_raw[mlp_lds_bytes<NT>()];
  const int tpp = ((g.max_mid + 63) / 64) * g.Hkv;
  float* Gt = (float*)(ws + g.off_act) + (size_t)blockIdx.x * 2 * 64 * g.d_emb;
  float* Ht = Gt + (size_t)64 * g.d_emb;
  for (int T = blockIdx.x; T < tpp * np; T += gridDim.x) {
    const int slot = T / tpp, rem = T % tpp;
    const tkphi_problem pr = probs[p0 + slot];
    if (pr.L < 1 || pr.L > g.max_L) continue;          // (uniform over the workgroup)
    const int n = mid_size(pr.L, g.n_sink, g.n_tail);
    const int h = rem % g.Hkv, tok0 = (rem / g.Hkv) * 64;
    if (tok0 >= n) continue;
    const int rows_valid = min(64, n - tok0);
    const tkphi_mlp mp = pr.mlp_k[h];
    float* feat = key_feature_rows(g, pr, ws, slot, h, n);
    mlp_gemm_tile<EPI_STEM, NT, 0>(g, pr, mp, ws, lds_raw, h, n, tok0, rows_valid, Gt, Ht, 0, slot, feat);
    __syncthreads();                                   // g0 of the tile is visible to the workgroup; LDS is free
    mlp_gemm_tile<EPI_HID, NT, 0>(g, pr, mp, ws, lds_raw, h, n, tok0, rows_valid, Gt, Ht, 0, slot, feat);
    __syncthreads();
    mlp_gemm_tile<EPI_RESOUT, NT, NTO>(g, pr, mp, ws, lds_raw, h, n, tok0, rows_valid, Gt, Ht, 0, slot, feat);
    __syncthreads();                                   // the next tile overwrites g, h and the planes
  }
}

// Decode without a feature cache: the same chain over the retrieved keys.  Tile T -> problem slot T / tpp, query
// head (T % tpp) % Hq, entries [64 ((T % tpp) / Hq), + 64) of that head's retrieved list (tpp = Hq ceil(max_K / 64));
// row i of a head is mid token sel_idx[i], its features go to row i of the head's block of Geom::off_selphi.
template <int NT, int NTO>
__global__ __launch_bounds__(kThreads, 2) void mlp_chain_sel_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                    char* __restrict__ ws, int p0, int np) {
  __shared__ __attribute__((aligned(16))) char lds_raw[mlp_lds_bytes<NT>()];
  const int tpp = ((g.max_K + 63) / 64) * g.Hq;
  float* Gt = (float*)(ws + g.off_act) + (size_t)blockIdx.x * 2 * 64 * g.d_emb;
  float* Ht = Gt + (size_t)64 * g.d_emb;
  for (int T = blockIdx.x; T < tpp * np; T += gridDim.x) {
    const int slot = T / tpp, rem = T % tpp;
    const tkphi_problem pr = probs[p0 + slot];
    if (pr.L < 1 || pr.L > g.max_L) continue;
    const int n = mid_size(pr.L, g.n_sink, g.n_tail);
    const int gq = rem % g.Hq, tok0 = (rem / g.Hq) * 64, h = gq / g.G;
    char* blk = problem_block(g, ws, p0 + slot);
    const int Ksel = min(((const SelPlan*)(blk + g.off_plan))[gq].n_sel, g.max_K);
    if (n == 0 || tok0 >= Ksel) continue;
    const int rows_valid = min(64, Ksel - tok0);
    const tkphi_mlp mp = pr.mlp_k[h];
    const int32_t* rowmap = (const int32_t*)(blk + g.off_selidx) + (size_t)gq * g.max_K;
    float* feat = (float*)(blk + g.off_selphi) + (size_t)gq * g.max_K * g.dphi;
    mlp_gemm_tile<EPI_STEM, NT, 0>(g, pr, mp, ws, lds_raw, h, n, tok0, rows_valid, Gt, Ht, 0, slot, feat, rowmap);
    __syncthreads();
    mlp_gemm_tile<EPI_HID, NT, 0>(g, pr, mp, ws, lds_raw, h, n, tok0, rows_valid, Gt, Ht, 0, slot, feat, rowmap);
    __syncthreads();
    mlp_gemm_tile<EPI_RESOUT, NT, NTO>(g, pr, mp, ws, lds_raw, h, n, tok0, rows_valid, Gt, Ht, 0, slot, feat, rowmap);
    __syncthreads();
  }
}

template <int EPI>
static void launch_mlp_gemm(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s, int rows, int Nout,
                            int p, int t0) {
  // column tiles per wavefront: the smallest power of two whose 64 NT outputs cover Nout, at most 8
  const int nt = Nout > 256 ? 8 : Nout > 128 ? 4 : Nout > 64 ? 2 : 1;
  dim3 grid(g.Hkv * ((rows + 63) / 64), (Nout + 64 * nt - 1) / (64 * nt));
  if (nt == 8) hipLaunchKernelGGL((mlp_gemm_kernel<EPI, 8>), grid, dim3(kThreads), 0, s, g, probs, ws, p, t0);
  else if (nt == 4) hipLaunchKernelGGL((mlp_gemm_kernel<EPI, 4>), grid, dim3(kThreads), 0, s, g, probs, ws, p, t0);
  else if (nt == 2) hipLaunchKernelGGL((mlp_gemm_kernel<EPI, 2>), grid, dim3(kThreads), 0, s, g, probs, ws, p, t0);
  else hipLaunchKernelGGL((mlp_gemm_kernel<EPI, 1>), grid, dim3(kThreads), 0, s, g, probs, ws, p, t0);
}

// residual + output layer in one launch: d_emb == 64 NT (one workgroup spans all of g1; a wavefront's
// 16 NT features are at least one MFMA K step of 32) and d_phi == 64 NTO
static bool resout_fusable(const Geom& g) {
  return (g.d_emb == 128 || g.d_emb == 256 || g.d_emb == 512) && (g.dphi == 64 || g.dphi == 128 || g.dphi == 256);
}

template <int NT>
static void launch_mlp_resout_nt(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s, int rows, int p, int t0) {
  dim3 grid(g.Hkv * ((rows + 63) / 64));
  if (g.dphi == 64) hipLaunchKernelGGL((mlp_gemm_kernel<EPI_RESOUT, NT, 1>), grid, dim3(kThreads), 0, s, g, probs, ws, p, t0);
  else if (g.dphi == 128) hipLaunchKernelGGL((mlp_gemm_kernel<EPI_RESOUT, NT, 2>), grid, dim3(kThreads), 0, s, g, probs, ws, p, t0);
  else hipLaunchKernelGGL((mlp_gemm_kernel<EPI_RESOUT, NT, 4>), grid, dim3(kThreads), 0, s, g, probs, ws, p, t0);
}

template <int NT>
static void launch_mlp_chain_nt(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s, int p0, int np, bool sel) {
  const int64_t tiles = sel ? (int64_t)(g.max_K + 63) / 64 * g.Hq * np : (int64_t)(g.max_mid + 63) / 64 * g.Hkv * np;
  dim3 grid((unsigned)std::min<int64_t>(tiles, kMlpChainWGs));
  if (sel) {
    if (g.dphi == 64) hipLaunchKernelGGL((mlp_chain_sel_kernel<NT, 1>), grid, dim3(kThreads), 0, s, g, probs, ws, p0, np);
    else if (g.dphi == 128) hipLaunchKernelGGL((mlp_chain_sel_kernel<NT, 2>), grid, dim3(kThreads), 0, s, g, probs, ws, p0, np);
    else hipLaunchKernelGGL((mlp_chain_sel_kernel<NT, 4>), grid, dim3(kThreads), 0, s, g, probs, ws, p0, np);
  } else {
    if (g.dphi == 64) hipLaunchKernelGGL((mlp_chain_kernel<NT, 1>), grid, dim3(kThreads), 0, s, g, probs, ws, p0, np);
    else if (g.dphi == 128) hipLaunchKernelGGL((mlp_chain_kernel<NT, 2>), grid, dim3(kThreads), 0, s, g, probs, ws, p0, np);
    else hipLaunchKernelGGL((mlp_chain_kernel<NT, 4>), grid, dim3(kThreads), 0, s, g, probs, ws, p0, np);
  }
}

static void launch_mlp_chain(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s, int p0, int np, bool sel) {
  if (g.d_emb == 512) launch_mlp_chain_nt<8>(g, probs, ws, s, p0, np, sel);
  else if (g.d_emb == 256) launch_mlp_chain_nt<4>(g, probs, ws, s, p0, np, sel);
  else launch_mlp_chain_nt<2>(g, probs, ws, s, p0, np, sel);
}

static void launch_mlp_pack(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s, int p0, int np) {
  const size_t pieces = ((size_t)g.d_emb * g.d + (size_t)2 * g.d_emb * g.d_emb + (size_t)g.dphi * g.d_emb) / 8;
  hipLaunchKernelGGL(mlp_pack_weights_kernel, dim3((unsigned)((pieces + kThreads - 1) / kThreads), g.Hkv, np), dim3(kThreads), 0, s,
                     g, probs, ws, p0);
}

// Build with the MLP maps: the key features of every problem's mid-region (-> phi_cache, or the workspace buffer of
// the group) and their summary contraction (-> chunk partials), group of problems by group.
void launch_mlp_build(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  if (g.max_mid == 0) return;
  // tkphi_tuning::mlp_mode 1: layer-wise launches per problem and token block; 2: also residual and output apart
  const bool fusable = resout_fusable(g) && g.mlp_mode != 2;
  const bool chain = fusable && g.mlp_mode != 1;
  const int group = chain ? g.mlp_group : 1;
  for (int p0 = 0; p0 < g.n_problems; p0 += group) {
    const int np = std::min(group, g.n_problems - p0);
    launch_mlp_pack(g, probs, ws, s, p0, np);
    if (chain) {
      launch_mlp_chain(g, probs, ws, s, p0, np, false);
    } else {
      for (int t0 = 0; t0 < g.max_mid; t0 += g.mlp_block) {
        const int rows = std::min(g.mlp_block, g.max_mid - t0);
        launch_mlp_gemm<EPI_STEM>(g, probs, ws, s, rows, g.d_emb, p0, t0);
        launch_mlp_gemm<EPI_HID>(g, probs, ws, s, rows, g.d_emb, p0, t0);
        if (fusable) {
          if (g.d_emb == 512) launch_mlp_resout_nt<8>(g, probs, ws, s, rows, p0, t0);
          else if (g.d_emb == 256) launch_mlp_resout_nt<4>(g, probs, ws, s, rows, p0, t0);
          else launch_mlp_resout_nt<2>(g, probs, ws, s, rows, p0, t0);
        } else {
          launch_mlp_gemm<EPI_RES>(g, probs, ws, s, rows, g.d_emb, p0, t0);
          launch_mlp_gemm<EPI_OUT>(g, probs, ws, s, rows, g.dphi, p0, t0);
        }
      }
    }
    launch_summary_from_cache(g, probs, ws, s, p0, np);
  }
}

// Decode without a feature cache: phi_k of every query head's retrieved keys -> Geom::off_selphi (after the select)
void launch_mlp_sel_features(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  if (g.max_mid == 0 || g.max_K == 0) return;
  for (int p0 = 0; p0 < g.n_problems; p0 += g.mlp_group) {
    const int np = std::min(g.mlp_group, g.n_problems - p0);
    launch_mlp_pack(g, probs, ws, s, p0, np);
    launch_mlp_chain(g, probs, ws, s, p0, np, true);
  }
}

// ------------------------------------------------------------------------------------
// summary contraction from stored features: grid (n_build_chunks, Hkv, problems of the group), 256
// threads; problem p0 + blockIdx.z, whose features are in its cache or in slot blockIdx.z of the workspace
// buffer; writes the same chunk partials as the other build kernels.
// Tiles of 64 tokens: the feature rows (fp32) are split into bf16 hi / lo and transposed
// in registers (4 tokens x 4 features per load group) into feature-major LDS planes, the
// value tile is transposed as in the fused build; wavefront w owns the feature tiles
// w, w + 4, ...  (FTW = ceil(d_phi / 64) of them); hi and lo are two MFMAs per product.
// ------------------------------------------------------------------------------------
template <int D, int FTW>
__global__ __launch_bounds__(kThreads) void summary_from_cache_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                      char* __restrict__ ws, int p0) {
  constexpr int CT = D / 16, SEGS = D / 8;
  constexpr int TROW = 64 * 2 + 16;                // bytes per staged row of 64 tokens
  constexpr int QMAX = FTW * 4 / 4;                // feature quads per thread: dphi / 4 / 16 <= FTW
  extern __shared__ __attribute__((aligned(16))) char lds[];   // f_hi [dphi][TROW], f_lo [dphi][TROW], v_t [D][TROW]
  const int ch = blockIdx.x, h = blockIdx.y, p = p0 + blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  const int n = mid_size(pr.L, g.n_sink, g.n_tail);
  const int c0 = ch * g.build_chunk;
  if (c0 >= n) return;
  const int c1 = min(n, c0 + g.build_chunk);
  const int dphi = g.dphi, NFT = dphi / 16;
  char* f_hi = lds;
  char* f_lo = lds + (size_t)dphi * TROW;
  char* v_t = lds + (size_t)2 * dphi * TROW;
  const int lane = tid & 63, wv = tid >> 6, r = lane & 15, kg = lane >> 4;

  floatx4 sacc[FTW][CT];
#pragma unroll
  for (int k = 0; k < FTW; ++k)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) sacc[k][ct] = (floatx4){0.f, 0.f, 0.f, 0.f};
  float usum[QMAX][4];
#pragma unroll
  for (int k = 0; k < QMAX; ++k)
#pragma unroll
    for (int e = 0; e < 4; ++e) usum[k][e] = 0.f;

  const int tq = tid % 16, fs = tid / 16;          // tokens 4tq .. 4tq+3 of the tile; feature quads fs, fs + 16, ...
  const float* cache_h = key_feature_rows(g, pr, ws, (int)blockIdx.z, h, n);
  const size_t row_bytes = (size_t)pr.stride_tok * 2;
  const bool v_active = tid < 16 * SEGS;
  const int sg = tid / 16;
  const char* Vb = (const char*)pr.V + ((size_t)h * pr.stride_head + (size_t)g.n_sink * pr.stride_tok) * 2 + (size_t)sg * 16;

  for (int t0 = c0; t0 < c1; t0 += 64) {
    // ---- loads: 4 tokens x (QMAX feature quads + one 16-byte value segment) ----------------------
    u32x4 fq[QMAX][4], vv[4];
#pragma unroll
    for (int k = 0; k < QMAX; ++k) {
      const int q4 = min(fs + 16 * k, dphi / 4 - 1);
#pragma unroll
      for (int i = 0; i < 4; ++i) fq[k][i] = gload128(cache_h + (size_t)min(t0 + tq * 4 + i, c1 - 1) * dphi + q4 * 4);
    }
    if (v_active) {
#pragma unroll
      for (int i = 0; i < 4; ++i) vv[i] = gload128(Vb + (size_t)min(t0 + tq * 4 + i, c1 - 1) * row_bytes);
    }
    const bool ok[4] = {t0 + tq * 4 + 0 < c1, t0 + tq * 4 + 1 < c1, t0 + tq * 4 + 2 < c1, t0 + tq * 4 + 3 < c1};
    __syncthreads();                                // the previous tile's readers are done
#pragma unroll
    for (int k = 0; k < QMAX; ++k) {
      const int q4 = fs + 16 * k;
      if (q4 < dphi / 4) {
        float f[4][4];                              // [token][feature of the quad]
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f[i][0] = ok[i] ? __uint_as_float(fq[k][i].x) : 0.f; f[i][1] = ok[i] ? __uint_as_float(fq[k][i].y) : 0.f;
          f[i][2] = ok[i] ? __uint_as_float(fq[k][i].z) : 0.f; f[i][3] = ok[i] ? __uint_as_float(fq[k][i].w) : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          usum[k][e] += (f[0][e] + f[1][e]) + (f[2][e] + f[3][e]);
          uint32_t h01, l01, h23, l23;
          split_bf16_pair(f[0][e], f[1][e], &h01, &l01);
          split_bf16_pair(f[2][e], f[3][e], &h23, &l23);
          *(u32x2*)(f_hi + (q4 * 4 + e) * TROW + tq * 8) = (u32x2){h01, h23};
          *(u32x2*)(f_lo + (q4 * 4 + e) * TROW + tq * 8) = (u32x2){l01, l23};
        }
      }
    }
    if (v_active) {
      uint32_t w[4][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        w[i][0] = ok[i] ? vv[i].x : 0u; w[i][1] = ok[i] ? vv[i].y : 0u;
        w[i][2] = ok[i] ? vv[i].z : 0u; w[i][3] = ok[i] ? vv[i].w : 0u;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {      // dword q of a token holds channels 2q (low half) and 2q+1 (high half)
        const u32x2 even = (u32x2){(w[0][q] & 0xffffu) | (w[1][q] << 16), (w[2][q] & 0xffffu) | (w[3][q] << 16)};
        const u32x2 odd = (u32x2){(w[0][q] >> 16) | (w[1][q] & 0xffff0000u), (w[2][q] >> 16) | (w[3][q] & 0xffff0000u)};
        *(u32x2*)(v_t + (sg * 8 + 2 * q) * TROW + tq * 8) = even;
        *(u32x2*)(v_t + (sg * 8 + 2 * q + 1) * TROW + tq * 8) = odd;
      }
    }
    __syncthreads();
    // ---- S[own feature tiles][all channels] += Phi^T V over the tile's 64 tokens -------------------
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int k = 0; k < FTW; ++k) {
        const int ft = wv + 4 * k;
        if (ft < NFT) {
          Frag ahi, alo;
          ahi.u = *(const u32x4*)(f_hi + (ft * 16 + r) * TROW + (32 * ks + 8 * kg) * 2);
          alo.u = *(const u32x4*)(f_lo + (ft * 16 + r) * TROW + (32 * ks + 8 * kg) * 2);
#pragma unroll
          for (int ct = 0; ct < CT; ++ct) {
            Frag vb;
            vb.u = *(const u32x4*)(v_t + (ct * 16 + r) * TROW + (32 * ks + 8 * kg) * 2);
            sacc[k][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(alo.v, vb.v, sacc[k][ct], 0, 0, 0);
            sacc[k][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ahi.v, vb.v, sacc[k][ct], 0, 0, 0);
          }
        }
      }
    }
  }

  // ---- chunk partial: S part [dphi][D] then u part [dphi] ------------------------------------------
  float* bp = (float*)(ws + g.off_bpart) + ((size_t)(p * g.Hkv + h) * g.n_build_chunks + ch) * ((size_t)dphi * (D + 1));
#pragma unroll
  for (int k = 0; k < FTW; ++k) {
    const int ft = wv + 4 * k;
    if (ft < NFT) {
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int i = 0; i < 4; ++i) bp[(size_t)(ft * 16 + 4 * kg + i) * D + ct * 16 + r] = sacc[k][ct][i];
    }
  }
#pragma unroll
  for (int k = 0; k < QMAX; ++k) {
    const int q4 = fs + 16 * k;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float x = usum[k][e];
      x += __shfl_xor(x, 1); x += __shfl_xor(x, 2); x += __shfl_xor(x, 4); x += __shfl_xor(x, 8);
      if (tq == 0 && q4 < dphi / 4) bp[(size_t)dphi * D + q4 * 4 + e] = x;
    }
  }
}

// ------------------------------------------------------------------------------------
// phi_q of every query head (decode side): the same chain as matrix-vector products in fp32,
// three launches so that each layer is spread over the chip.  grid (slices, Hq, n_problems),
// 1024 threads; a workgroup owns 64 output rows of its layer:
//   stage 0: g0 = Ws q + bs (every workgroup of the head recomputes it: 2 d d_emb bytes from L2),
//            h[rows] = GeLU(W1[rows] g0 + b1[rows]); slice 0 also stores g0
//   stage 1: g[rows] = g0[rows] + alpha (W2[rows] h + b2[rows])
//   stage 2: phi_q[rows] = exp(Wo[rows] g + bo[rows])
// ------------------------------------------------------------------------------------
// Every global load of a workgroup (weights of its first row groups, biases, input vector) is
// issued before anything is consumed: one memory round trip per launch.
template <int STAGE, int SPL>   // SPL = 1 for d_emb <= 512, 2 for 1024
__global__ __launch_bounds__(kSelThreads) void mlp_phi_q_kernel(Geom g, const tkphi_problem* __restrict__ probs,
                                                                char* __restrict__ ws) {
  __shared__ float xs[128];
  __shared__ float vin[1024], sb[1024];
  __shared__ float sb2[64], sg[64];
  const int gq = blockIdx.y, p = blockIdx.z, tid = threadIdx.x;
  const tkphi_problem pr = probs[p];
  if (pr.L < 1 || pr.L > g.max_L) return;
  char* blk = problem_block(g, ws, p);
  const int E = g.d_emb;
  float* gbuf = (float*)(blk + g.off_mlpq) + (size_t)gq * 2 * E;
  float* hbuf = gbuf + E;
  const tkphi_mlp mp = pr.mlp_q[gq];
  const int j0 = blockIdx.x * 64;
  const int nrows = min(64, (STAGE == 2 ? g.dphi : E) - j0);
  const char* Wslice = (const char*)(STAGE == 0 ? mp.W1 : STAGE == 1 ? mp.W2 : mp.Wo) + (size_t)j0 * E * 2;
  const float* bslice = (STAGE == 0 ? mp.b1 : STAGE == 1 ? mp.b2 : mp.bo) + j0;
  u32x4 ts[8], tw[8];
  if (STAGE == 0) gemv_load<1>(mp.Ws, E, g.d, 0, ts);
  gemv_load<SPL>(Wslice, nrows, E, 0, tw);
  if (tid < 64) sb2[tid] = bslice[min(tid, nrows - 1)];
  if (STAGE == 0) {
    if (tid < g.d) xs[tid] = Elem<uint16_t>::load1(pr.q, (int64_t)gq * g.d + tid);
    if (tid < E) sb[tid] = mp.bs[tid];
    __syncthreads();
    gemv_bf16_rows<1>(mp.Ws, E, g.d, xs, ts, [&](int j, float dot) { vin[j] = dot + sb[j]; });
    __syncthreads();
    if (blockIdx.x == 0 && tid < E) gbuf[tid] = vin[tid];
    gemv_bf16_rows<SPL>(Wslice, nrows, E, vin, tw, [&](int j, float dot) { hbuf[j0 + j] = gelu_erf(dot + sb2[j]); });
  } else if (STAGE == 1) {
    if (tid < E) vin[tid] = hbuf[tid];
    if (tid < 64) sg[tid] = gbuf[j0 + min(tid, nrows - 1)];
    __syncthreads();
    gemv_bf16_rows<SPL>(Wslice, nrows, E, vin, tw, [&](int j, float dot) { gbuf[j0 + j] = fmaf(mp.alpha, dot + sb2[j], sg[j]); });
  } else {
    if (tid < E) vin[tid] = gbuf[tid];
    __syncthreads();
    float* phiq = (float*)(blk + g.off_phiq) + (size_t)gq * g.dphi;
    gemv_bf16_rows<SPL>(Wslice, nrows, E, vin, tw, [&](int j, float dot) { phiq[j0 + j] = expf(dot + sb2[j]); });
  }
}

void launch_mlp_phi_q(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s) {
  dim3 ge(g.d_emb / 64, g.Hq, g.n_problems), go((g.dphi + 63) / 64, g.Hq, g.n_problems);
  KernelTimer* t = g_kernel_timer;            // the three launches are one timed stage
  if (t) t->used[ST_PHIQ] = true;
  hipEvent_t e0 = t ? t->start[ST_PHIQ] : nullptr, e1 = t ? t->stop[ST_PHIQ] : nullptr;
  if (g.d_emb <= 512) {
    hipExtLaunchKernelGGL((mlp_phi_q_kernel<0, 1>), ge, dim3(kSelThreads), 0, s, e0, nullptr, 0, g, probs, ws);
    hipLaunchKernelGGL((mlp_phi_q_kernel<1, 1>), ge, dim3(kSelThreads), 0, s, g, probs, ws);
    hipExtLaunchKernelGGL((mlp_phi_q_kernel<2, 1>), go, dim3(kSelThreads), 0, s, nullptr, e1, 0, g, probs, ws);
  } else {
    hipExtLaunchKernelGGL((mlp_phi_q_kernel<0, 2>), ge, dim3(kSelThreads), 0, s, e0, nullptr, 0, g, probs, ws);
    hipLaunchKernelGGL((mlp_phi_q_kernel<1, 2>), ge, dim3(kSelThreads), 0, s, g, probs, ws);
    hipExtLaunchKernelGGL((mlp_phi_q_kernel<2, 2>), go, dim3(kSelThreads), 0, s, nullptr, e1, 0, g, probs, ws);
  }
}

template <int D, int FTW>
static void launch_sfc(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s, int p0, int np) {
  dim3 grid(g.n_build_chunks, g.Hkv, np);
  const size_t lds = (size_t)(2 * g.dphi + g.d) * (64 * 2 + 16);
  if (lds > 48 * 1024) {
    const hipError_t e = hipFuncSetAttribute((const void*)summary_from_cache_kernel<D, FTW>,
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) { set_error("hipFuncSetAttribute(%zu bytes of LDS): %s", lds, hipGetErrorString(e)); return; }
  }
  hipLaunchKernelGGL((summary_from_cache_kernel<D, FTW>), grid, dim3(kThreads), lds, s, g, probs, ws, p0);
}

void launch_summary_from_cache(const Geom& g, const tkphi_problem* probs, char* ws, hipStream_t s, int p0, int np) {
  if (g.max_mid == 0) return;
  const int ftw = (g.dphi + 63) / 64;              // feature tiles per wavefront: 1, 2 or (3, 4 ->) 4
  if (g.d == 128) { if (ftw <= 1) launch_sfc<128, 1>(g, probs, ws, s, p0, np); else if (ftw == 2) launch_sfc<128, 2>(g, probs, ws, s, p0, np); else launch_sfc<128, 4>(g, probs, ws, s, p0, np); }
  else { if (ftw <= 1) launch_sfc<64, 1>(g, probs, ws, s, p0, np); else if (ftw == 2) launch_sfc<64, 2>(g, probs, ws, s, p0, np); else launch_sfc<64, 4>(g, probs, ws, s, p0, np); }
}

}  // namespace tkphi
