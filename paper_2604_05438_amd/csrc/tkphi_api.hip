// Host layer of libtkphi: argument validation, launch geometry / workspace planning and
// the extern "C" entry points declared in include/tkphi.h.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "tkphi_internal.h"

namespace tkphi {

static thread_local char g_last_error[512] = "";
thread_local KernelTimer* g_kernel_timer = nullptr;

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
  va_end(ap);
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

tkphi_status make_geom(const tkphi_config* cfg, int n_problems, int max_L, int max_K, Geom* g) {
  if (!cfg) { set_error("cfg is null"); return TKPHI_EINVAL; }
  if (n_problems < 0 || max_L < 1 || max_K < 0) {
    set_error("n_problems=%d max_L=%d max_K=%d out of range", n_problems, max_L, max_K);
    return TKPHI_EINVAL;
  }
  if (cfg->kv_dtype != TKPHI_F32 && cfg->kv_dtype != TKPHI_BF16) {
    set_error("kv_dtype=%d is not a tkphi_dtype", cfg->kv_dtype);
    return TKPHI_EINVAL;
  }
  if (cfg->n_kv_heads < 1 || cfg->n_q_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads != 0 ||
      cfg->n_q_heads / cfg->n_kv_heads > kMaxGroup) {
    set_error("head counts %d/%d unsupported (need Hq %% Hkv == 0, ratio <= %d)", cfg->n_q_heads,
              cfg->n_kv_heads, kMaxGroup);
    return TKPHI_ESHAPE;
  }
  if (cfg->d_head != 64 && cfg->d_head != 128) {
    set_error("d_head=%d unsupported (64 or 128)", cfg->d_head);
    return TKPHI_ESHAPE;
  }
  if (cfg->d_phi < 16 || cfg->d_phi > kMaxDim || cfg->d_phi % 16 != 0) {
    set_error("d_phi=%d unsupported (multiple of 16 in [16, %d])", cfg->d_phi, kMaxDim);
    return TKPHI_ESHAPE;
  }
  if (cfg->phi_kind != TKPHI_PHI_EXP_AFFINE && cfg->phi_kind != TKPHI_PHI_MLP) {
    set_error("phi_kind=%d is not a tkphi_phi_kind", cfg->phi_kind);
    return TKPHI_EINVAL;
  }
  if (cfg->phi_kind == TKPHI_PHI_MLP) {
    if (cfg->kv_dtype != TKPHI_BF16) {
      set_error("the MLP feature maps need bf16 storage");
      return TKPHI_EUNSUPPORTED;
    }
    if (cfg->d_emb < 64 || cfg->d_emb > 1024 || (cfg->d_emb & (cfg->d_emb - 1)) != 0) {
      set_error("d_emb=%d unsupported (a power of two in [64, 1024])", cfg->d_emb);
      return TKPHI_ESHAPE;
    }
    // decode recomputes retrieved-key features with the one-launch chain only (the widths it is built for)
    const bool chain_widths = (cfg->d_emb == 128 || cfg->d_emb == 256 || cfg->d_emb == 512) && cfg->d_phi <= 256;
    if (!cfg->cache_features && !chain_widths) {
      set_error("the MLP feature maps without cache_features need d_emb in {128, 256, 512} and d_phi <= 256 "
                "(d_emb=%d, d_phi=%d)", cfg->d_emb, cfg->d_phi);
      return TKPHI_EUNSUPPORTED;
    }
  }
  if (cfg->max_gen < 0 || cfg->max_gen > (1 << 20)) { set_error("max_gen=%d out of range [0, 2^20]", cfg->max_gen); return TKPHI_EINVAL; }
  const tkphi_tuning& tn = cfg->tuning;
  if (tn.force_generic < 0 || tn.force_generic > 1 || tn.scan_chunk < 0 || tn.scan_chunk > 32768 || tn.interleave < 0 ||
      tn.interleave > 2 || tn.build_chunk < 0 || tn.build_chunk > (1 << 20) || tn.mlp_block < 0 || tn.mlp_block > 8192 ||
      tn.mlp_mode < 0 || tn.mlp_mode > 2 || tn.select_mode < 0 || tn.select_mode > 2 || tn.select_test < 0 || tn.select_test > 2) {
    set_error("tuning field out of range (force_generic=%d scan_chunk=%d interleave=%d build_chunk=%d mlp_block=%d mlp_mode=%d "
              "select_mode=%d select_test=%d)", tn.force_generic, tn.scan_chunk, tn.interleave, tn.build_chunk, tn.mlp_block,
              tn.mlp_mode, tn.select_mode, tn.select_test);
    return TKPHI_EINVAL;
  }
  for (int i = 0; i < 4; ++i)
    if (tn.reserved[i] != 0) { set_error("tuning.reserved[%d] must be 0", i); return TKPHI_EINVAL; }
  if (n_problems > 65535) { set_error("n_problems=%d exceeds 65535", n_problems); return TKPHI_ESHAPE; }
  if (cfg->n_sink < 0 || cfg->n_tail < 0) {
    set_error("n_sink=%d n_tail=%d must be >= 0", cfg->n_sink, cfg->n_tail);
    return TKPHI_EINVAL;
  }
  memset(g, 0, sizeof(*g));
  g->Hq = cfg->n_q_heads; g->Hkv = cfg->n_kv_heads; g->G = g->Hq / g->Hkv;
  g->d = cfg->d_head; g->dphi = cfg->d_phi; g->n_sink = cfg->n_sink; g->n_tail = cfg->n_tail;
  g->dtype = cfg->kv_dtype;
  g->cache = cfg->cache_features ? 1 : 0;
  g->phi_kind = cfg->phi_kind; g->d_emb = cfg->d_emb;
  g->max_gen = cfg->max_gen;
  g->mlp_mode = tn.mlp_mode;
  g->use_mfma = (cfg->kv_dtype == TKPHI_BF16 && cfg->d_phi == cfg->d_head && !tn.force_generic) ? 1 : 0;
  g->n_problems = n_problems; g->max_L = max_L;
  const int64_t mid = (int64_t)max_L - cfg->n_sink - cfg->n_tail;
  g->max_mid = (int)std::max<int64_t>(mid, 0);
  g->max_K = max_K;
  g->mid_stride = (int)align_up((size_t)std::max(g->max_mid, 1), 64);
  g->score_scale = cfg->score_scale; g->a = cfg->phi_in_scale; g->c = cfg->phi_norm_coef;

  const int64_t units = (int64_t)g->max_mid * g->Hkv * std::max(n_problems, 1);
  // score_mid: about 1024 workgroups, 256..8192 tokens each (uint16 chunk histograms: < 65536)
  int sc = (int)align_up((size_t)std::clamp<int64_t>(ceil_div(units, 1024), 256, 8192), 256);
  if (tn.scan_chunk > 0) sc = tn.scan_chunk;
  // matrix-core score kernel: 4 wavefronts x 64 (d = 128) or 128 (d = 64) tokens per iteration;
  // a chunk is a whole number of such units
  g->scan_unit = g->use_mfma ? (g->d == 128 ? 256 : 512) : 256;
  g->scan_chunk = std::clamp((int)align_up((size_t)std::max(sc, 1), g->scan_unit), g->scan_unit, 32768);
  while (ceil_div(g->max_mid, g->scan_chunk) > kMaxScanChunks && g->scan_chunk < 32768) g->scan_chunk *= 2;
  if (ceil_div(g->max_mid, g->scan_chunk) > kMaxScanChunks) {
    set_error("max_L=%d too long: more than %d score chunks of 32768 tokens", max_L, kMaxScanChunks);
    return TKPHI_ESHAPE;
  }
  g->n_scan_chunks = (int)std::max<int64_t>(1, ceil_div(g->max_mid, g->scan_chunk));
  // with many chunks per head (one long sequence) the workgroups read neighbouring rows at any
  // moment instead of 1024 far-apart ranges: measured 5 % faster; with few chunks per head
  // (many problems) contiguous ranges are faster
  g->interleave = tn.interleave ? (tn.interleave == 1 ? 1 : 0) : (g->use_mfma && g->scan_unit < g->scan_chunk && g->n_scan_chunks >= 64) ? 1 : 0;
  if (!g->use_mfma || g->scan_unit >= g->scan_chunk) g->interleave = 0;
  // filtered pipeline: where the matrix-core score kernel applies.  Chosen by default where it measured faster
  // than the spill pipeline: a budget of at most 1/64 of the mid-region (128K layer: 86 / 89 against 95 / 100 us
  // per step at 0.5 / 1 %; 32K layer 42.5 against 44.5 us; 28 layers per call 1.62 against 1.87 ms; the ragged
  // 256-problem batch 3.36 against 3.65 ms).  At 2 % and 4 % candidate lists overflow their compact heads and the
  // fused select falls back to its general path: 110 / 124 against 108 / 123 us
  g->filtered = (g->use_mfma && cfg->phi_kind == TKPHI_PHI_EXP_AFFINE && !g->cache && tn.select_mode != 1 &&
                 (tn.select_mode == 2 || (int64_t)max_K * 64 <= g->max_mid)) ? 1 : 0;
  g->sel_test = tn.select_test;
  // gather: tiles of kPairsPerWG retrieved tokens per query head
  g->n_tiles = (int)ceil_div(std::min<int64_t>(max_K, g->max_mid), kPairsPerWG);
  // (filtered pipeline: the workgroups that share a query head in the fused select + gather kernel, one
  // partial each: about one workgroup per CU for a single layer, one per head in big batches)
  g->sg_split = g->filtered ? std::clamp(256 / std::max(1, g->Hq * std::max(n_problems, 1)), 1, 16) : 0;
  g->n_atiles = (int)std::max<int64_t>(1, ceil_div(std::min<int64_t>((int64_t)cfg->n_sink + cfg->n_tail, max_L) + cfg->max_gen, 64));
  // summary_build: 512 workgroups fill the chip (2 per CU); larger jobs get about 2048 chunks of at
  // least 2048 tokens so that the last, partly filled round of workgroups stays a small share
  const int64_t bc_small = std::clamp<int64_t>(ceil_div(units, 512), 256, 2048);
  int bc = (int)align_up((size_t)std::clamp<int64_t>(ceil_div(units, 2048), bc_small, 1 << 20), 64);
  if (!g->use_mfma) bc = std::min(bc, 4096);    // fp32 FMA chains stay short on the generic kernel
  // Several resident rounds of the matrix-core kernel (512 workgroup slots at d = 128, 1024 at d = 64): among the
  // chunk counts within two of that guess, the one whose last round is fullest (28 layers of 128K: 9 chunks per head
  // = 2016 workgroups = 3.94 rounds instead of 10 = 4.375, which pays for 5)
  if (g->use_mfma && cfg->phi_kind == TKPHI_PHI_EXP_AFFINE && g->max_mid > 0) {
    const int64_t slots = g->d == 64 ? 1024 : 512, heads = (int64_t)g->Hkv * std::max(n_problems, 1);
    const int64_t c0 = ceil_div(g->max_mid, bc);
    if (c0 * heads > slots) {
      double best_fill = -1.0;
      int best_bc = bc;
      for (int64_t c = std::max<int64_t>(1, c0 - 2); c <= c0 + 2; ++c) {
        const int cand = (int)align_up((size_t)std::max<int64_t>(256, ceil_div(g->max_mid, c)), 64);
        const int64_t wgs = ceil_div(g->max_mid, cand) * heads;
        const double fill = (double)wgs / (double)(ceil_div(wgs, slots) * slots);
        if (fill > best_fill + 1e-9 || (std::fabs(fill - best_fill) <= 1e-9 && std::abs(cand - bc) < std::abs(best_bc - bc))) {
          best_fill = fill; best_bc = cand;
        }
      }
      bc = best_bc;
    }
  }
  if (tn.build_chunk > 0) bc = tn.build_chunk;
  g->build_chunk = std::max(64, bc / 64 * 64);
  g->n_build_chunks = (int)std::max<int64_t>(1, ceil_div(g->max_mid, g->build_chunk));
  g->part_stride = 2 * g->d + 4;

  // workspace layout
  size_t off = 0;
  g->off_status = off; off += 4096;
  g->off_problem0 = off;
  size_t p = 0;
  g->off_scores = p;
  g->off_candf = p;     // (the two pipelines never run in the same call)
  p = align_up(p + std::max((size_t)g->Hq * g->mid_stride * sizeof(float),
                            g->filtered ? (size_t)g->Hq * g->n_scan_chunks * g->scan_chunk * sizeof(uint2) : (size_t)0), 256);
  // compact part of a candidate list: 24 entries, or 3/32 of the list's capacity if that is more (about three
  // times the expected length); with 128 chunks per head the compact lists of a head are one sweep of the
  // fused select + gather kernel
  g->cand_T = (int)align_up((size_t)std::max(24, g->scan_chunk / 4 * 3 / 32), 12);
  g->head_strip = (size_t)4 * g->G * g->cand_T * sizeof(uint2) <= 32768 ? 1 : 0;
  // Non-temporal key loads leave the candidate lists, phi_q and the problem record in the caches for the select kernel
  // (l3b_128k: score pass unchanged, select 25.5 -> 24.9 us, step -1.4 us).  Only for one problem of 256-byte rows:
  // with 128-byte rows the two loads that share a cache line fetch it twice (ragged batch: score pass +20 %), and
  // the 28-layer call measured 2 % slower
  g->stream_keys = (n_problems == 1 && g->d == 128) ? 1 : 0;
  g->off_candc = p;   p = align_up(p + (g->filtered ? (size_t)g->Hq * g->n_scan_chunks * 4 * g->cand_T * sizeof(uint2) : (size_t)0), 256);
  g->off_ccount = p;  p = align_up(p + (g->filtered ? (size_t)g->Hq * g->n_scan_chunks * 4 * sizeof(uint32_t) : (size_t)0), 256);
  g->off_resf = p;    p = align_up(p + (g->filtered ? (size_t)g->Hq * g->n_scan_chunks * g->scan_chunk * sizeof(uint2) : (size_t)0), 256);
  g->off_resc = p;    p = align_up(p + (g->filtered ? (size_t)g->Hq * g->n_scan_chunks * 4 * g->cand_T * sizeof(uint2) : (size_t)0), 256);
  g->off_rescount = p; p = align_up(p + (g->filtered ? (size_t)g->Hq * g->n_scan_chunks * 4 * sizeof(uint32_t) : (size_t)0), 256);
  g->off_thr = p;     p = align_up(p + (size_t)g->Hq * sizeof(uint32_t), 256);
  g->off_mcount = p;  p = align_up(p + (size_t)g->Hq * sizeof(uint32_t), 256);
  g->off_sphi = p;    p = align_up(p + (size_t)g->Hq * g->d * sizeof(float), 256);
  g->off_uphi = p;    p = align_up(p + (size_t)g->Hq * sizeof(float), 256);
  g->off_hist = p;    p = align_up(p + (size_t)g->n_scan_chunks * g->Hq * kBins * sizeof(uint16_t), 256);
  g->off_plan = p;    p = align_up(p + (size_t)g->Hq * sizeof(SelPlan), 256);
  g->off_diag = p;    p = align_up(p + (size_t)g->n_scan_chunks * g->Hq * 4 * sizeof(float), 256);
  g->off_chunkoff = p; p = align_up(p + (size_t)g->Hq * g->n_scan_chunks * 2 * sizeof(int32_t), 256);
  g->off_cand = p;    p = align_up(p + (size_t)g->Hq * kCandCap * sizeof(uint2), 256);
  g->off_selidx = p;  p = align_up(p + (size_t)g->Hq * std::max(max_K, 1) * sizeof(int32_t), 256);
  g->off_selscore = p; p = align_up(p + (size_t)g->Hq * std::max(max_K, 1) * sizeof(float), 256);
  g->off_phiq = p;    p = align_up(p + (size_t)g->Hq * g->dphi * sizeof(float), 256);
  g->off_mlpq = p;    p = align_up(p + (size_t)g->Hq * 2 * g->d_emb * sizeof(float), 256);
  g->sel_feat = cfg->phi_kind == TKPHI_PHI_MLP && !g->cache;
  g->off_selphi = p;  p = align_up(p + (g->sel_feat ? (size_t)g->Hq * std::max(max_K, 1) * g->dphi * sizeof(float) : (size_t)0), 256);
  g->off_part = p;
  p = align_up(p + (size_t)g->Hq * (std::max(g->n_tiles, g->sg_split) + g->n_atiles) * g->part_stride * sizeof(float), 256);
  g->per_problem = p;
  const size_t decode_total = g->off_problem0 + (size_t)std::max(n_problems, 1) * g->per_problem;
  size_t decode_all = decode_total;
  g->off_bpart = g->off_problem0;
  const size_t build_total = g->off_bpart + (size_t)std::max(n_problems, 1) * g->Hkv * g->n_build_chunks *
                                                (size_t)g->dphi * (g->d + 1) * sizeof(float);
  size_t build_all = build_total;
  if (cfg->phi_kind == TKPHI_PHI_MLP) {
    // the fp32 activations of a token block (g and h, every KV head) are written by one GEMM launch and
    // read by the next: a block of about 64 MB stays in the 256 MB last-level cache between the
    // launches, but a launch should also bring two 64-token workgroups per CU (512 in all), which
    // measured faster than the smaller block (4.6 against 6.5 ms for 8 KV heads of 131004 tokens)
    const int64_t blk = std::max<int64_t>(((int64_t)64 << 20) / ((int64_t)2 * g->Hkv * g->d_emb * sizeof(float)),
                                          (int64_t)512 * 64 / g->Hkv);
    g->mlp_block = (int)std::clamp<int64_t>((tn.mlp_block > 0 ? tn.mlp_block : (int)blk) / 64 * 64, 64, 8192);
    // (the activations, the packed weights and the feature buffer lie behind the decode blocks as well: a decode
    // without a feature cache sends the retrieved keys through the same chain)
    g->off_act = align_up(std::max(build_total, decode_total), 256);
    // (or, for the one-launch build, 2 x 64 x d_emb floats per persistent workgroup)
    const size_t act_bytes = std::max((size_t)2 * g->Hkv * g->mlp_block, (size_t)2 * 64 * kMlpChainWGs) * g->d_emb * sizeof(float);
    g->off_wpack = align_up(g->off_act + act_bytes, 256);
    // Problems per chain launch: their packed weights (and, without a feature cache, the features of their
    // mid-regions, fp32) are held together; up to 16 problems, the feature buffer at most 1 GiB (one problem if a
    // single one is larger).
    const size_t wpack_one = (size_t)g->Hkv * ((size_t)g->d_emb * g->d + (size_t)2 * g->d_emb * g->d_emb + (size_t)g->dphi * g->d_emb) * 2;
    const size_t feat_one = g->cache ? 0 : (size_t)g->Hkv * std::max<int64_t>(g->max_mid, 1) * g->dphi * sizeof(float);
    g->mlp_group = std::clamp(n_problems, 1, 16);
    if (feat_one > 0) g->mlp_group = (int)std::clamp<size_t>(((size_t)1 << 30) / feat_one, 1, (size_t)g->mlp_group);
    g->off_feat = align_up(g->off_wpack + (size_t)g->mlp_group * wpack_one, 256);
    build_all = g->off_feat + (size_t)g->mlp_group * feat_one;
    if (g->sel_feat) decode_all = g->off_feat;          // activations and packed weights
  }
  g->decode_bytes = align_up(decode_all, 256);
  g->build_bytes = align_up(build_all, 256);
  g->total_bytes = align_up(std::max(decode_all, build_all), 256);
  return TKPHI_OK;
}

static tkphi_status check_call(const tkphi_problem* problems, int n_problems, const void* ws,
                               size_t ws_bytes, const Geom& g, size_t need = 0) {
  if (need == 0) need = g.total_bytes;
  if (n_problems > 0 && !problems) { set_error("problems is null"); return TKPHI_EINVAL; }
  if (!ws) { set_error("workspace is null"); return TKPHI_EWORKSPACE; }
  if (((uintptr_t)ws) % 256 != 0) { set_error("workspace must be 256-byte aligned"); return TKPHI_EWORKSPACE; }
  if (ws_bytes < need) {
    set_error("workspace too small: %zu < %zu bytes", ws_bytes, need);
    return TKPHI_EWORKSPACE;
  }
  if (((uintptr_t)problems) % 8 != 0) { set_error("problem table must be 8-byte aligned"); return TKPHI_EALIGN; }
  return TKPHI_OK;
}

static tkphi_status hip_ok(hipError_t e, const char* what) {
  if (e == hipSuccess) return TKPHI_OK;
  set_error("%s: %s", what, hipGetErrorString(e));
  return TKPHI_EHIP;
}

}  // namespace tkphi

using namespace tkphi;

extern "C" {

size_t tkphi_workspace_bytes(const tkphi_config* cfg, int32_t n_problems, int32_t max_L, int32_t max_K) {
  Geom g;
  if (make_geom(cfg, n_problems, max_L, max_K, &g) != TKPHI_OK) return 0;
  return g.total_bytes;
}

tkphi_status tkphi_build_summaries(const tkphi_config* cfg, const tkphi_problem* problems,
                                   int32_t n_problems, int32_t max_L, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
  Geom g;
  tkphi_status st = make_geom(cfg, n_problems, max_L, 0, &g);
  if (st != TKPHI_OK) return st;
  st = check_call(problems, n_problems, workspace, workspace_bytes, g, g.build_bytes);   // (the decode scratch depends on max_K)
  if (st != TKPHI_OK) return st;
  if (n_problems == 0) return TKPHI_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  (void)hipGetLastError();
  launch_build(g, problems, (char*)workspace, s);
  return hip_ok(hipGetLastError(), "tkphi_build_summaries launch");
}

// The kernels of one decode call in stream order.  With the MLP feature maps the three phi_q
// launches (a chain of small cold-weight matrix-vector products, ~30 us if serialised) go to a
// second stream of the library's own that forks from `s` at the start of the call and joins
// before the gather, so that they run beside the score pass.  One such stream and event pair per
// device, created on first use at the default priority and kept until the process ends; MLP decode
// calls hold a mutex while they enqueue (the events are shared).
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
};
static std::mutex g_side_mutex;
static SideStream g_side[64];

static tkphi_status side_stream(SideStream** out) {
  int dev = 0;
  tkphi_status st = hip_ok(hipGetDevice(&dev), "hipGetDevice");
  if (st != TKPHI_OK) return st;
  if (dev < 0 || dev >= 64) { set_error("device ordinal %d out of range", dev); return TKPHI_EINVAL; }
  SideStream& ss = g_side[dev];
  if (!ss.stream) {
    hipStream_t str = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    st = hip_ok(hipStreamCreateWithFlags(&str, hipStreamNonBlocking), "hipStreamCreateWithFlags");
    if (st == TKPHI_OK) st = hip_ok(hipEventCreateWithFlags(&e0, hipEventDisableTiming), "hipEventCreateWithFlags");
    if (st == TKPHI_OK) st = hip_ok(hipEventCreateWithFlags(&e1, hipEventDisableTiming), "hipEventCreateWithFlags");
    if (st != TKPHI_OK) {
      if (e0) (void)hipEventDestroy(e0);
      if (e1) (void)hipEventDestroy(e1);
      if (str) (void)hipStreamDestroy(str);
      return st;
    }
    ss.stream = str; ss.fork = e0; ss.join = e1;
  }
  *out = &ss;
  return TKPHI_OK;
}

static tkphi_status enqueue_decode(const Geom& g, const tkphi_problem* problems, char* ws, int acct, hipStream_t s) {
  if (g.filtered && !g.diag) {         // (the diagnostics are by-products of the spill pipeline's emit pass)
    Geom gf = g;
    gf.n_tiles = g.sg_split;           // one partial per workgroup of the fused select + gather kernel
    launch_prep(gf, problems, ws, s);
    launch_score_filtered(gf, problems, ws, s);
    launch_select_gather(gf, problems, ws, acct, s);   // (its last workgroup per head merges)
    return TKPHI_OK;
  }
  if (g.phi_kind != TKPHI_PHI_MLP) {
    launch_score_mid(g, problems, ws, s);
    launch_select(g, problems, ws, s);
    launch_gather(g, problems, ws, s);
    launch_merge(g, problems, ws, acct, false, s);
    return TKPHI_OK;
  }
  std::lock_guard<std::mutex> lock(g_side_mutex);
  SideStream* ss = nullptr;
  tkphi_status st = side_stream(&ss);
  if (st != TKPHI_OK) return st;
  st = hip_ok(hipEventRecord(ss->fork, s), "hipEventRecord");
  if (st == TKPHI_OK) st = hip_ok(hipStreamWaitEvent(ss->stream, ss->fork, 0), "hipStreamWaitEvent");
  if (st != TKPHI_OK) return st;
  launch_mlp_phi_q(g, problems, ws, ss->stream);
  st = hip_ok(hipEventRecord(ss->join, ss->stream), "hipEventRecord");
  launch_score_mid(g, problems, ws, s);
  launch_select(g, problems, ws, s);
  if (g.sel_feat) launch_mlp_sel_features(g, problems, ws, s);    // no feature cache: phi_k of the retrieved keys
  // (the join is enqueued even after an error above: the side stream must not be left forked)
  const tkphi_status st2 = hip_ok(hipStreamWaitEvent(s, ss->join, 0), "hipStreamWaitEvent");
  if (st != TKPHI_OK) return st;
  if (st2 != TKPHI_OK) return st2;
  launch_gather(g, problems, ws, s);
  launch_merge(g, problems, ws, acct, false, s);
  return TKPHI_OK;
}

tkphi_status tkphi_decode(const tkphi_config* cfg, const tkphi_problem* problems, int32_t n_problems,
                          int32_t max_L, int32_t max_K, int32_t mode, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  const int acct = mode & ~TKPHI_FLAG_DIAG;
  if (acct != TKPHI_MODE_SUB && acct != TKPHI_MODE_NOSUB && acct != TKPHI_MODE_TOPK_ONLY) {
    set_error("mode=%d is not a tkphi_mode (optionally | TKPHI_FLAG_DIAG)", mode);
    return TKPHI_EINVAL;
  }
  Geom g;
  tkphi_status st = make_geom(cfg, n_problems, max_L, max_K, &g);
  g.diag = (mode & TKPHI_FLAG_DIAG) ? 1 : 0;
  if (st != TKPHI_OK) return st;
  st = check_call(problems, n_problems, workspace, workspace_bytes, g, g.decode_bytes);
  if (st != TKPHI_OK) return st;
  if (n_problems == 0) return TKPHI_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  (void)hipGetLastError();
  st = enqueue_decode(g, problems, ws, acct, s);
  if (st != TKPHI_OK) return st;
  return hip_ok(hipGetLastError(), "tkphi_decode launch");
}

// ---- decode for callers that cannot allocate ------------------------------------------------
// The scratch memory of a decode call (everything tkphi_decode keeps in the caller's workspace)
// in a file-scope device array.  Each GPU the library runs on holds its own copy of the array,
// at its own address, until the process ends; the address is resolved once per device, with that
// device current, and kept.  Host code never uses the array's name for anything else: kernels,
// like every other consumer, get the resolved pointer.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[TKPHI_STATIC_SCRATCH_BYTES];
static std::mutex g_scratch_mutex;
static char* g_scratch_ptr[64];

static tkphi_status static_scratch(char** out) {
  int dev = 0;
  tkphi_status st = hip_ok(hipGetDevice(&dev), "hipGetDevice");
  if (st != TKPHI_OK) return st;
  if (dev < 0 || dev >= 64) { set_error("device ordinal %d out of range", dev); return TKPHI_EINVAL; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    st = hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
    if (st != TKPHI_OK) return st;
    if (!ptr || ((uintptr_t)ptr) % 256 != 0) { set_error("static scratch resolved to %p", ptr); return TKPHI_EHIP; }
    g_scratch_ptr[dev] = (char*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return TKPHI_OK;
}

tkphi_status tkphi_decode_static(const tkphi_config* cfg, const tkphi_problem* problems, int32_t n_problems,
                                 int32_t max_L, int32_t max_K, int32_t mode, void* hip_stream) {
  const int acct = mode & ~TKPHI_FLAG_DIAG;
  if (acct != TKPHI_MODE_SUB && acct != TKPHI_MODE_NOSUB && acct != TKPHI_MODE_TOPK_ONLY) {
    set_error("mode=%d is not a tkphi_mode (optionally | TKPHI_FLAG_DIAG)", mode);
    return TKPHI_EINVAL;
  }
  Geom g;
  tkphi_status st = make_geom(cfg, n_problems, max_L, max_K, &g);
  if (st != TKPHI_OK) return st;
  g.diag = (mode & TKPHI_FLAG_DIAG) ? 1 : 0;
  if (g.phi_kind == TKPHI_PHI_MLP) {      // that path creates a stream and events on first use
    set_error("tkphi_decode_static does not run the MLP feature maps");
    return TKPHI_EUNSUPPORTED;
  }
  if (g.decode_bytes > (size_t)TKPHI_STATIC_SCRATCH_BYTES) {
    set_error("decode scratch of %zu bytes exceeds the static array of %zu bytes (n_problems=%d max_L=%d max_K=%d)",
              g.decode_bytes, (size_t)TKPHI_STATIC_SCRATCH_BYTES, n_problems, max_L, max_K);
    return TKPHI_EWORKSPACE;
  }
  char* ws = nullptr;
  st = static_scratch(&ws);
  if (st != TKPHI_OK) return st;
  st = check_call(problems, n_problems, ws, g.decode_bytes, g, g.decode_bytes);
  if (st != TKPHI_OK) return st;
  if (n_problems == 0) return TKPHI_OK;
  (void)hipGetLastError();
  st = enqueue_decode(g, problems, ws, acct, (hipStream_t)hip_stream);
  if (st != TKPHI_OK) return st;
  return hip_ok(hipGetLastError(), "tkphi_decode_static launch");
}

tkphi_status tkphi_decode_stage_times(const tkphi_config* cfg, const tkphi_problem* problems,
                                      int32_t n_problems, int32_t max_L, int32_t max_K, int32_t mode,
                                      void* workspace, size_t workspace_bytes, void* hip_stream,
                                      float* stage_ms_out) {
  if (!stage_ms_out) { set_error("stage_ms_out is null"); return TKPHI_EINVAL; }
  const int acct = mode & ~TKPHI_FLAG_DIAG;
  if (acct != TKPHI_MODE_SUB && acct != TKPHI_MODE_NOSUB && acct != TKPHI_MODE_TOPK_ONLY) {
    set_error("mode=%d is not a tkphi_mode (optionally | TKPHI_FLAG_DIAG)", mode);
    return TKPHI_EINVAL;
  }
  Geom g;
  tkphi_status st = make_geom(cfg, n_problems, max_L, max_K, &g);
  g.diag = (mode & TKPHI_FLAG_DIAG) ? 1 : 0;
  if (st != TKPHI_OK) return st;
  st = check_call(problems, n_problems, workspace, workspace_bytes, g, g.decode_bytes);
  if (st != TKPHI_OK) return st;
  for (int i = 0; i < TKPHI_N_STAGES; ++i) stage_ms_out[i] = 0.f;
  if (n_problems == 0) return TKPHI_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  // one (start, stop) event pair per kernel, recorded at the kernel's own begin and end
  static_assert(TKPHI_N_STAGES == ST_COUNT, "stage list out of sync with include/tkphi.h");
  hipEvent_t ev[2 * ST_COUNT];
  int made = 0;
  for (; made < 2 * ST_COUNT; ++made)
    if ((st = hip_ok(hipEventCreate(&ev[made]), "hipEventCreate")) != TKPHI_OK) break;
  if (st == TKPHI_OK) {
    KernelTimer t;
    for (int i = 0; i < ST_COUNT; ++i) { t.start[i] = ev[2 * i]; t.stop[i] = ev[2 * i + 1]; t.used[i] = false; }
    (void)hipGetLastError();
    g_kernel_timer = &t;
    st = enqueue_decode(g, problems, ws, acct, s);
    g_kernel_timer = nullptr;
    if (st == TKPHI_OK) st = hip_ok(hipGetLastError(), "tkphi_decode_stage_times launch");
    if (st == TKPHI_OK) st = hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize");
    for (int i = 0; st == TKPHI_OK && i < ST_COUNT; ++i)
      if (t.used[i]) st = hip_ok(hipEventElapsedTime(&stage_ms_out[i], t.start[i], t.stop[i]), "hipEventElapsedTime");
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  return st;
}

tkphi_status tkphi_check_problems(const tkphi_config* cfg, const tkphi_problem* ph, int32_t n_problems,
                                  int32_t max_L, int32_t max_K, int32_t for_decode) {
  Geom g;
  tkphi_status st = make_geom(cfg, n_problems, max_L, max_K, &g);
  if (st != TKPHI_OK) return st;
  if (n_problems > 0 && !ph) { set_error("problems_host is null"); return TKPHI_EINVAL; }
  const size_t es = cfg->kv_dtype == TKPHI_BF16 ? 2 : 4;
  for (int p = 0; p < n_problems; ++p) {
    const tkphi_problem& q = ph[p];
    const bool mlp = cfg->phi_kind == TKPHI_PHI_MLP;     // then Wq, bq, Wk, bk are not read
    const void* req[] = {q.K, q.V, q.S, q.u, q.Wk, q.bk};
    const char* names[] = {"K", "V", "S", "u", "Wk", "bk"};
    for (int i = 0; i < (mlp ? 4 : 6); ++i) {
      if (!req[i]) { set_error("problem %d: %s is null", p, names[i]); return TKPHI_EINVAL; }
      if (((uintptr_t)req[i]) % 16 != 0) { set_error("problem %d: %s not 16-byte aligned", p, names[i]); return TKPHI_EALIGN; }
    }
    if (cfg->phi_kind == TKPHI_PHI_MLP) {
      if (!q.mlp_k || (for_decode && !q.mlp_q)) { set_error("problem %d: mlp_k / mlp_q is null", p); return TKPHI_EINVAL; }
      if (((uintptr_t)q.mlp_k) % 8 != 0 || ((uintptr_t)q.mlp_q) % 8 != 0) { set_error("problem %d: mlp table misaligned", p); return TKPHI_EALIGN; }
    }
    if (cfg->cache_features) {
      if (!q.phi_cache) { set_error("problem %d: phi_cache is null (cfg.cache_features is set)", p); return TKPHI_EINVAL; }
      if (((uintptr_t)q.phi_cache) % 16 != 0) { set_error("problem %d: phi_cache not 16-byte aligned", p); return TKPHI_EALIGN; }
    }
    if (q.diag && ((uintptr_t)q.diag) % 4 != 0) { set_error("problem %d: diag misaligned", p); return TKPHI_EALIGN; }
    if (for_decode) {
      const void* rq[] = {q.q, q.out, q.Wq, q.bq};
      const char* nq[] = {"q", "out", "Wq", "bq"};
      for (int i = 0; i < (mlp ? 2 : 4); ++i) {
        if (!rq[i]) { set_error("problem %d: %s is null", p, nq[i]); return TKPHI_EINVAL; }
        if (((uintptr_t)rq[i]) % 16 != 0) { set_error("problem %d: %s not 16-byte aligned", p, nq[i]); return TKPHI_EALIGN; }
      }
      if (q.n_gen < 0 || q.n_gen > cfg->max_gen) { set_error("problem %d: n_gen=%d outside [0, cfg.max_gen=%d]", p, q.n_gen, cfg->max_gen); return TKPHI_ESHAPE; }
      if (q.topk < 0 || q.topk > max_K) { set_error("problem %d: topk=%d outside [0, max_K=%d]", p, q.topk, max_K); return TKPHI_ESHAPE; }
      if (q.topk_idx && ((uintptr_t)q.topk_idx) % 4 != 0) { set_error("problem %d: topk_idx misaligned", p); return TKPHI_EALIGN; }
      if (q.aux && ((uintptr_t)q.aux) % 4 != 0) { set_error("problem %d: aux misaligned", p); return TKPHI_EALIGN; }
      if (q.scores && ((uintptr_t)q.scores) % 4 != 0) { set_error("problem %d: scores misaligned", p); return TKPHI_EALIGN; }
    }
    if (q.L < 1 || q.L > max_L) { set_error("problem %d: L=%d outside [1, max_L=%d]", p, q.L, max_L); return TKPHI_ESHAPE; }
    if (q.stride_tok < cfg->d_head || (q.stride_tok * es) % 16 != 0) {
      set_error("problem %d: stride_tok=%lld invalid (>= d_head, 16-byte multiple)", p, (long long)q.stride_tok);
      return TKPHI_EALIGN;
    }
    if (q.stride_head < 0 || (q.stride_head * es) % 16 != 0 ||
        (cfg->n_kv_heads > 1 && q.stride_head < cfg->d_head)) {
      set_error("problem %d: stride_head=%lld invalid", p, (long long)q.stride_head);
      return TKPHI_EALIGN;
    }
  }
  return TKPHI_OK;
}

tkphi_status tkphi_read_device_status(const void* workspace, void* hip_stream, uint32_t* status_out) {
  if (!workspace || !status_out) { set_error("null argument"); return TKPHI_EINVAL; }
  hipStream_t s = (hipStream_t)hip_stream;
  tkphi_status st = hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize");
  if (st != TKPHI_OK) return st;
  return hip_ok(hipMemcpy(status_out, workspace, sizeof(uint32_t), hipMemcpyDeviceToHost), "hipMemcpy status");
}

int32_t tkphi_budget_paper(int64_t L, int32_t r_bp, int32_t n_sink, int32_t n_tail) {
  if (L < 0 || r_bp < 0 || n_sink < 0 || n_tail < 0) return 0;
  const int64_t anchors = std::min<int64_t>(L, (int64_t)n_sink + n_tail);
  const int64_t ceil_rL = (L * r_bp + 9999) / 10000;
  return (int32_t)std::max<int64_t>(0, ceil_rL - anchors);
}

int32_t tkphi_budget_mid(int64_t L, int32_t r_bp, int32_t n_sink, int32_t n_tail) {
  if (L < 0 || r_bp < 0 || n_sink < 0 || n_tail < 0) return 0;
  const int64_t mid = std::max<int64_t>(0, L - n_sink - n_tail);
  return (int32_t)(mid * r_bp / 10000);
}

const char* tkphi_status_string(int32_t status) {
  switch (status) {
    case TKPHI_OK: return "ok";
    case TKPHI_EINVAL: return "invalid argument";
    case TKPHI_ESHAPE: return "unsupported shape";
    case TKPHI_EALIGN: return "misaligned pointer or stride";
    case TKPHI_EWORKSPACE: return "workspace null, misaligned or too small";
    case TKPHI_EHIP: return "HIP runtime error";
    case TKPHI_EUNSUPPORTED: return "unsupported request";
    default: return "unknown status";
  }
}

const char* tkphi_last_error(void) { return g_last_error; }

}  // extern "C"
