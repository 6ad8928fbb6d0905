/*
 * tkphi.h -- C ABI of libtkphi: Top-K+phi residual-mass decode attention on one
 * AMD MI355X (gfx950).
 *
 * The library implements, per attention layer, the per-decode-step attention over a
 * long prefill KV cache described in "Residual-Mass Accounting for Partial-KV
 * Decoding":
 *
 *   prefill   tkphi_build_summaries   S_M = sum_{i in M} phi_k(k_i) v_i^T,
 *                                     u_M = sum_{i in M} phi_k(k_i)
 *                                     (Sec. "Positive feature maps and summary
 *                                     states", eq. (natural_cache))
 *   decode    tkphi_decode            y = (nu_E + nu_R^) / (Z_E + Z_R^)
 *                                     (Sec. "Single-normalization merge",
 *                                     eq. (hybrid_merge)), with the exact support
 *                                     E = A u TopK(M) (eq. (partition),
 *                                     eq. (exact_terms)) chosen by an exhaustive
 *                                     Top-K over the mid-region M, and the residual
 *                                     read from (S_M, u_M) minus the retrieved
 *                                     tokens' feature contributions
 *                                     (eq. (subtraction)); already generated tokens
 *                                     are one more exact branch under the same
 *                                     normalisation (eq. (implemented_decode)).
 *
 * Everything runs in hand-written HIP kernels enqueued on the caller's stream (with the
 * MLP feature maps, decode also uses one stream of the library's own per device, forked
 * from and joined to the caller's: see tkphi_phi_kind).  The library owns no device
 * memory: every buffer, including scratch ("workspace"), is allocated by the caller.
 * Calls only enqueue work; they never synchronise the stream and never copy device data
 * to the host (tkphi_read_device_status and tkphi_decode_stage_times excepted).
 *
 * Pointer kinds.  Unless a parameter is marked HOST, pointers are DEVICE pointers.
 * The tkphi_config struct itself and the outermost arguments are read on the host
 * at call time; the tkphi_problem table is read by the kernels (DEVICE memory).
 *
 * Errors.  Every entry point returns a tkphi_status (or a size/count documented
 * below); nothing throws or aborts across the boundary.  Host-visible arguments are
 * validated before any launch, and a call that fails validation enqueues nothing.
 * tkphi_last_error() returns a thread-local detail string for the last failure.
 * Fields of the device-resident problem table cannot be seen by the host; kernels
 * clip topk to min(topk, |M|, max_K) and skip a problem whose L exceeds max_L (or is < 1),
 * recording TKPHI_DEV_BAD_LENGTH in the workspace status word (both tkphi_build_summaries and
 * tkphi_decode rewrite the word on every call; the outputs of a skipped problem, S and u
 * included, are left untouched).  tkphi_check_problems validates a HOST copy of the table.
 */
#ifndef TKPHI_H_
#define TKPHI_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tkphi_status {
  TKPHI_OK = 0,
  TKPHI_EINVAL = -1,       /* null pointer, negative count, bad enum value          */
  TKPHI_ESHAPE = -2,       /* head counts / head_dim / d_phi / lengths unsupported  */
  TKPHI_EALIGN = -3,       /* pointer or stride not 16-byte aligned                 */
  TKPHI_EWORKSPACE = -4,   /* workspace null, misaligned or too small               */
  TKPHI_EHIP = -5,         /* a HIP runtime call failed (see tkphi_last_error)      */
  TKPHI_EUNSUPPORTED = -6  /* valid request the library has no kernel for           */
} tkphi_status;

typedef enum tkphi_dtype { TKPHI_F32 = 0, TKPHI_BF16 = 1 } tkphi_dtype;

/* Accounting variants (Sec. "Models, tasks, and protocol"):
 *   SUB        Top-K+phi, retrieved tokens subtracted from the summaries (the method)
 *   NOSUB      ablation: summaries merged un-subtracted (double counts the retrieved set)
 *   TOPK_ONLY  selection-only Top-K: y = nu_E / Z_E, no residual branch               */
typedef enum tkphi_mode { TKPHI_MODE_SUB = 0, TKPHI_MODE_NOSUB = 1, TKPHI_MODE_TOPK_ONLY = 2 } tkphi_mode;
/* May be OR-ed into the mode argument of tkphi_decode: also compute the entropy / mass-recovery
 * diagnostics below for every problem whose `diag` pointer is non-NULL (one extra exp per
 * score in the select pass; off by default). */
#define TKPHI_FLAG_DIAG 0x100

/* bits of the device status word (tkphi_read_device_status) */
#define TKPHI_DEV_BAD_LENGTH 1u   /* a problem had L < 1 or L > max_L and was skipped, or an
                                     n_gen outside [0, cfg.max_gen] that was clamped           */
#define TKPHI_DEV_CLAMPED    2u   /* a residual denominator came out <= 0 after subtraction
                                     and the residual branch was dropped for that head
                                     (App. "Why positivity matters": numerical clamp)         */

/* Feature-map families.
 *   EXP_AFFINE  phi(x) = exp(phi_in_scale * W x - phi_norm_coef * |x|^2 + b), per-head W, b
 *               (tkphi_problem::Wq, bq, Wk, bk)
 *   MLP         the head-wise one-block ReZero MLP of App. "Head-wise phi architecture":
 *                 g0 = Ws x + bs;  Delta = W2 GeLU(W1 g0 + b1) + b2;  g1 = g0 + alpha Delta;
 *                 phi(x) = exp(Wo g1 + bo)
 *               with internal width cfg.d_emb (the paper: 512), one tkphi_mlp per query head
 *               (tkphi_problem::mlp_q) and per KV head (mlp_k).  Requires bf16 storage.  The key
 *               features of the mid-region are evaluated at build time by a chain of
 *               matrix-core GEMMs whose fp32 activations enter as bf16 hi + lo pairs (GeLU
 *               uses erfc to 1.5e-7 absolute), groups of up to 16 problems per launch.  With
 *               cfg.cache_features = 1 they are stored in phi_cache and decode gathers them;
 *               with cfg.cache_features = 0 (d_emb in {128, 256, 512} and d_phi <= 256 only)
 *               the build keeps a group's features in the workspace until they are contracted
 *               into S, u, and every decode step sends the retrieved key rows through the same
 *               chain (Sec. "Retrieved-token subtraction": retrieved-key feature
 *               recomputation).  tkphi_decode evaluates phi_q with
 *               three small launches on a second stream that the library creates per device
 *               on first use (default priority, kept until the process ends): forked from the
 *               caller's stream at the start of the call and joined to it before the gather, so
 *               the caller still sees one in-order unit of work; such calls serialise on a
 *               mutex while they enqueue.  The device of hip_stream must be the current device;
 *               a caller that captures decode calls into a HIP graph makes one call outside the
 *               capture first (the stream and its two events are created then). */
typedef enum tkphi_phi_kind { TKPHI_PHI_EXP_AFFINE = 0, TKPHI_PHI_MLP = 1 } tkphi_phi_kind;

/* One head's MLP feature map.  DEVICE struct (arrays of it live in device memory); weights are
 * row-major [out][in] in the storage type (bf16), biases fp32; all pointers 16-byte aligned. */
typedef struct tkphi_mlp {
  const void* Ws;        /* [d_emb][d_head]  */
  const float* bs;       /* [d_emb]          */
  const void* W1;        /* [d_emb][d_emb]   */
  const float* b1;       /* [d_emb]          */
  const void* W2;        /* [d_emb][d_emb]   */
  const float* b2;       /* [d_emb]          */
  const void* Wo;        /* [d_phi][d_emb]   */
  const float* bo;       /* [d_phi]          */
  float alpha;           /* residual gate    */
  int32_t reserved;      /* 0                */
} tkphi_mlp;

/* Launch-geometry overrides: for tests that must reach a particular kernel variant at small
 * sizes, and for tuning sweeps.  Every field 0 = the library's own choice (what production callers
 * pass).  Part of tkphi_config, so tkphi_workspace_bytes, tkphi_build_summaries and tkphi_decode
 * always see the same values; out-of-range values are rejected with TKPHI_EINVAL. */
typedef struct tkphi_tuning {
  int32_t force_generic;  /* 1: run the generic fp32-arithmetic kernels where the matrix-core ones apply  */
  int32_t scan_chunk;     /* score_mid: mid tokens per workgroup (rounded up to the kernel's unit of
                             256 / 512 rows, at most 32768); 0 = about 1024 workgroups per call           */
  int32_t interleave;     /* score_mid chunk-to-row mapping: 1 = chunk c takes the units c, c + n_chunks,
                             ..., 2 = one contiguous range per chunk; 0 = by the number of chunks         */
  int32_t build_chunk;    /* summary build: mid tokens per workgroup (multiple of 64); 0 = auto          */
  int32_t mlp_block;      /* MLP build, layer-wise launches: tokens per KV head held at once; 0 = auto   */
  int32_t mlp_mode;       /* MLP build: 0 = one persistent launch where the widths allow it,
                             1 = layer-wise launches per token block (residual + output fused),
                             2 = all four layers as separate launches                                    */
  int32_t select_mode;    /* decode pipeline of the bf16 matrix-core shapes: 0 = by the bounds (filtered where it
                             measured faster: max_K at most 1/64 of the largest mid-region),
                             1 = spill (score_mid writes
                             every score and chunk histograms; plan / emit / resolve select from them),
                             2 = filtered (a sampled lower bound of the K-th score prunes what the score pass
                             writes; one select kernel per step).  Ignored where only the spill pipeline applies
                             (fp32 storage, d_phi != d_head, MLP maps, TKPHI_FLAG_DIAG)                    */
  int32_t select_test;    /* filtered pipeline, tests only: 1 = the sampled bound is replaced by one no score
                             passes (every head takes the rescan), 2 = by one every score passes           */
  int32_t reserved[4];    /* 0                                                                            */
} tkphi_tuning;

/* Fixed per model.  HOST struct.
 * The feature maps have the form phi(x) = exp(phi_in_scale * W x - phi_norm_coef * |x|^2 + b)
 * with per-head W, b (exponentiated affine output, App. "Head-wise phi architecture").
 * Query head g uses KV head g / (n_q_heads / n_kv_heads).
 * Supported: d_head in {64, 128}; d_phi a multiple of 16 in [16, 256];
 * n_q_heads a multiple of n_kv_heads with ratio <= 8; bf16 storage additionally
 * requires d_phi == d_head for the MFMA path (other d_phi run on the generic path). */
typedef struct tkphi_config {
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t d_head;        /* d_h == d_v (Sec. "Setup and residual-mass bias")                */
  int32_t d_phi;
  int32_t n_sink;        /* anchors: first n_sink and last n_tail tokens (eq. (partition)) */
  int32_t n_tail;
  int32_t kv_dtype;      /* tkphi_dtype of q, K, V, Wq, Wk                                  */
  float score_scale;     /* 1/sqrt(d_head) (eq. (full_attention))                           */
  float phi_in_scale;    /* a                                                               */
  float phi_norm_coef;   /* c                                                               */
  int32_t cache_features; /* 0: decode recomputes phi_k of the retrieved keys (the paper's prototype);
                             1: tkphi_build_summaries also stores phi_k(k_i) of every mid token in
                             tkphi_problem::phi_cache and tkphi_decode gathers it instead (the cached
                             variant named in Sec. "Retrieved-token subtraction": d_phi * 4 bytes per
                             token and KV head of extra cache)                              */
  int32_t phi_kind;      /* tkphi_phi_kind; 0 = EXP_AFFINE                                  */
  int32_t d_emb;         /* MLP only: internal width, a power of two in [64, 1024]          */
  int32_t max_gen;       /* upper bound of tkphi_problem::n_gen (generated tokens kept exact,
                            eq. (implemented_decode)); 0 if the feature is not used          */
  tkphi_tuning tuning;   /* all zero = defaults                                             */
} tkphi_config;

/* Optional per-query-head diagnostics / unnormalised outputs written by tkphi_decode,
 * TKPHI_AUX_STRIDE(d_head) floats per query head:
 *   [0] m        shift = max score over the exact support E
 *   [1] Z_E      sum_{i in E} exp(s_i - m)
 *   [2] Z_R^     phi_q . u_R (unshifted; 0 in TOPK_ONLY mode or if clamped)
 *   [3] flags    1.0 if the clamp fired for this head, else 0.0
 *   [4 .. 4+d)        nu_E  (shifted by m)
 *   [4+d .. 4+2d)     nu_R^ (unshifted)
 * so that y = (nu_E + exp(-m) nu_R^) / (Z_E + exp(-m) Z_R^); a caller can add further
 * exact branches (e.g. generated tokens, eq. (implemented_decode)) before dividing. */
#define TKPHI_AUX_STRIDE(d_head) (4 + 2 * (d_head))

/* Optional per-query-head diagnostics of the entropy / mass-recovery analysis
 * (Sec. "Analysis: entropy and completion gains"; App. "Entropy, mass recovery, and
 * residual-denominator diagnostics"), by-products of the score pass, TKPHI_DIAG_STRIDE
 * floats per query head (requires TKPHI_FLAG_DIAG):
 *   [0] H_mid        normalised entropy of the mid-normalised attention, in [0, 1]
 *   [1] log Z_M      log of the mid-region softmax mass sum_{j in M} exp(s_j)
 *   [2] C_mid(K)     Z_K / Z_M: mid-region mass recovered by the retrieved tokens
 *   [3] rho_res      Z_R^ / (Z_E + Z_R^): residual share of the merged denominator
 *   [4] rho_res*     Z_R / (Z_A + Z_M): the true residual share
 *   [5] log Z_R^ - log Z_R   residual log-partition error (NaN if either is <= 0)
 *   [6] log Z_A      log of the anchor mass;  [7] reserved (0)
 * All zero if the mid-region is empty. */
#define TKPHI_DIAG_STRIDE 8

/* One problem = one (sequence, layer).  The table lives in DEVICE memory; all
 * pointers inside are DEVICE pointers to caller-owned buffers that must stay valid
 * until the enqueued work has finished.  16-byte alignment is required for K, V, q,
 * Wq, Wk, S, u, out, and stride_tok * sizeof(elem) and stride_head * sizeof(elem)
 * must be multiples of 16.  */
typedef struct tkphi_problem {
  const void* K;         /* keys   [n_kv_heads][L][d_head], strides below (elements)   */
  const void* V;         /* values [n_kv_heads][L][d_head], same strides               */
  int64_t stride_head;   /* elements between consecutive KV heads                      */
  int64_t stride_tok;    /* elements between consecutive tokens (>= d_head)            */
  const void* Wq;        /* [n_q_heads ][d_phi][d_head] kv_dtype                       */
  const float* bq;       /* [n_q_heads ][d_phi]                                        */
  const void* Wk;        /* [n_kv_heads][d_phi][d_head] kv_dtype                       */
  const float* bk;       /* [n_kv_heads][d_phi]                                        */
  float* S;              /* [n_kv_heads][d_phi][d_head] fp32: written by build, read by decode */
  float* u;              /* [n_kv_heads][d_phi]         fp32: written by build, read by decode */
  const void* q;         /* [n_q_heads][d_head] kv_dtype (decode only)                 */
  float* out;            /* [n_q_heads][d_head] fp32 y (decode only)                   */
  int32_t* topk_idx;     /* optional [n_q_heads][max_K]: retrieved token indices (absolute
                            positions in [n_sink, L - n_tail)), ascending, first min(K,|M|)
                            entries of each row valid; may be NULL                      */
  float* aux;            /* optional [n_q_heads][TKPHI_AUX_STRIDE(d_head)]; may be NULL */
  float* scores;         /* optional [n_q_heads][L - n_sink - n_tail] fp32 mid-region
                            scores s_i, i in M (diagnostic copy); may be NULL           */
  float* diag;           /* optional [n_q_heads][TKPHI_DIAG_STRIDE]; may be NULL        */
  float* phi_cache;      /* [n_kv_heads][L - n_sink - n_tail][d_phi] fp32 key features of the
                            mid-region, exactly the values the build contracted; written by
                            build and read by decode when cfg.cache_features != 0 (then
                            required), ignored otherwise                                */
  const tkphi_mlp* mlp_q; /* [n_q_heads]  feature maps of the query heads (TKPHI_PHI_MLP only) */
  const tkphi_mlp* mlp_k; /* [n_kv_heads] feature maps of the KV heads    (TKPHI_PHI_MLP only);
                             with TKPHI_PHI_MLP the fields Wq, bq, Wk, bk are ignored          */
  int32_t L;             /* prefill length, 1 <= L <= max_L                            */
  int32_t topk;          /* the paper's K: retrieved mid-region tokens per query head (the
                            budget); clipped to min(topk, |M|, max_K); 0 is legal      */
  int32_t n_gen;         /* generated tokens at the current step, 0 <= n_gen <= cfg.max_gen: rows
                            [L, L + n_gen) of K and V.  They are outside the prefill partition
                            (never retrieved, not in S, u) and enter the output as one more exact
                            branch under the same normalisation (eq. (implemented_decode)); in the
                            aux / diag outputs they count with the exact support (Z_E, nu_E, Z_A).
                            A value outside the range is clamped to it by the kernels and sets
                            TKPHI_DEV_BAD_LENGTH in the device status word.              */
  int32_t reserved;      /* 0                                                          */
} tkphi_problem;

/* Bytes of DEVICE workspace tkphi_build_summaries / tkphi_decode need for the given
 * launch bounds (the larger of the two).  Returns 0 if the config is invalid.
 * The workspace must be 256-byte aligned.  Its contents need not be preserved between
 * calls and need not be initialised.  Two calls that overlap in time (different
 * streams) must not share a workspace. */
size_t tkphi_workspace_bytes(const tkphi_config* cfg /*HOST*/, int32_t n_problems,
                             int32_t max_L, int32_t max_K);

/* Prefill: for every problem and KV head, S = sum_{i in M} phi_k(k_i) v_i^T and
 * u = sum_{i in M} phi_k(k_i) over the mid-region M = [n_sink, L - n_tail)
 * (eq. (natural_cache)); feature-major S[h][j][c] (j feature, c value channel).
 * Reads K, V, L and Wk, bk (TKPHI_PHI_MLP: mlp_k instead); writes S, u (fully overwritten;
 * zeros if M is empty) and, with cfg.cache_features, phi_cache (the features of the mid
 * tokens, exactly the values that were contracted).  Rows past L (generated tokens) are
 * not read.  Deterministic: the same inputs give bit-identical S, u. */
tkphi_status tkphi_build_summaries(const tkphi_config* cfg /*HOST*/,
                                   const tkphi_problem* problems /*DEVICE table*/,
                                   int32_t n_problems, int32_t max_L,
                                   void* workspace, size_t workspace_bytes,
                                   void* hip_stream);

/* One decode step for every problem and query head: scores the mid-region, selects
 * the K highest-scoring mid tokens (ties to the lower index), accumulates the exact
 * max-shifted terms over anchors + retrieved tokens, evaluates the residual from
 * (S, u) with the retrieved tokens' features subtracted, and merges under one
 * normalisation (eq. (exact_terms), eq. (subtraction), eq. (hybrid_merge)); the n_gen
 * generated tokens after the prefill rows are added as exact terms (eq. (implemented_decode)).
 * Reads q, K, V, Wq, bq, Wk, bk, S, u, L, topk, n_gen (with cfg.cache_features phi_cache
 * instead of Wk, bk; TKPHI_PHI_MLP: mlp_q instead of Wq, bq); writes out (and topk_idx,
 * aux, scores, diag when non-NULL).  If L <= n_sink + n_tail the mid-region is empty and
 * the result is dense attention over all L + n_gen tokens.  Deterministic for fixed inputs. */
tkphi_status tkphi_decode(const tkphi_config* cfg /*HOST*/,
                          const tkphi_problem* problems /*DEVICE table*/,
                          int32_t n_problems, int32_t max_L, int32_t max_K,
                          int32_t mode /* tkphi_mode, optionally | TKPHI_FLAG_DIAG */,
                          void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/* tkphi_decode for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus
 * the workspace), same validation, same kernels and bit-identical results; the scratch memory is a
 * static device array of TKPHI_STATIC_SCRATCH_BYTES inside the library, of which every GPU the
 * library runs on holds one copy until the process ends.  A request whose decode scratch does not
 * fit (tkphi_workspace_bytes is an upper bound of it; one 128K-token layer of 24 query heads needs
 * about 17 MiB) fails with TKPHI_EWORKSPACE and enqueues nothing; TKPHI_PHI_MLP is refused with
 * TKPHI_EUNSUPPORTED (that path creates a stream on first use).  The call allocates nothing and frees
 * nothing.  The first call on a device resolves the array's address (with that device current: the
 * device of hip_stream must be the current device); a caller that captures calls into a HIP graph makes
 * one call outside the capture first.  All calls on one GPU share the array, which keeps the last call's contents
 * (nothing in it needs to start at zero): two calls that overlap in time on one GPU, on different
 * streams or threads, race; calls on one stream are ordered and safe.  tkphi_read_device_status
 * cannot be used with it (the status word lives in the array). */
#define TKPHI_STATIC_SCRATCH_BYTES (32u << 20)
tkphi_status tkphi_decode_static(const tkphi_config* cfg /*HOST*/,
                                 const tkphi_problem* problems /*DEVICE table*/,
                                 int32_t n_problems, int32_t max_L, int32_t max_K,
                                 int32_t mode /* tkphi_mode, optionally | TKPHI_FLAG_DIAG */,
                                 void* hip_stream);

/* Profiling helper: the same work as tkphi_decode, with a pair of HIP events attached to
 * every kernel launch (recorded at the kernel's own begin and end on the stream), then a
 * stream synchronisation; stage_ms_out (HOST, TKPHI_N_STAGES floats) receives the
 * duration in milliseconds of each stage:
 *   score_mid (either pipeline's score pass), select_plan (+ the exp-affine phi_q), select_emit,
 *   select_resolve, gather (exact branch + subtraction sums), merge (spill pipeline), phi_q (the
 *   three phi_q launches of the MLP feature maps, begin of the first to end of the third; or, for a
 *   batch on the filtered pipeline, the phi / anchor jobs of prep as a launch of their own), and the
 *   two kernels only the filtered pipeline has: prep (sampled score bound; for a few problems also phi_q,
 *   the summary terms and the anchors; runs first) and select (selection, gather and merge)
 * (0 for a stage that the given configuration and bounds do not launch).  Same validation and results as
 * tkphi_decode; creates and destroys HIP events (no device memory). */
#define TKPHI_N_STAGES 9
tkphi_status tkphi_decode_stage_times(const tkphi_config* cfg /*HOST*/,
                                      const tkphi_problem* problems /*DEVICE table*/,
                                      int32_t n_problems, int32_t max_L, int32_t max_K,
                                      int32_t mode, void* workspace, size_t workspace_bytes,
                                      void* hip_stream, float* stage_ms_out /*HOST*/);

/* Validates a HOST copy of a problem table against cfg and the launch bounds: non-null
 * required pointers, alignment, strides, 1 <= L <= max_L, 0 <= topk <= max_K,
 * 0 <= n_gen <= cfg.max_gen.
 * for_decode != 0 additionally requires q and out.  Pure host code. */
tkphi_status tkphi_check_problems(const tkphi_config* cfg /*HOST*/,
                                  const tkphi_problem* problems_host /*HOST*/,
                                  int32_t n_problems, int32_t max_L, int32_t max_K,
                                  int32_t for_decode);

/* Copies the device status word (TKPHI_DEV_* bits, accumulated by the kernels of the
 * last call that used this workspace) to *status_out (HOST).  Synchronises the stream. */
tkphi_status tkphi_read_device_status(const void* workspace, void* hip_stream,
                                      uint32_t* status_out /*HOST*/);

/* K = max(0, ceil(r L) - |A|): the paper's rule, anchors counted toward the total
 * exact-support budget r (Sec. "Models, tasks, and protocol"); r in basis points. */
int32_t tkphi_budget_paper(int64_t L, int32_t r_bp, int32_t n_sink, int32_t n_tail);
/* K = floor(r |M|): budget as a fraction of the mid-region size; r in basis points. */
int32_t tkphi_budget_mid(int64_t L, int32_t r_bp, int32_t n_sink, int32_t n_tail);

/* Static, never-null strings. */
const char* tkphi_status_string(int32_t status);
const char* tkphi_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TKPHI_H_ */
