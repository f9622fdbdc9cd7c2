/*
 * codecomp.h - C ABI of the MI355X (gfx950) prefill KV-eviction path of CodeComp:
 *              score -> select -> gather.
 *
 * The operation is the one stated in the paper's section "Attention-based KV Cache
 * Compression": with Q the W observation-window queries and K the N cached keys of one
 * attention head,  A = softmax(Q K^T / sqrt(d)),  u(j) = sum_t A(t, j);  the scores are
 * average-pooled over a sliding window (appendix "Compression settings"), combined with the
 * structural prior of section "Span-Level Structural Protection", the top-ranked tokens are
 * retained up to the budget, independently at each transformer layer, and the retained K/V
 * rows form the compact cache.
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers unless the name ends in _host.  bf16 tensors are
 *     passed as `const void*` (16-bit patterns).  The library allocates nothing and never
 *     synchronises: work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and the call returns.  It reads no environment variable, and all it remembers
 *     between calls is, per device, how many workgroups of each score kernel fit on the device at
 *     once (asked of the runtime on the first call that needs it): calls are re-entrant.
 *   - Query head h_q reads KV head h_q / G with G = n_q_heads / n_kv_heads; the G heads of a
 *     group are averaged.
 *   - Requests are packed along the token axis: request r owns tokens
 *     [cu_seqlens[r], cu_seqlens[r+1]) and output slots [cu_budgets[r], cu_budgets[r+1]).
 *     Its length is N_r and its budget B_r (the last W tokens are always kept and count
 *     towards B_r, so W <= B_r <= N_r).  T = cu_seqlens[n_seqs], TB = cu_budgets[n_seqs].
 *   - Layouts (innermost dimension contiguous; a stride of 0 selects the dense default):
 *       q_obs  bf16 [n_layers][n_seqs][n_q_heads][W][d]
 *       k, v   bf16 [n_layers][n_kv_heads][T][d]        (or FP8 codes, see kv_dtype)
 *       prior  f32  [T]                      (one value per token, shared by layers and heads,
 *                                             finite and >= 0)
 *       scores f32  [n_layers][n_kv_heads][T]          (dense)
 *       idx    i32  [n_layers][n_kv_heads][TB]         (dense; request-local token indices,
 *                                                       ascending within a request)
 *       k_out, v_out bf16 [n_layers][n_kv_heads][TB][d]
 *   - Return value: 0 on success; a negative CODECOMP_E* code when an argument is rejected
 *     (checked on the host before anything is launched: nothing has been enqueued); a positive
 *     value is a hipError_t reported by a launch.  Device data is not validated.
 *   - Inputs are read-only; outputs and workspace must not alias inputs or each other.
 *     Results are deterministic: the same inputs give bit-identical outputs on every call.
 */
#ifndef CODECOMP_H
#define CODECOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CODECOMP_OK = 0,
  CODECOMP_EINVAL_NULL = -1,      /* a required pointer is NULL                                  */
  CODECOMP_EINVAL_SHAPE = -2,     /* n_layers < 1, n_seqs < 1, a negative stride, G*W too large,
                                     score_workgroups < 0, score_lead_tiles > 64                    */
  CODECOMP_EINVAL_WINDOW = -3,    /* W < 1 or W > N_r for some request                            */
  CODECOMP_EINVAL_BUDGET = -4,    /* B_r < W or B_r > N_r for some request                        */
  CODECOMP_EINVAL_POOL = -5,      /* pool_kernel even, < 1 or > 1025                              */
  CODECOMP_EINVAL_HEADS = -6,     /* n_kv_heads < 1 or n_q_heads not a multiple of n_kv_heads     */
  CODECOMP_EINVAL_HEADDIM = -7,   /* head_dim not in {64, 128}                                    */
  CODECOMP_EINVAL_SEQLENS = -8,   /* cu_seqlens / cu_budgets not starting at 0 or not increasing  */
  CODECOMP_EINVAL_WORKSPACE = -9, /* workspace NULL, misaligned (256 B) or too small              */
  CODECOMP_EINVAL_PRIOR = -10,    /* prior_weight negative or not finite; softmax_scale < 0       */
  CODECOMP_EINVAL_MODE = -11      /* select_mode / score_variant / kv_dtype unknown or unsupported for the shape, bad span budget */
};

typedef struct codecomp_params {
  int32_t n_layers;            /* layers are independent problems batched in one call; >= 1      */
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;            /* d: 64 or 128                                                    */
  int32_t window;              /* W: the last W tokens of a request are the observation queries   */
  int32_t pool_kernel;         /* k: odd, 1 <= k <= 1025 (1 = no pooling)                         */
  float prior_weight;          /* lambda >= 0                                                     */
  float softmax_scale;         /* 0 selects 1/sqrt(head_dim)                                      */
  int32_t n_seqs;              /* number of packed requests; 1 = dense                            */
  int32_t select_mode;         /* CODECOMP_SELECT_ADDITIVE (0) or CODECOMP_SELECT_TWO_STAGE (1)  */
  const int32_t* cu_seqlens_host; /* [n_seqs+1] HOST copy: sizes the launches and is validated    */
  const int32_t* cu_seqlens_dev;  /* [n_seqs+1] DEVICE copy of the same values                    */
  const int32_t* cu_budgets_host; /* [n_seqs+1] HOST                                              */
  const int32_t* cu_budgets_dev;  /* [n_seqs+1] DEVICE                                            */
  /* strides in elements; 0 = dense default for the layouts above */
  int64_t q_stride_layer, q_stride_seq, q_stride_head, q_stride_tok;
  int64_t kv_stride_layer, kv_stride_head, kv_stride_tok;      /* shared by k and v              */
  int64_t out_stride_layer, out_stride_head, out_stride_tok;   /* shared by k_out and v_out      */
  /* two-stage selection only (ignored otherwise): span budget = min(Bp, max(span_budget_min,
   * floor(span_budget_ratio * Bp))) with Bp = B_r - W; the paper uses a ratio of 0.5 */
  float span_budget_ratio;     /* rho_span in [0, 1]                                              */
  int32_t span_budget_min;     /* B_min >= 0                                                      */
  int32_t score_variant;       /* bit flags CODECOMP_VARIANT_*; 0 = the default readings          */
  int32_t kv_dtype;            /* CODECOMP_KV_BF16 (0) or CODECOMP_KV_FP8_E4M3 (1): element type of k, v, k_out, v_out */
  /* How the two logit passes of codecomp_score are cut into workgroups; the results do not depend on either
   * value beyond the regrouping of fp32 sums (for tests of exactly that, and for tuning).  Leave both 0. */
  int32_t score_workgroups;    /* 0 = as many as the device holds at once; n > 0 = n (at most 2048, at most one per
                                  64-key tile; with more than 512 softmax rows per KV head the rows are split over
                                  teams of workgroups and n is rounded down to whole teams)          */
  int32_t score_lead_tiles;    /* weight, in 64-key tiles, given to the start of a request when the tiles are shared
                                  out: 0 = built-in value, < 0 = none, 1..64 = that many             */
} codecomp_params;

/* Other readings of what the paper leaves open about the tail of the score step (section
 * "Attention-based KV Cache Compression" and appendix "Compression settings"), for comparison with the
 * defaults (mean over the query-head group, average pooling, softmax and pooling over the whole request):
 *   GROUP_SUM      the masses of the G query heads of a KV head are summed, not averaged;
 *   GROUP_MAX      the largest head mass wins (needs window % 32 == 0 and G * window <= 512);
 *   POOL_MAX       max pooling over the pool_kernel neighbours instead of their average;
 *   SOFTMAX_PREFIX the softmax runs over the N - W context keys only (the K with one row per context token of the
 *                  section); window positions get no attention mass;
 *   POOL_PREFIX    pooling stays inside the N - W context positions; window positions get none.
 * GROUP_SUM and GROUP_MAX exclude each other.  Unknown bits are rejected (CODECOMP_EINVAL_MODE). */
enum {
  CODECOMP_VARIANT_GROUP_SUM = 1,
  CODECOMP_VARIANT_GROUP_MAX = 2,
  CODECOMP_VARIANT_POOL_MAX = 4,
  CODECOMP_VARIANT_SOFTMAX_PREFIX = 8,
  CODECOMP_VARIANT_POOL_PREFIX = 16
};

/* Storage type of the KV cache (k, v and the compact k_out, v_out; q_obs is always bf16).  Not from the paper,
 * whose caches are 16-bit: serving stacks also keep the cache as 8-bit floating point.
 *   FP8_E4M3: one byte per element, OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinity,
 *   S.1111.111 = NaN).  A key element counts as exactly the number its code encodes (the kernels widen it
 *   to bf16, which holds every E4M3 number, so the logits are the same as for that bf16 cache); a per-tensor
 *   dequantisation factor is folded into softmax_scale by the caller.  Strides stay in elements (= bytes) and
 *   the kv / out strides must be multiples of 16.  The gather copies codes bit for bit. */
enum { CODECOMP_KV_BF16 = 0, CODECOMP_KV_FP8_E4M3 = 1 };

/* How the structural prior enters the selection.
 * ADDITIVE : scores = pooled attention + lambda * prior, one top-(B - W) over them.
 * TWO_STAGE: the order stated in sections "Span-Level Structural Protection" / "Attention-based KV Cache
 *            Compression": first up to span-budget prefix tokens with prior > 0 are kept, largest prior
 *            first (equal priors: first in sequence), then pooled attention fills the remaining B - W - |P|
 *            slots among the other prefix tokens.  In this mode codecomp_score leaves the prior out
 *            (scores = pooled attention, prior_weight is ignored) and codecomp_compress selects with
 *            codecomp_select_two_stage. */
enum { CODECOMP_SELECT_ADDITIVE = 0, CODECOMP_SELECT_TWO_STAGE = 1 };

/* Host-only: bytes of device workspace the calls below need for these parameters (the largest
 * of score / select / compress).  Returns 0 when the parameters are invalid. Never touches a GPU. */
size_t codecomp_workspace_bytes(const codecomp_params* params);

/* Host-only: validates parameters exactly as the launching calls do (0 or a CODECOMP_E* code). */
int codecomp_validate(const codecomp_params* params);

/* Host-only: how codecomp_score lays the R = (n_q_heads / n_kv_heads) * window softmax rows of the
 * attention equation (section "Attention-based KV Cache Compression") over the wavefronts of a
 * workgroup.  Rows are cut into row_splits groups (one workgroup each) of row_blocks blocks of 32.
 * wave_desc[w], w < waves (array of 8): block of slot 0 | block of slot 1 << 8 | halves << 16; slot 0
 * is computed for both 32-key halves of every 64-key tile, slot 1 for the halves in `halves` (bit 0
 * first, bit 1 second, 0 = no slot 1).  Waves w and w + 4 share a SIMD; the layout evens out the
 * number of (block, half) units per SIMD.  For tests and tuning.  Returns 0 or a CODECOMP_E* code;
 * any output pointer may be NULL. */
int codecomp_score_layout(const codecomp_params* params, int32_t* row_splits, int32_t* row_blocks,
                          int32_t* waves, uint32_t* wave_desc);

/* scores[l][h][j] = pooled_u[l][h][j] + lambda * prior[j], where u is the window attention mass
 * of the equation above averaged over the query-head group, and pooled_u its zero-padded
 * stride-1 average over pool_kernel neighbours (divisor always pool_kernel), per request.
 * Logits and probabilities are computed in fp32 from the bf16 inputs (bf16 MFMA products are
 * exact, accumulation fp32).  workspace: >= codecomp_workspace_bytes(), 256-byte aligned. */
int codecomp_score(const void* q_obs, const void* k, const float* prior, const codecomp_params* params,
                   float* scores, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The kernels of codecomp_score, selectable one by one (a bit mask of CODECOMP_STAGE_*), in the
 * order row statistics -> row merge -> attention mass -> pool + prior.  Meant for per-kernel
 * timing and stage-wise debugging: a later stage reads what the earlier ones left in `workspace`,
 * so the stages of one problem must be enqueued in order with the same arguments.
 * CODECOMP_STAGE_ALL is exactly codecomp_score. */
enum {
  CODECOMP_STAGE_ROW_STATS = 1,   /* pass 1: per-chunk (max, sum) of every softmax row             */
  CODECOMP_STAGE_ROW_MERGE = 2,   /* log-sum-exp of every row over the chunks of its request       */
  CODECOMP_STAGE_MASS = 4,        /* pass 2: u(j) = sum over rows of softmax probabilities, / G    */
  CODECOMP_STAGE_FINISH = 8,      /* average pool + lambda * prior -> scores                       */
  CODECOMP_STAGE_ALL = 15
};
int codecomp_score_stages(const void* q_obs, const void* k, const float* prior, const codecomp_params* params,
                          float* scores, void* workspace, size_t workspace_bytes, unsigned stages,
                          void* hip_stream);

/* Per (layer, KV head, request): keep tokens N_r-W .. N_r-1, add the B_r - W tokens of the
 * prefix [0, N_r - W) with the largest scores (equal scores: the lower index wins; scores are
 * ordered as IEEE floats, -0 == +0, NaN unspecified), write the B_r indices in ascending
 * order.  Follows section "Attention-based KV Cache Compression": the best-scored context tokens are kept
 * until the remaining budget of the chunk is used up.  workspace (>= codecomp_workspace_bytes(), 256-byte aligned)
 * is scratch for long requests, which several workgroups select together; its contents on entry do not matter. */
int codecomp_select(const float* scores, const codecomp_params* params, int32_t* idx,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* The two-stage rule (see CODECOMP_SELECT_TWO_STAGE) on `scores` = pooled attention and the per-token
 * `prior`; params->select_mode must be CODECOMP_SELECT_TWO_STAGE.  Output as codecomp_select. */
int codecomp_select_two_stage(const float* scores, const float* prior, const codecomp_params* params, int32_t* idx,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* k_out[l][h][cu_budgets[r] + i][:] = k[l][h][cu_seqlens[r] + idx[l][h][cu_budgets[r] + i]][:],
 * same for v: a bit copy of the retained rows.  This builds the compressed chunk of section "Position
 * Encoding" (the retained tokens of a chunk, in their original order, which is what lets them keep their
 * original position indices), once per layer because section "Attention-based KV Cache Compression" applies the
 * compression independently at each transformer layer.  idx values must lie in [0, N_r) (values outside are
 * clamped into the request, so a corrupt index cannot read out of bounds); rows are moved as 16-byte pieces. */
int codecomp_gather(const void* k, const void* v, const int32_t* idx, const codecomp_params* params,
                    void* k_out, void* v_out, void* hip_stream);

/* The compression of section "Attention-based KV Cache Compression" from end to end, for every layer, KV head
 * and request of the batch: window attention mass (the equation of that section) -> pooled, fused with the
 * prior -> the best-scored context tokens kept up to the budget -> their K/V rows copied into the compact
 * cache.  Exactly codecomp_score, then codecomp_select (or codecomp_select_two_stage when
 * params->select_mode says so), then codecomp_gather, enqueued back to back on `hip_stream`; `scores` and
 * `idx` are outputs too.  Arguments, layouts and errors as for those calls; nothing is enqueued when an
 * argument is rejected. */
int codecomp_compress(const void* q_obs, const void* k, const void* v, const float* prior,
                      const codecomp_params* params, float* scores, int32_t* idx, void* k_out, void* v_out,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* For callers that cannot allocate device memory or bring a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): codecomp_compress with the same kernels, arguments, outputs
 * and errors, but without the workspace arguments.  The scratch memory lives in a device array inside the
 * library, CODECOMP_STATIC_SCRATCH_BYTES per GPU, held from the library's first use of that GPU until the
 * process ends; the call allocates and frees nothing.  Parameters whose codecomp_workspace_bytes() exceeds
 * CODECOMP_STATIC_SCRATCH_BYTES are rejected with CODECOMP_EINVAL_WORKSPACE before anything is enqueued.  All
 * calls on one GPU share that GPU's array (its contents are whatever the last call left; nothing needs to be
 * cleared): two calls whose kernels may run at the same time on one GPU - different streams, different threads -
 * race.  Calls on one stream, one after the other, are fine.  The first call on a device asks the runtime for
 * the array's address on that device (hipGetSymbolAddress): make it outside a graph capture. */
#define CODECOMP_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
int codecomp_compress_static(const void* q_obs, const void* k, const void* v, const float* prior,
                             const codecomp_params* params, float* scores, int32_t* idx, void* k_out, void* v_out,
                             void* hip_stream);

/* Str. Score of section "Experiment": retained[l][h][r] = |{kept tokens j of request r : prior[j] > 0}| /
 * |{tokens j of request r : prior[j] > 0}| (NaN when the request has no such token).  `retained` is a
 * device f32 [n_layers][n_kv_heads][n_seqs]; idx as written by codecomp_select. */
int codecomp_structure_score(const int32_t* idx, const float* prior, const codecomp_params* params, float* retained,
                             void* hip_stream);

/* Host-only arithmetic of sections "Structural Feature Extraction" and "Structure-Aware Budget Allocation"
 * (all pointers are HOST pointers; nothing touches a GPU).
 *   sigma_i = sum_k w_k * min(1, log(1 + f_ik) / log(1 + tau_k))          features [n_chunks][n_features] >= 0
 *   s_i = 0.5 if all sigma are equal, else (sigma_i - sigma_min) / max(eps, sigma_max - sigma_min)
 *   m_i = m_min + (m_max - m_min) * clip(s_i, 0, 1)
 *   B_i = floor(len_i * min(r_max, ratio * m_i)), then clamped into [window, len_i] because the hot path
 *         always keeps the observation window (pass window = 0 for the paper's bare formula).
 * The feature scales tau_k, weights w_k, eps, r_max are not given in the paper: they are arguments. */
int codecomp_chunk_structure_scores(const double* features_host, const double* tau_host, const double* weights_host,
                                    int32_t n_chunks, int32_t n_features, double* sigma_host);
int codecomp_chunk_budgets(const double* sigma_host, const int32_t* chunk_len_host, int32_t n_chunks, double ratio,
                           double m_min, double m_max, double r_max, double eps, int32_t window,
                           int32_t* budgets_host);

/* Host-only: static description of a status code returned by the calls above. */
const char* codecomp_status_string(int status);

/* Host-only: library version as major*10000 + minor*100 + patch. */
int codecomp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CODECOMP_H */
