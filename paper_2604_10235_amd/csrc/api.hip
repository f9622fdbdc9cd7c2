// C ABI of libcodecomp: argument validation, workspace layout and the enqueue order of the
// score -> select -> gather path.  Everything here runs on the host; validation happens before
// the first HIP call so that rejected arguments never reach a GPU.
#include <math.h>

#include "plan.h"

namespace codecomp {

static inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// A wave runs on SIMD (wave % 4) of its compute unit (consecutive waves of a workgroup go to consecutive
// SIMDs), and a score workgroup with more than four waves has a compute unit to itself.  The cost of a
// wave is its number of (row block, half tile) units: 2 for a block it computes for both halves of every
// tile, 1 for a block it shares with another wave.  Up to 8 blocks: pairs of blocks per wave, as many
// waves as that takes (several such workgroups share a compute unit).  More: eight waves, one block each,
// and the remaining blocks dealt out so that the four SIMDs carry the same number of units (+-1).
void assign_row_blocks(Plan* pl) {
  const int nb = pl->row_blocks;
  for (int b = 0; b < 2 * kMaxWaves; ++b) pl->rb_holder[b][0] = pl->rb_holder[b][1] = 255;
  for (int w = 0; w < kMaxWaves; ++w) pl->wave_desc[w] = 0;
  auto hold = [&](int rb, int wave, int slot) {
    uint8_t* h = pl->rb_holder[rb];
    h[h[0] == 255 ? 0 : 1] = (uint8_t)(wave * 2 + slot);
  };
  if (nb <= 8) {
    pl->waves = (nb + 1) / 2;
    for (int w = 0; w < pl->waves; ++w) {
      const int rb0 = 2 * w, rb1 = 2 * w + 1;
      hold(rb0, w, 0);
      if (rb1 < nb) { hold(rb1, w, 1); pl->wave_desc[w] = (uint32_t)rb0 | ((uint32_t)rb1 << 8) | (3u << 16); }
      else pl->wave_desc[w] = (uint32_t)rb0;
    }
    return;
  }
  pl->waves = kMaxWaves;
  int extra[kMaxWaves];                       // half-tile units of a second block per wave: 0, 1 or 2
  const int units = 2 * (nb - kMaxWaves);     // 2 .. 16
  for (int s = 0; s < 4; ++s) {
    const int e = units / 4 + (s < units % 4 ? 1 : 0);
    extra[s] = e < 2 ? e : 2;
    extra[s + 4] = e - extra[s];
  }
  int next = kMaxWaves;                       // next block to hand out
  for (int w = 0; w < kMaxWaves; ++w) {
    hold(w, w, 0);
    pl->wave_desc[w] = (uint32_t)w;
    if (extra[w] == 2) { hold(next, w, 1); pl->wave_desc[w] |= ((uint32_t)next << 8) | (3u << 16); ++next; }
  }
  int pending = -1;                           // wave that took the first half of block `next`
  for (int w = 0; w < kMaxWaves; ++w) {
    if (extra[w] != 1) continue;
    hold(next, w, 1);
    if (pending < 0) { pl->wave_desc[w] |= ((uint32_t)next << 8) | (1u << 16); pending = w; }
    else { pl->wave_desc[w] |= ((uint32_t)next << 8) | (2u << 16); pending = -1; ++next; }
  }
}

int make_plan(const codecomp_params* p, Plan* pl) {
  if (!p) return CODECOMP_EINVAL_NULL;
  if (p->n_layers < 1 || p->n_seqs < 1 || p->n_seqs > 65535) return CODECOMP_EINVAL_SHAPE;
  if (p->select_mode != CODECOMP_SELECT_ADDITIVE && p->select_mode != CODECOMP_SELECT_TWO_STAGE) return CODECOMP_EINVAL_MODE;
  if (p->select_mode == CODECOMP_SELECT_TWO_STAGE &&
      (!(p->span_budget_ratio >= 0.0f) || !(p->span_budget_ratio <= 1.0f) || p->span_budget_min < 0))
    return CODECOMP_EINVAL_MODE;
  constexpr int kKnownVariants = CODECOMP_VARIANT_GROUP_SUM | CODECOMP_VARIANT_GROUP_MAX | CODECOMP_VARIANT_POOL_MAX |
                                 CODECOMP_VARIANT_SOFTMAX_PREFIX | CODECOMP_VARIANT_POOL_PREFIX;
  if ((p->score_variant & ~kKnownVariants) != 0) return CODECOMP_EINVAL_MODE;
  if (p->kv_dtype != CODECOMP_KV_BF16 && p->kv_dtype != CODECOMP_KV_FP8_E4M3) return CODECOMP_EINVAL_MODE;
  if ((p->score_variant & CODECOMP_VARIANT_GROUP_SUM) && (p->score_variant & CODECOMP_VARIANT_GROUP_MAX)) return CODECOMP_EINVAL_MODE;
  if ((int64_t)p->n_layers * p->n_kv_heads > 65535) return CODECOMP_EINVAL_SHAPE;   // one grid axis
  if (p->n_kv_heads < 1 || p->n_q_heads < 1 || p->n_q_heads % p->n_kv_heads != 0) return CODECOMP_EINVAL_HEADS;
  if (p->head_dim != 64 && p->head_dim != 128) return CODECOMP_EINVAL_HEADDIM;
  if (p->pool_kernel < 1 || p->pool_kernel % 2 == 0 || p->pool_kernel > 1025) return CODECOMP_EINVAL_POOL;
  if (!(p->prior_weight >= 0.0f) || !isfinite(p->prior_weight)) return CODECOMP_EINVAL_PRIOR;
  if (!(p->softmax_scale >= 0.0f) || !isfinite(p->softmax_scale)) return CODECOMP_EINVAL_PRIOR;
  if (!p->cu_seqlens_host || !p->cu_seqlens_dev || !p->cu_budgets_host || !p->cu_budgets_dev)
    return CODECOMP_EINVAL_NULL;
  if (p->window < 1) return CODECOMP_EINVAL_WINDOW;
  if (p->cu_seqlens_host[0] != 0 || p->cu_budgets_host[0] != 0) return CODECOMP_EINVAL_SEQLENS;
  int max_n = 0;
  for (int r = 0; r < p->n_seqs; ++r) {
    int64_t n = (int64_t)p->cu_seqlens_host[r + 1] - p->cu_seqlens_host[r];
    int64_t b = (int64_t)p->cu_budgets_host[r + 1] - p->cu_budgets_host[r];
    if (n < 1 || b < 0) return CODECOMP_EINVAL_SEQLENS;
    if (p->window > n) return CODECOMP_EINVAL_WINDOW;
    if (b < p->window || b > n) return CODECOMP_EINVAL_BUDGET;
    if (n > max_n) max_n = (int)n;
  }
  const int64_t strides[] = {p->q_stride_layer, p->q_stride_seq, p->q_stride_head, p->q_stride_tok,
                             p->kv_stride_layer, p->kv_stride_head, p->kv_stride_tok,
                             p->out_stride_layer, p->out_stride_head, p->out_stride_tok};
  for (int64_t s : strides)
    if (s < 0 || s % 8 != 0) return CODECOMP_EINVAL_SHAPE;   // rows are moved as 16-byte pieces
  if (p->kv_dtype == CODECOMP_KV_FP8_E4M3)                   // ... which hold 16 one-byte elements
    for (int i = 4; i < 10; ++i)
      if (strides[i] % 16 != 0) return CODECOMP_EINVAL_SHAPE;

  pl->L = p->n_layers; pl->Hq = p->n_q_heads; pl->Hkv = p->n_kv_heads; pl->G = pl->Hq / pl->Hkv;
  pl->d = p->head_dim; pl->W = p->window; pl->pool = p->pool_kernel; pl->n_seqs = p->n_seqs;
  pl->select_mode = p->select_mode;
  pl->variant = p->score_variant;
  pl->kv_fp8 = p->kv_dtype == CODECOMP_KV_FP8_E4M3 ? 1 : 0;
  pl->key_trim = (p->score_variant & CODECOMP_VARIANT_SOFTMAX_PREFIX) ? p->window : 0;
  pl->span_ratio = p->span_budget_ratio; pl->span_min = p->span_budget_min;
  // two-stage selection keeps the prior out of the scores: structure is handled by the selection itself
  pl->lambda = p->select_mode == CODECOMP_SELECT_TWO_STAGE ? 0.0f : p->prior_weight;
  pl->scale = p->softmax_scale > 0.0f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
  pl->T = p->cu_seqlens_host[p->n_seqs];
  pl->TB = p->cu_budgets_host[p->n_seqs];
  pl->max_n = max_n;
  int64_t R = (int64_t)pl->G * pl->W;
  if (R > (1 << 16)) return CODECOMP_EINVAL_SHAPE;
  pl->R = (int)R;
  const int max_rows = kMaxWaves * kRowsPerWave;
  pl->row_splits = (pl->R + max_rows - 1) / max_rows;
  int per = (pl->R + pl->row_splits - 1) / pl->row_splits;
  pl->row_blocks = (per + 31) / 32;
  assign_row_blocks(pl);
  // the largest head mass is taken per workgroup from whole row blocks: one head per block, all rows in one workgroup
  if ((pl->variant & CODECOMP_VARIANT_GROUP_MAX) && (pl->W % 32 != 0 || pl->row_splits != 1)) return CODECOMP_EINVAL_MODE;
  if (p->score_workgroups < 0 || p->score_lead_tiles > 64) return CODECOMP_EINVAL_SHAPE;
  pl->grid_override = p->score_workgroups;
  pl->lead_tiles = p->score_lead_tiles == 0 ? kLeadTiles : (p->score_lead_tiles < 0 ? 0 : p->score_lead_tiles);
  int64_t tiles = 0;
  for (int r = 0; r < p->n_seqs; ++r) {
    int n = p->cu_seqlens_host[r + 1] - p->cu_seqlens_host[r] - pl->key_trim;     // >= 0: W <= N_r was checked
    tiles += (n + kTileKeys - 1) / kTileKeys;
  }
  const int64_t problems = (int64_t)pl->L * pl->Hkv * pl->row_splits;
  const int64_t positions = tiles + (int64_t)pl->lead_tiles * pl->n_seqs;
  if (positions * problems > (1 << 30)) return CODECOMP_EINVAL_SHAPE;
  pl->tiles_per_problem = (int)positions;
  pl->total_tiles = (int)(positions * pl->L * pl->Hkv);      // the row splits of a problem walk the same positions
  pl->real_tiles = (int)(tiles * pl->L * pl->Hkv);

  const int64_t d = pl->d;
  pl->q_st = p->q_stride_tok ? p->q_stride_tok : d;
  pl->q_sh = p->q_stride_head ? p->q_stride_head : (int64_t)pl->W * d;
  pl->q_ss = p->q_stride_seq ? p->q_stride_seq : (int64_t)pl->Hq * pl->W * d;
  pl->q_sl = p->q_stride_layer ? p->q_stride_layer : (int64_t)pl->n_seqs * pl->Hq * pl->W * d;
  pl->kv_st = p->kv_stride_tok ? p->kv_stride_tok : d;
  pl->kv_sh = p->kv_stride_head ? p->kv_stride_head : (int64_t)pl->T * d;
  pl->kv_sl = p->kv_stride_layer ? p->kv_stride_layer : (int64_t)pl->Hkv * pl->T * d;
  pl->o_st = p->out_stride_tok ? p->out_stride_tok : d;
  pl->o_sh = p->out_stride_head ? p->out_stride_head : (int64_t)pl->TB * d;
  pl->o_sl = p->out_stride_layer ? p->out_stride_layer : (int64_t)pl->Hkv * pl->TB * d;
  if (pl->q_st < d || pl->kv_st < d || pl->o_st < d) return CODECOMP_EINVAL_SHAPE;
  if (pl->kv_st > (1 << 20)) return CODECOMP_EINVAL_SHAPE;   // tile staging keeps 32-bit byte offsets inside a tile
  pl->cu_seqlens_dev = p->cu_seqlens_dev;
  pl->cu_budgets_dev = p->cu_budgets_dev;

  // workspace: per-chunk softmax statistics, merged row normalisers, raw attention mass
  const size_t LH = (size_t)pl->L * pl->Hkv;
  const size_t lpad = (size_t)pl->row_splits * pl->row_blocks * 32;        // normaliser rows
  size_t off = 0;
  // one statistics slot per segment and row split; slot numbers stay below (teams + problems) * row_splits
  const size_t slots = (size_t)kMaxScoreGrid + LH * pl->row_splits * pl->n_seqs;
  pl->off_stats = off; off = align256(off + slots * (pl->waves * kRowsPerWave) * 2 * sizeof(float));
  pl->off_lse = off;   off = align256(off + LH * pl->n_seqs * lpad * sizeof(float));
  pl->off_uraw = off;  off = align256(off + (size_t)pl->row_splits * LH * pl->T * sizeof(float));
  pl->off_member = off; off = align256(off + (size_t)pl->T);
  pl->off_member_count = off; off = align256(off + (size_t)pl->n_seqs * sizeof(int32_t));
  // selection by parts: per (layer*head, part) the first-digit counts and the number of candidates admitted whatever
  // the cut; per (layer*head, request) what the parts agreed on.  The keys near the cut reuse the raw attention mass
  // (dead once the scores exist): one 32-bit word per token and layer*head, exactly its size.
  pl->sel_parts = 0;
  const int max_npre = max_n - p->window;
  if (max_npre > kSelectMaxCandidates || (max_npre >= kPartMinCandidates && LH * (size_t)p->n_seqs < (size_t)kPartFewProblems)) {
    int64_t parts = 0;
    for (int r = 0; r < p->n_seqs; ++r) {
      const int npre = p->cu_seqlens_host[r + 1] - p->cu_seqlens_host[r] - p->window;
      parts += npre > kPartChunk ? (npre + kPartChunk - 1) / kPartChunk : 1;
    }
    if (parts > (1 << 24)) return CODECOMP_EINVAL_SHAPE;
    pl->sel_parts = (int)parts;
    pl->off_part_hist = off; off = align256(off + LH * (size_t)parts * kFirstDigitBins * sizeof(uint16_t));
    pl->off_part_sure = off; off = align256(off + LH * (size_t)parts * sizeof(int32_t));
    pl->off_part_head = off; off = align256(off + LH * (size_t)pl->n_seqs * 8 * sizeof(uint32_t));
    pl->off_part_before = off; off = align256(off + LH * (size_t)parts * 2 * sizeof(int32_t));
  }
  pl->ws_bytes = off;
  return CODECOMP_OK;
}

static int check_ws(const Plan& pl, const void* ws, size_t bytes) {
  if (!ws || ((uintptr_t)ws & 255) != 0 || bytes < pl.ws_bytes) return CODECOMP_EINVAL_WORKSPACE;
  return CODECOMP_OK;
}

static bool misaligned16(const void* p) { return ((uintptr_t)p & 15) != 0; }

}  // namespace codecomp

using namespace codecomp;

extern "C" {

size_t codecomp_workspace_bytes(const codecomp_params* params) {
  Plan pl;
  if (make_plan(params, &pl) != CODECOMP_OK) return 0;
  return pl.ws_bytes;
}

int codecomp_validate(const codecomp_params* params) {
  Plan pl;
  return make_plan(params, &pl);
}

int codecomp_score_layout(const codecomp_params* params, int32_t* row_splits, int32_t* row_blocks,
                          int32_t* waves, uint32_t* wave_desc) {
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  if (row_splits) *row_splits = pl.row_splits;
  if (row_blocks) *row_blocks = pl.row_blocks;
  if (waves) *waves = pl.waves;
  if (wave_desc)
    for (int w = 0; w < kMaxWaves; ++w) wave_desc[w] = w < pl.waves ? pl.wave_desc[w] : 0u;
  return CODECOMP_OK;
}

int codecomp_score(const void* q_obs, const void* k, const float* prior, const codecomp_params* params,
                   float* scores, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!q_obs || !k || !prior || !params || !scores) return CODECOMP_EINVAL_NULL;
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  if (misaligned16(q_obs) || misaligned16(k)) return CODECOMP_EINVAL_SHAPE;
  if (int rc = check_ws(pl, workspace, workspace_bytes)) return rc;
  return launch_score(pl, q_obs, k, prior, scores, workspace, (hipStream_t)hip_stream);
}

int codecomp_score_stages(const void* q_obs, const void* k, const float* prior, const codecomp_params* params,
                          float* scores, void* workspace, size_t workspace_bytes, unsigned stages,
                          void* hip_stream) {
  if (!q_obs || !k || !prior || !params || !scores) return CODECOMP_EINVAL_NULL;
  if (stages == 0 || (stages & ~(unsigned)CODECOMP_STAGE_ALL)) return CODECOMP_EINVAL_SHAPE;
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  if (misaligned16(q_obs) || misaligned16(k)) return CODECOMP_EINVAL_SHAPE;
  if (int rc = check_ws(pl, workspace, workspace_bytes)) return rc;
  return launch_score(pl, q_obs, k, prior, scores, workspace, (hipStream_t)hip_stream, stages);
}

int codecomp_select(const float* scores, const codecomp_params* params, int32_t* idx, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (!scores || !params || !idx) return CODECOMP_EINVAL_NULL;
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  if (pl.select_mode != CODECOMP_SELECT_ADDITIVE) return CODECOMP_EINVAL_MODE;   // the prior is needed: other entry
  if (int rc = check_ws(pl, workspace, workspace_bytes)) return rc;
  return launch_select(pl, scores, idx, workspace, (hipStream_t)hip_stream);
}

int codecomp_select_two_stage(const float* scores, const float* prior, const codecomp_params* params, int32_t* idx,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!scores || !prior || !params || !idx) return CODECOMP_EINVAL_NULL;
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  if (pl.select_mode != CODECOMP_SELECT_TWO_STAGE) return CODECOMP_EINVAL_MODE;
  if (int rc = check_ws(pl, workspace, workspace_bytes)) return rc;
  return launch_select_two_stage(pl, scores, prior, idx, workspace, (hipStream_t)hip_stream);
}

int codecomp_gather(const void* k, const void* v, const int32_t* idx, const codecomp_params* params,
                    void* k_out, void* v_out, void* hip_stream) {
  if (!k || !v || !idx || !params || !k_out || !v_out) return CODECOMP_EINVAL_NULL;
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  if (misaligned16(k) || misaligned16(v) || misaligned16(k_out) || misaligned16(v_out)) return CODECOMP_EINVAL_SHAPE;
  return launch_gather(pl, k, v, idx, k_out, v_out, (hipStream_t)hip_stream);
}

int codecomp_compress(const void* q_obs, const void* k, const void* v, const float* prior,
                      const codecomp_params* params, float* scores, int32_t* idx, void* k_out, void* v_out,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!q_obs || !k || !v || !prior || !params || !scores || !idx || !k_out || !v_out) return CODECOMP_EINVAL_NULL;
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  if (misaligned16(q_obs) || misaligned16(k) || misaligned16(v) || misaligned16(k_out) || misaligned16(v_out))
    return CODECOMP_EINVAL_SHAPE;
  if (int rc = check_ws(pl, workspace, workspace_bytes)) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  if (int rc = launch_score(pl, q_obs, k, prior, scores, workspace, s)) return rc;
  if (pl.select_mode == CODECOMP_SELECT_TWO_STAGE) {
    if (int rc = launch_select_two_stage(pl, scores, prior, idx, workspace, s)) return rc;
  } else {
    if (int rc = launch_select(pl, scores, idx, workspace, s)) return rc;
  }
  return launch_gather(pl, k, v, idx, k_out, v_out, s);
}

const char* codecomp_status_string(int status) {
  switch (status) {
    case CODECOMP_OK: return "ok";
    case CODECOMP_EINVAL_NULL: return "a required pointer is NULL";
    case CODECOMP_EINVAL_SHAPE: return "bad shape, stride or alignment";
    case CODECOMP_EINVAL_WINDOW: return "window must satisfy 1 <= W <= N_r for every request";
    case CODECOMP_EINVAL_BUDGET: return "budget must satisfy W <= B_r <= N_r for every request";
    case CODECOMP_EINVAL_POOL: return "pool_kernel must be odd and >= 1";
    case CODECOMP_EINVAL_HEADS: return "n_q_heads must be a positive multiple of n_kv_heads";
    case CODECOMP_EINVAL_HEADDIM: return "head_dim must be 64 or 128";
    case CODECOMP_EINVAL_SEQLENS: return "cu_seqlens / cu_budgets must start at 0 and increase";
    case CODECOMP_EINVAL_WORKSPACE: return "workspace is NULL, not 256-byte aligned or too small";
    case CODECOMP_EINVAL_PRIOR: return "prior_weight / softmax_scale must be finite and >= 0";
    case CODECOMP_EINVAL_MODE: return "select_mode unknown or wrong for this call, or span budget out of range";
    default: return status > 0 ? "HIP runtime error (hipError_t value)" : "unknown status";
  }
}

int codecomp_version(void) { return 100; }

}  // extern "C"
