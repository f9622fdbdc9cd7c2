// Host-side launch plan shared by the translation units of libcodecomp (internal header).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "codecomp.h"

namespace codecomp {

constexpr int kRowsPerWave = 64;      // query rows (window x group) one wavefront can own: two blocks of 32
constexpr int kMaxWaves = 8;          // wavefronts per workgroup in the score kernels
constexpr int kTileKeys = 64;         // keys staged through LDS per pipeline step
constexpr int kMaxScoreGrid = 2048;   // most workgroups a score pass is launched with
constexpr int kMinTilesPerWorkgroup = 4;
constexpr int kLeadTiles = 4;         // a segment start (query fragments, first K tile) costs about this many tiles
constexpr int kSelectThreads = 1024;  // one workgroup per (layer, head, request) in select, for short requests
constexpr int kSelectSmallThreads = 256;    // ... and in batches of many requests of at most 256 x 16 candidates
constexpr int kSelectSmallMaxItems = 16;
constexpr int kSelectSmallProblems = 1024;  // problems from which on the small workgroups are used
// Longer requests are selected by several workgroups each: parts of kPartChunk candidates, one 256-thread workgroup
// per part and step (first-digit counts, the candidates near the cut, the ordered output; between the last two one
// workgroup per request finishes the radix select on those candidates).
constexpr int kPartThreads = 256;
constexpr int kPartItems = 32;                             // candidates a thread holds
constexpr int kPartChunk = kPartThreads * kPartItems;      // candidates per part
constexpr int kSelectMaxCandidates = 65536;                // most candidates one workgroup keeps in registers (64 per thread)
constexpr int kPartMinCandidates = 16384;                  // few problems: parts are used from this many candidates on
constexpr int kPartFewProblems = 100;                      // (layer, head, request) problems below which one workgroup each leaves the device idle
constexpr int kFirstDigitBins = 2048;

struct Plan {
  int L, Hq, Hkv, G, d, W, pool, n_seqs;
  float lambda, scale;
  int select_mode;           // CODECOMP_SELECT_*
  int variant;               // CODECOMP_VARIANT_* flags
  int key_trim;              // keys at the end of every request that the softmax leaves out (W or 0)
  int kv_fp8;                // 1: k, v and the compact cache hold one FP8 E4M3 code per element (else bf16)
  float span_ratio; int span_min;
  int T, TB;                 // total tokens / total output slots over the packed requests
  int max_n;                 // longest request
  int R;                     // G * W softmax rows per (layer, KV head, request)
  int row_splits;            // workgroups along the row axis (each <= kMaxWaves * kRowsPerWave rows)
  int row_blocks;            // blocks of 32 rows per split
  int waves;                 // wavefronts per workgroup of the score passes
  // Which row blocks each wave computes: block of slot 0 | block of slot 1 << 8 | halves << 16, where
  // slot 0 covers both 32-key halves of every tile and `halves` (bit 0 first, bit 1 second) says which
  // ones slot 1 covers (0: the wave has no slot 1).
  uint32_t wave_desc[kMaxWaves];
  uint8_t rb_holder[2 * kMaxWaves][2];   // per row block: wave * 2 + slot of its (one or two) owners, 255 = none
  int grid_override;         // > 0: the caller fixed the number of workgroups of the score passes
  int lead_tiles;            // empty positions before each request's tiles in the sequence below: the cost of starting a segment
  int tiles_per_problem;     // sum over requests of (lead_tiles + ceil(N_r / kTileKeys)): positions of one (layer, head)
  int total_tiles;           // L * Hkv * tiles_per_problem, shared out evenly over the teams of row_splits workgroups
  int real_tiles;            // the same without the leads
  int64_t q_sl, q_ss, q_sh, q_st;
  int64_t kv_sl, kv_sh, kv_st;
  int64_t o_sl, o_sh, o_st;
  const int32_t* cu_seqlens_dev;
  const int32_t* cu_budgets_dev;
  // workspace layout (byte offsets, each 256-byte aligned)
  size_t off_stats, off_lse, off_uraw, off_member, off_member_count, ws_bytes;
  // selection by parts (0 parts: one workgroup per request does it all)
  int sel_parts;             // sum over requests of max(1, ceil((N_r - W) / kPartChunk))
  size_t off_part_hist, off_part_sure, off_part_head, off_part_before;
};

// Spreads `row_blocks` blocks over the waves of a workgroup (fills waves, wave_desc, rb_holder).
void assign_row_blocks(Plan* plan);

// Validates `p` and fills `plan`.  Returns 0 or a CODECOMP_E* code.  Host only, no HIP calls.
int make_plan(const codecomp_params* p, Plan* plan);

int launch_score(const Plan& pl, const void* q, const void* k, const float* prior, float* scores,
                 void* workspace, hipStream_t stream, unsigned stages = CODECOMP_STAGE_ALL);
int launch_select(const Plan& pl, const float* scores, int32_t* idx, void* workspace, hipStream_t stream);
int launch_select_two_stage(const Plan& pl, const float* scores, const float* prior, int32_t* idx, void* workspace,
                            hipStream_t stream);
int launch_gather(const Plan& pl, const void* k, const void* v, const int32_t* idx, void* k_out, void* v_out,
                  hipStream_t stream);

}  // namespace codecomp
