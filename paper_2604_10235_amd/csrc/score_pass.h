// Internal header: the two MFMA passes of the score step and their launch code (score.hip holds the small
// kernels and the entry; score_pass_*.hip instantiate the passes).
//
// Score step: window attention mass -> group mean -> average pool -> + lambda * prior.
//
// For one (layer, KV head, request) the R = G*W observation rows are soft-maxed over all N_r
// keys and summed per key (the equation of section "Attention-based KV Cache Compression").
// A column sum of a row softmax needs every row normaliser first, so the logits are formed
// twice on the matrix cores:
//   pass 1  S^T tile = K Q^T   (lane = query row)  -> per-row running (max, sum) -> per-segment stats
//   merge   per-row log2-sum-exp over the segments of a request
//   pass 2  S tile   = Q K^T   (lane = key)        -> exp2(s*c - lse) summed over rows -> u
//   finish  average pool over pool_kernel neighbours inside the request, add lambda * prior
// Both passes keep a wave's query rows as MFMA fragments in registers for the whole
// workgroup lifetime and stream 64-key tiles of K through LDS (double buffered, one barrier
// per tile).  Rows come in blocks of 32 (one MFMA tile side); a wave owns one block outright
// (slot 0) and possibly a second one (slot 1) for both 32-key halves of every tile, for the
// first half only or for the second half only.  Half ownership lets the host spread a block
// count that four SIMDs cannot share evenly (14 blocks for 7 query heads x 64 window rows):
// waves w and w+4 run on the same SIMD, and every SIMD ends up with the same number of
// (row block, half tile) units.  v_mfma_f32_32x32x16_bf16: the A and B fragments have the same lane layout
// (lane%32 = row/column, lane/32 = which 8 of the 16 k values), so swapping the operands
// transposes the output tile without touching the loads.
#pragma once
#include <atomic>
#include <type_traits>

#include "plan.h"

namespace codecomp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// 16-byte register quantum for loads/stores and MFMA fragments (a native vector: plain loads, no struct copies)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

struct ScoreArgs {
  const uint16_t* q;
  const unsigned char* k;   // keys: bf16 patterns, or one FP8 E4M3 code per element (strides stay in elements)
  const int32_t* cu_seqlens;
  float* stats;   // [segment slot][waves*64][2] : (max * c, sum of exp2(s*c - max*c)) per wave slot row
  float* lse;     // [L*Hkv][n_seqs][lrows]         : log2 sum_j exp2(s_j * c), lrows = row_splits * nb * 32
  float* uraw;    // [row_splits][L*Hkv][T]         : (1/G) * sum over this split's rows of A
  int n_seqs, Hkv, LH, G, W, R, row_splits, nb, srows, lrows, T;
  // Work distribution.  The 64-key tiles of all problems (layer*head, request), in that order, form one
  // sequence.  The workgroups of a launch form teams of row_splits members (one per row split; a team of one
  // when all rows fit one workgroup); team q of `teams` takes positions [q*total/teams, (q+1)*total/teams) and
  // every member walks through the "segments" in which that range meets the problems, for its own rows.  The
  // members of a team run on the same accelerator die and stream the same keys at the same time, so that all
  // but the first of them find a K tile in that die's L2.  Every problem is preceded by
  // `lead` empty positions: starting a segment costs about that many tiles (query fragments, first K
  // tile), so a range that crosses into a new problem gets that many tiles less, and all workgroups
  // finish together.  Pass 1 leaves the statistics of the segment of team q in problem p = layer*head * n_seqs +
  // request, row split s, in slot (q + p) * row_splits + s (distinct for distinct segments: along the sequence
  // neither q nor p decreases and one of them grows from one segment to the next).
  int lead;                          // empty positions before the tiles of each problem
  int tiles_per_problem;             // sum over requests of (lead + ceil(N_r / 64))
  int total_tiles;                   // L*Hkv * tiles_per_problem
  int stat_teams;                    // teams of the pass-1 launch whose statistics `stats` holds
  int key_trim;                      // keys at the end of every request left out of the softmax (prefix-only variant)
  int blocks_per_head;               // largest-head-mass variant: row blocks of one query head (window / 32)
  uint32_t wave_desc[kMaxWaves];     // row block of slot 0 | row block of slot 1 << 8 | halves of slot 1 << 16 (bit 0: first, bit 1: second)
  uint8_t rb_holder[2 * kMaxWaves][2];   // per row block: the (wave * 2 + slot) indices that hold its statistics, 255 = none
  int64_t q_sl, q_ss, q_sh, q_st, kv_sl, kv_sh, kv_st;
  float c;        // softmax_scale * log2(e)
  float inv_g;
};

#define NEG_BIG (-1.0e30f)


__device__ __forceinline__ bf16x8 frag(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// What goes into the LDS tile for one staged piece of 8 key elements: bf16 as it is; 8 FP8 E4M3 codes widened to
// bf16 (exact: every E4M3 number is a bf16 number).  v_cvt_scalef32_pk_bf16_fp8 turns the two codes in the low
// or the high half of its source into two bf16, times a power of two taken from the float operand (2^0 here).
__device__ __forceinline__ u32x4 to_bf16x8(u32x4 v) { return v; }
__device__ __forceinline__ u32x4 to_bf16x8(u32x2 v) {
  u32x4 r;
  r.x = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v.x, 1.0f, false));
  r.y = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v.x, 1.0f, true));
  r.z = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v.y, 1.0f, false));
  r.w = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v.y, 1.0f, true));
  return r;
}

// Positions that request r takes in the tile sequence of a problem: its lead and its tiles.
__device__ __forceinline__ int tiles_of(int len, int trim) { return (len - trim + kTileKeys - 1) / kTileKeys; }

// Where a workgroup enters a problem's sequence: the request that holds position `xr` and the position at which
// that request's lead begins.  All threads of the workgroup call it together (two barriers): every thread adds up
// a contiguous share of the requests, a prefix sum over the threads finds the share that holds xr, and its owner
// walks that share.  The segment loop then only ever steps from one request to the next.
template <int NT>
__device__ __forceinline__ void locate_first(const int32_t* cu, int n_seqs, int lead, int trim, int xr, int& seq, int& acc) {
  __shared__ int wave_total[NT / 64];
  __shared__ int found[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (n_seqs + NT - 1) / NT;
  const int r0 = min(tid * per, n_seqs), r1 = min(r0 + per, n_seqs);
  int mine = 0;
  for (int r = r0; r < r1; ++r) mine += lead + tiles_of(cu[r + 1] - cu[r], trim);
  int incl = mine;                                   // inclusive prefix sum inside the wave
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int up = __shfl_up(incl, off);
    if (lane >= off) incl += up;
  }
  if (lane == 63) wave_total[wave] = incl;
  if (tid == 0) { found[0] = n_seqs - 1; found[1] = -1; }
  __syncthreads();
  int start = incl - mine;
  for (int w = 0; w < wave; ++w) start += wave_total[w];
  if (xr >= start && xr < start + mine) {            // exactly one thread, when xr lies inside the sequence
    int pos = start, r = r0;
    for (;; ++r) {
      const int span = lead + tiles_of(cu[r + 1] - cu[r], trim);
      if (xr < pos + span) break;
      pos += span;
    }
    found[0] = r; found[1] = pos;
  }
  __syncthreads();
  seq = found[0]; acc = found[1];
  if (acc < 0) {                                     // past the end (never for a position inside the sequence): last request
    acc = 0;
    for (int r = 0; r < n_seqs - 1; ++r) acc += lead + tiles_of(cu[r + 1] - cu[r], trim);
  }
}

// Team (of `wgs`) whose tile range [g*total/wgs, (g+1)*total/wgs) holds tile x.
__device__ __forceinline__ int wg_of_tile(int x, int total, int wgs) {
  return (int)((((int64_t)x + 1) * wgs + total - 1) / total) - 1;
}

// Team and row split of workgroup b in a launch of `grid` workgroups (grid = teams * row_splits).  Workgroups are
// handed to the eight accelerator dies in turn (b % 8), so the members of a team are 8 apart wherever the number of
// teams allows it: they then share a die, and its L2.
__host__ __device__ __forceinline__ void team_of(int b, int grid, int row_splits, int& team, int& split) {
  if (row_splits == 1) { team = b; split = 0; return; }
  if (grid % (8 * row_splits) == 0) {
    const int die = b & 7, t = b >> 3;
    team = 8 * (t / row_splits) + die;
    split = t % row_splits;
  } else {
    team = b / row_splits;
    split = b % row_splits;
  }
}

// MFMA helper: D = A * B + C on one 32x32x16 bf16 step.  PASS 1 puts the keys on the A side
// (output lane = query row), PASS 2 the queries (output lane = key).
template <int PASS>
__device__ __forceinline__ f32x16 mma_step(u32x4 qfrag, u32x4 kfrag, f32x16 acc) {
  if constexpr (PASS == 1)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(kfrag), frag(qfrag), acc, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(qfrag), frag(kfrag), acc, 0, 0, 0);
}

// GMAX (pass 2 only): the largest query-head mass of the group instead of the (scaled) sum over its heads.
// K8: the keys are FP8 E4M3 codes; they are widened to bf16 on their way into LDS, everything after is the same.
template <int D, int NW, int PASS, bool GMAX = false, bool K8 = false>
__global__ __launch_bounds__(NW * 64, (NW >= 3 ? 2 : 1)) void score_pass_kernel(ScoreArgs a) {
  static_assert(PASS == 2 || !GMAX, "the group reduction happens in pass 2");
  constexpr int NT = NW * 64;
  constexpr int KS = D / 16;                   // MFMA k-steps per logit
  constexpr int ROWB = D * 2 + 16;             // LDS bytes per key row (+16: spreads rows over banks)
  constexpr int CH_PER_ROW = D / 8;            // pieces of 8 elements per key row (16 bytes in LDS)
  constexpr int ESZ = K8 ? 1 : 2;              // bytes per stored key element
  using stage_t = std::conditional_t<K8, u32x2, u32x4>;   // one piece as loaded
  constexpr int NCH = kTileKeys * CH_PER_ROW;  // pieces per tile
  constexpr int LD = (NCH + NT - 1) / NT;      // pieces staged per thread
  constexpr int LDS_ROWS = LD * NT / CH_PER_ROW;   // >= kTileKeys: rows past the tile are staging slack, never read
  static_assert(LDS_ROWS >= kTileKeys, "tile staging");

  __shared__ __attribute__((aligned(16))) unsigned char ktile[2][LDS_ROWS * ROWB];
  // pass 2: column partials of the last four tiles, one row per (wave, half wave); with group_max one
  // row per (wave, slot, half wave), because the two slots of a wave may belong to different query heads
  __shared__ float colbuf[PASS == 2 ? 4 : 1][PASS == 2 ? NW * (GMAX ? 4 : 2) : 1][kTileKeys];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hf = lane >> 5;
  // ---- what this wave owns (the same for every lane: keep it in scalar registers)
  const uint32_t desc = __builtin_amdgcn_readfirstlane(a.wave_desc[wave]);
  const int rb_of[2] = {(int)(desc & 255u), (int)((desc >> 8) & 255u)};
  const uint32_t halves1 = (desc >> 16) & 3u;              // halves of every tile that slot 1 computes

  // ---- this workgroup's share of the tile sequence, one segment (part of one problem) at a time
  int team, split;
  team_of((int)blockIdx.x, (int)gridDim.x, a.row_splits, team, split);
  team = __builtin_amdgcn_readfirstlane(team);
  split = __builtin_amdgcn_readfirstlane(split);
  const int teams = (int)gridDim.x / a.row_splits;
  const int x_begin = (int)((int64_t)team * a.total_tiles / teams);
  const int x_end = (int)((int64_t)(team + 1) * a.total_tiles / teams);
  // the request the walk stands in: request cur_seq of problem cur_lz, whose lead begins at position cur_acc
  int cur_lz = x_begin / a.tiles_per_problem, cur_seq = 0, cur_acc = 0;
  if (a.n_seqs > 16 && x_begin < x_end)                      // few requests: walking there from the first one is as quick
    locate_first<NT>(a.cu_seqlens, a.n_seqs, a.lead, a.key_trim, x_begin - cur_lz * a.tiles_per_problem, cur_seq, cur_acc);
  cur_seq = __builtin_amdgcn_readfirstlane(cur_seq);         // the same in every lane: scalar registers from here on
  cur_acc = __builtin_amdgcn_readfirstlane(cur_acc);
  for (int x = x_begin; x < x_end;) {
  const int lz = x / a.tiles_per_problem;                  // layer * Hkv + head
  const int layer = lz / a.Hkv;
  const int head = lz - layer * a.Hkv;
  if (lz != cur_lz) { cur_lz = lz; cur_seq = 0; cur_acc = 0; }     // crossed into the next problem: its first request
  const int xr = x - lz * a.tiles_per_problem;
  int tok0 = a.cu_seqlens[cur_seq], tok1 = a.cu_seqlens[cur_seq + 1];
  int tiles_of_seq = tiles_of(tok1 - tok0, a.key_trim);
  while (xr >= cur_acc + a.lead + tiles_of_seq && cur_seq < a.n_seqs - 1) {       // usually no step or one
    cur_acc += a.lead + tiles_of_seq;
    ++cur_seq;
    tok0 = tok1; tok1 = a.cu_seqlens[cur_seq + 1];
    tiles_of_seq = tiles_of(tok1 - tok0, a.key_trim);
  }
  const int seq = cur_seq, n = tok1 - tok0 - a.key_trim;     // keys of the request: all but the last key_trim
  int tile_in_seq = xr - cur_acc - a.lead;                   // < 0 inside the lead
  if (tile_in_seq < 0) {                                    // inside the lead: the problem's tiles start after it
    x -= tile_in_seq;
    tile_in_seq = 0;
    if (x >= x_end) break;
  }
  if (tile_in_seq >= tiles_of_seq) continue;                // a request without keys (prefix-only softmax, N == W)
  const int ntiles = min(x_end - x, tiles_of_seq - tile_in_seq);
  const int kstart = tile_in_seq * kTileKeys;
  const int kend = min(n, kstart + ntiles * kTileKeys);
  const int rem = (kend - kstart) & (kTileKeys - 1);        // keys of a partial last tile (0 = it is full)
  const int split_row0 = split * a.nb * 32;

  // ---- K tile staging: global -> registers -> LDS.  Rows past the end of the chunk re-read its
  // last key (always in bounds); such columns are masked (pass 1) or never stored (pass 2).
  const unsigned char* kb = a.k + ((int64_t)layer * a.kv_sl + (int64_t)head * a.kv_sh + (int64_t)tok0 * a.kv_st) * ESZ;
  // Workgroups of four or eight waves keep two tiles in flight in two register sets in pass 2: a tile that
  // arrives late stalls every SIMD the workgroup runs on.  (Measured: 4% off pass 2 with eight waves, one
  // workgroup per compute unit; 6% with four waves, two per unit; nothing off pass 1, whose loop is the
  // shorter one.)
  constexpr bool DEEP = NW >= 4 && PASS == 2;
  stage_t stage[LD];
  stage_t stage2[DEEP ? LD : 1];
  // byte offset of this thread's first piece inside a tile; its i-th piece is NT / CH_PER_ROW rows further
  static_assert(NT % CH_PER_ROW == 0, "pieces of one thread share a column");
  const uint32_t soff0 = (uint32_t)((tid / CH_PER_ROW) * (int)a.kv_st + (tid % CH_PER_ROW) * 8) * (uint32_t)ESZ;
  const uint32_t sstep = (uint32_t)((NT / CH_PER_ROW) * (int)a.kv_st) * (uint32_t)ESZ;
  // fast path: every staged row (slack rows included) lies inside the chunk -> uniform base + lane offset
#define CODECOMP_GLOAD(KEY0, ST)                                                                    \
  {                                                                                                 \
    const int key0_ = (KEY0);                                                                       \
    if (key0_ + LDS_ROWS <= kend) {                                                                 \
      const unsigned char* tb_ = kb + (int64_t)key0_ * a.kv_st * ESZ;                              \
      _Pragma("unroll") for (int i = 0; i < LD; ++i)                                                \
        ST[i] = *reinterpret_cast<const stage_t*>(tb_ + (size_t)i * sstep + soff0);                 \
    } else {                                                                                        \
      _Pragma("unroll") for (int i = 0; i < LD; ++i) {                                              \
        const int cidx = tid + i * NT;                                                              \
        const int row = cidx / CH_PER_ROW, col = cidx - row * CH_PER_ROW;                           \
        const int key = min(key0_ + row, kend - 1);                                                 \
        ST[i] = *reinterpret_cast<const stage_t*>(kb + ((int64_t)key * a.kv_st + col * 8) * ESZ);   \
      }                                                                                             \
    }                                                                                               \
  }
#define CODECOMP_SSTORE(BUF, ST)                                                                    \
  _Pragma("unroll") for (int i = 0; i < LD; ++i) {                                                  \
    const int cidx = tid + i * NT;                                                                  \
    const int row = cidx / CH_PER_ROW, col = cidx - row * CH_PER_ROW;                               \
    *reinterpret_cast<u32x4*>(&ktile[BUF][row * ROWB + col * 16]) = to_bf16x8(ST[i]);               \
  }

  // The first K tile of the segment is sent for before the query rows, so that both arrive in one round trip.
  CODECOMP_GLOAD(kstart, stage)

  // ---- this wave's query rows as MFMA fragments
  u32x4 qf[2][KS];
  {
    const uint16_t* qb = a.q + (int64_t)layer * a.q_sl + (int64_t)seq * a.q_ss;
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
      const int row = split_row0 + rb_of[sl] * 32 + l32;
      const bool ok = row < a.R && (sl == 0 || halves1 != 0);
      const int g = ok ? row / a.W : 0;
      const int t = ok ? row - g * a.W : 0;
      const uint16_t* p = qb + (int64_t)(head * a.G + g) * a.q_sh + (int64_t)t * a.q_st + hf * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        u32x4 v = *reinterpret_cast<const u32x4*>(p + ks * 16);     // row 0 of the group when !ok: in bounds
        if (!ok) v = u32x4{0, 0, 0, 0};
        qf[sl][ks] = v;
      }
    }
  }

  const float c = a.c;

  // pass 1 state: running (max, sum) of this lane's row over the keys this lane sees, per slot
  float m_run0 = NEG_BIG, m_run1 = NEG_BIG;
  float l_run0 = 0.f, l_run1 = 0.f;
  // pass 2 state: -lse of the 2 x 16 rows this lane holds in the S tiles
  float nl[2][16];
  if constexpr (PASS == 2) {
    const float* lse = a.lse + ((int64_t)lz * a.n_seqs + seq) * a.lrows;
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = split_row0 + rb_of[sl] * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
        const float x = lse[row];                 // row < lrows: in bounds; padding rows get no weight
        nl[sl][v] = row < a.R ? -x : -INFINITY;
      }
  }

  // Sum the per-wave column partials of one finished tile and store the attention mass (pass 2).
  // The last wave does it: where the waves are unevenly loaded it is one of the light ones.
  auto reduce_cols = [&](int tile) __attribute__((always_inline)) {
    if constexpr (PASS == 2) {
      if (tile >= 0 && wave == NW - 1) {
        float s = 0.f;
        if constexpr (!GMAX) {
#pragma unroll
          for (int w = 0; w < NW * 2; ++w) s += colbuf[tile & 3][w][lane];
          s *= a.inv_g;
        } else {
          // row blocks in order: the blocks of one query head are consecutive; a block's mass is the sum of its
          // owners' partials (both half waves of each); the head masses are compared, not added
          float cur = 0.f;
          for (int rb = 0; rb < a.nb; ++rb) {
            for (int h = 0; h < 2; ++h) {
              const int holder = a.rb_holder[rb][h];      // wave * 2 + slot
              if (holder != 255) cur += colbuf[tile & 3][holder * 2][lane] + colbuf[tile & 3][holder * 2 + 1][lane];
            }
            if ((rb + 1) % a.blocks_per_head == 0 || rb == a.nb - 1) { s = fmaxf(s, cur); cur = 0.f; }
          }
        }
        const int key = kstart + tile * kTileKeys + lane;
        if (key < kend) a.uraw[((int64_t)split * a.LH + lz) * a.T + tok0 + key] = s;
      }
    }
  };

  // ------------------------------------------------------------------------------------------
  // Software pipeline.  A tile (64 keys) is two sub-tiles (32 keys) a, b; each sub-tile is one
  // "phase" of KS MFMAs per active slot.  While the matrix core forms the logits of one sub-tile,
  // the VALU does the softmax arithmetic on the previous one, cut into 2*KS slices ("gaps", one
  // after every MFMA position); a scheduling pattern after every phase keeps the compiler from
  // regrouping them.  The K fragments of the next four k-steps are prefetched from LDS into a
  // 4-entry register ring, the next tile travels global -> registers -> LDS one tile ahead, and
  // the only workgroup barrier of a tile sits in the middle of phase b, where the first fragment
  // of the next tile is needed.  Global loads stay in flight across that barrier (it waits for
  // LDS traffic only).  Every wave passes the same barriers whatever it owns.
  // ------------------------------------------------------------------------------------------
  constexpr int MS = 2 * KS;                    // gaps per phase
  constexpr int RING = 4;                       // K fragments prefetched ahead
  constexpr int BAR_KS = KS - RING;             // k-step of phase b before which the barrier sits
  static_assert(KS >= RING, "fragment ring");

  f32x16 accA0, accA1, accB0, accB1;
  u32x4 ring[RING];

  auto kfrag_ptr = [&](int buf, int kh, int ks) __attribute__((always_inline)) {
    return reinterpret_cast<const u32x4*>(&ktile[buf][(kh * 32 + l32) * ROWB + hf * 16 + ks * 32]);
  };
  auto lds_barrier = [&]() __attribute__((always_inline)) {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  };
  // pass 1 only: logits of keys past the end of the segment must not enter any row sum.  A lane's 16
  // logits of a sub-tile are keys in ascending order, so the valid ones are a prefix of length nvalid.
  auto mask_tail = [&](f32x16& x, int kh) __attribute__((always_inline)) {
    if constexpr (PASS == 1) {
      // keys of this lane in sub-tile kh: kh*32 + 8*(v/4) + 4*hf + v%4; full groups of 8 keys below `rem`, then a part
      const int left = rem - kh * 32 - 4 * hf;                       // keys at or after this lane's first one
      const int part = left - 8 * (left >> 3);                       // 0..7
      const int nvalid = left <= 0 ? 0 : 4 * (left >> 3) + (part < 4 ? part : 4);
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (v >= nvalid) x[v] = -INFINITY;
    }
  };

  // Softmax state of the sub-tile being consumed.
  float s0, s1, mc0 = 0.f, mc1 = 0.f, al0, al1, mn0, mn1, t0, t1;
  // Pass 1 comes in two flavours.  FAST keeps one fixed reference per lane and slot (the largest
  // logit of the first sub-tile the slot computes) instead of a running maximum: no max3 chain, no
  // rescaling.  A later logit more than ~88 nats above that reference would overflow fp32; the
  // workgroup then notices the non-finite sum and redoes its chunk with the running maximum (SAFE).
  // SAFE spends the first quarter of the gaps on the row maxima, the rest on the exponentials.
  constexpr int MAXSTEPS_SAFE = MS / 4;

  // One gap's share of the softmax work on a finished sub-tile: p0 (slot 0) and, if BOTH, p1 (slot 1).
  auto soft_step = [&](const f32x16& p0, const f32x16& p1, int m, auto both, auto fast) __attribute__((always_inline)) {
    constexpr bool BOTH = decltype(both)::value;
    constexpr bool TRACK_MAX = PASS == 1 && !decltype(fast)::value;
    constexpr int NE = BOTH ? 32 : 16;          // logits per lane to consume in this phase
    constexpr int MAXSTEPS = TRACK_MAX ? MAXSTEPS_SAFE : 0;
    constexpr int EXPSTEPS = MS - MAXSTEPS;
    constexpr int EBASE = NE / EXPSTEPS, EEXTRA = NE % EXPSTEPS;
    if (m == 0) { s0 = 0.f; s1 = 0.f; }
    if constexpr (TRACK_MAX) {
      if (m < MAXSTEPS) {
        constexpr int PER = 16 / MAXSTEPS;      // logits of each slot folded into the maxima per gap
        if (m == 0) { t0 = m_run0; t1 = m_run1; }
#pragma unroll
        for (int e = 0; e < PER; e += 2) {
          t0 = fmaxf(fmaxf(t0, p0[m * PER + e]), p0[m * PER + e + 1]);
          if constexpr (BOTH) t1 = fmaxf(fmaxf(t1, p1[m * PER + e]), p1[m * PER + e + 1]);
        }
        if (m == MAXSTEPS - 1) {
          mn0 = t0;
          al0 = __builtin_amdgcn_exp2f((m_run0 - mn0) * c);
          mc0 = mn0 * c;
          if constexpr (BOTH) {
            mn1 = t1;
            al1 = __builtin_amdgcn_exp2f((m_run1 - mn1) * c);
            mc1 = mn1 * c;
          }
        }
        return;
      }
    }
    const int x = m - MAXSTEPS;
    const int e0 = x * EBASE + (x < EEXTRA ? x : EEXTRA);
    const int cnt = EBASE + (x < EEXTRA ? 1 : 0);
#pragma unroll
    for (int e = e0; e < e0 + cnt; ++e) {
      const int v = BOTH ? e >> 1 : e;
      const bool second = BOTH && (e & 1);
      if constexpr (PASS == 1) {
        if (second) s1 += __builtin_amdgcn_exp2f(__builtin_fmaf(p1[v], c, -mc1));
        else s0 += __builtin_amdgcn_exp2f(__builtin_fmaf(p0[v], c, -mc0));
      } else {
        if (second) s1 += __builtin_amdgcn_exp2f(__builtin_fmaf(p1[v], c, nl[1][v]));
        else s0 += __builtin_amdgcn_exp2f(__builtin_fmaf(p0[v], c, nl[0][v]));
      }
    }
  };
  auto soft_end = [&](int ptile, int pkh, auto both, auto fast) __attribute__((always_inline)) {
    constexpr bool BOTH = decltype(both)::value;
    if constexpr (PASS == 1) {
      if constexpr (decltype(fast)::value) {
        l_run0 += s0;
        if constexpr (BOTH) l_run1 += s1;
      } else {
        l_run0 = l_run0 * al0 + s0; m_run0 = mn0;
        if constexpr (BOTH) { l_run1 = l_run1 * al1 + s1; m_run1 = mn1; }
      }
    } else if constexpr (!GMAX) {
      colbuf[ptile & 3][wave * 2 + hf][pkh * 32 + l32] = BOTH ? s0 + s1 : s0;
    } else {
      colbuf[ptile & 3][wave * 4 + hf][pkh * 32 + l32] = s0;
      colbuf[ptile & 3][wave * 4 + 2 + hf][pkh * 32 + l32] = BOTH ? s1 : 0.f;
    }
  };

  // Scheduling pattern of one phase for the machine scheduler: per gap, the MFMA that opens it (slot 0
  // in even gaps, slot 1 in odd gaps when MF1), the ring refill, and the gap's share of softmax work
  // (SAFE pass 1: maxima in the first quarter of the phase, exponentials after).
  auto sched_phase = [&](auto mf1, auto both, auto fast) __attribute__((always_inline)) {
    constexpr bool MF1 = decltype(mf1)::value, BOTH = decltype(both)::value;
    constexpr bool TRACK_MAX = PASS == 1 && !decltype(fast)::value;
    constexpr int NE = BOTH ? 32 : 16;
    constexpr int MAXSTEPS = TRACK_MAX ? MAXSTEPS_SAFE : 0;
    constexpr int EXPSTEPS = MS - MAXSTEPS;
    constexpr int SG_MAX = TRACK_MAX ? (BOTH ? 2 : 1) * (8 / (MAXSTEPS > 0 ? MAXSTEPS : 1)) + 2 : 1;   // max3 ops (+ scalars) per gap
    constexpr int SG_E = (NE + EXPSTEPS - 1) / EXPSTEPS;                                             // logits per exponential gap
#pragma unroll
    for (int m = 0; m < MS; ++m) {
      if (!(m & 1) || MF1) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
      if (m & 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);             // the ring refill (LDS read)
      if (TRACK_MAX && m < MAXSTEPS) {
        __builtin_amdgcn_sched_group_barrier(0x002, SG_MAX, 0);                 // max3 chain (+ scalars)
      } else {
        __builtin_amdgcn_sched_group_barrier(0x002, SG_E, 0);                   // fma
        __builtin_amdgcn_sched_group_barrier(0x400, SG_E, 0);                   // exp2
        __builtin_amdgcn_sched_group_barrier(0x002, SG_E, 0);                   // add
      }
    }
  };

  // One tile = phase a + phase b.  A1 / B1: slot 1 computes sub-tile a / b.  MASKED (last, partial
  // tile only) clears the logits of keys past the end of the segment before they are consumed.
  // STG: which staging registers feed LDS in this tile: 0 = `stage`, next load two tiles ahead;
  // 1 / 2 = `stage` / `stage2`, next load three tiles ahead (DEEP); 3 = none (last tile of a segment).
  auto tile_body = [&](int t, auto masked, auto fast, auto a1, auto b1, auto stg) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked)::value;
    constexpr int STG = decltype(stg)::value;
    constexpr bool FAST = PASS == 1 && decltype(fast)::value;
    constexpr bool A1 = decltype(a1)::value, B1 = decltype(b1)::value;
    const int buf = t & 1;
    const f32x16 zero = {0};
    // ---------------- phase a: logits of sub-tile a -> accA; softmax of accB (tile t-1, sub-tile b)
    // tile t+1 waits in staging registers: park it in the other LDS buffer (its last readers passed
    // the previous barrier), then send the loads of a later tile on their way into the same registers
    if constexpr (STG == 0 || STG == 1) { CODECOMP_SSTORE(buf ^ 1, stage) }
    if constexpr (STG == 2) { CODECOMP_SSTORE(buf ^ 1, stage2) }
    if constexpr (STG == 0) CODECOMP_GLOAD(kstart + (t + 2) * kTileKeys, stage)
    if constexpr (STG == 1) CODECOMP_GLOAD(kstart + (t + 3) * kTileKeys, stage)
    if constexpr (STG == 2) CODECOMP_GLOAD(kstart + (t + 3) * kTileKeys, stage2)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      accA0 = mma_step<PASS>(qf[0][ks], ring[ks % RING], ks == 0 ? zero : accA0);
      soft_step(accB0, accB1, 2 * ks, b1, fast);
      if constexpr (A1) accA1 = mma_step<PASS>(qf[1][ks], ring[ks % RING], ks == 0 ? zero : accA1);
      ring[ks % RING] = ks + RING < KS ? *kfrag_ptr(buf, 0, ks + RING) : *kfrag_ptr(buf, 1, ks + RING - KS);
      soft_step(accB0, accB1, 2 * ks + 1, b1, fast);
    }
    soft_end(t - 1, 1, b1, fast);
    sched_phase(a1, b1, fast);
    // pass 2 of an eight-wave workgroup: each phase a scheduling region of its own (2 % off that pass; the four-wave
    // workgroups and pass 1 get slower with it)
    if constexpr (PASS == 2 && NW == 8) __builtin_amdgcn_sched_barrier(0);
    if constexpr (MASKED) { mask_tail(accA0, 0); if constexpr (A1) mask_tail(accA1, 0); }
    if constexpr (FAST) {
      if (t == 0) {                             // the chunk's fixed references: largest logit this lane sees first
        float r0 = NEG_BIG, r1 = NEG_BIG;
#pragma unroll
        for (int v = 0; v < 16; ++v) { r0 = fmaxf(r0, accA0[v]); if constexpr (A1) r1 = fmaxf(r1, accA1[v]); }
        m_run0 = r0; mc0 = r0 * c;
        if constexpr (A1) { m_run1 = r1; mc1 = r1 * c; }
      }
    }
    // ---------------- phase b: logits of sub-tile b -> accB; softmax of accA (tile t, sub-tile a)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks == BAR_KS) lds_barrier();          // tile t+1 is now complete in LDS buffer buf^1
      accB0 = mma_step<PASS>(qf[0][ks], ring[ks % RING], ks == 0 ? zero : accB0);
      soft_step(accA0, accA1, 2 * ks, a1, fast);
      if constexpr (B1) accB1 = mma_step<PASS>(qf[1][ks], ring[ks % RING], ks == 0 ? zero : accB1);
      ring[ks % RING] = ks + RING < KS ? *kfrag_ptr(buf, 1, ks + RING) : *kfrag_ptr(buf ^ 1, 0, ks + RING - KS);
      soft_step(accA0, accA1, 2 * ks + 1, a1, fast);
    }
    soft_end(t, 0, a1, fast);
    sched_phase(b1, a1, fast);
    if constexpr (PASS == 2 && NW == 8) __builtin_amdgcn_sched_barrier(0);
    if constexpr (MASKED) { mask_tail(accB0, 1); if constexpr (B1) mask_tail(accB1, 1); }
    if constexpr (FAST && !A1 && B1) {
      if (t == 0) {                             // slot 1 sees its first logits here (a sub-tile b may hold no valid key at all)
        float r1 = NEG_BIG;
#pragma unroll
        for (int v = 0; v < 16; ++v) r1 = fmaxf(r1, accB1[v]);
        m_run1 = r1; mc1 = r1 * c;
      }
    }
  };

  // The whole chunk: prologue (tile 0 into LDS buffer 0, tile 1 into the staging registers, first
  // fragments), the tiles, and the softmax of the very last sub-tile.
  auto run_chunk = [&](auto fast, auto a1, auto b1, auto reload) __attribute__((always_inline)) {
    // the first phase consumes a sub-tile that does not exist: -inf logits add nothing to any sum
#pragma unroll
    for (int v = 0; v < 16; ++v) { accB0[v] = -INFINITY; accB1[v] = -INFINITY; }
    m_run0 = NEG_BIG; m_run1 = NEG_BIG; l_run0 = 0.f; l_run1 = 0.f; mc0 = 0.f; mc1 = 0.f;
    if constexpr (decltype(reload)::value) CODECOMP_GLOAD(kstart, stage)      // a second run: tile 0 again
    CODECOMP_SSTORE(0, stage)
    CODECOMP_GLOAD(kstart + kTileKeys, stage)
    if constexpr (DEEP) CODECOMP_GLOAD(kstart + 2 * kTileKeys, stage2)
    lds_barrier();
#pragma unroll
    for (int r = 0; r < RING; ++r) ring[r] = *kfrag_ptr(0, 0, r);

    using stg = std::integral_constant<int, 0>;
    using stg_even = std::integral_constant<int, 1>;
    using stg_odd = std::integral_constant<int, 2>;
    using stg_none = std::integral_constant<int, 3>;
    const int nplain = rem != 0 ? ntiles - 1 : ntiles;
    if constexpr (DEEP) {
      int t = 0;
      for (; t + 1 < nplain; t += 2) {           // even tiles are fed from `stage`, odd ones from `stage2`
        reduce_cols(t - 2);
        tile_body(t, std::false_type{}, fast, a1, b1, stg_even{});
        reduce_cols(t - 1);
        tile_body(t + 1, std::false_type{}, fast, a1, b1, stg_odd{});
      }
      if (t < nplain) {
        reduce_cols(t - 2);
        tile_body(t, std::false_type{}, fast, a1, b1, stg_even{});
      }
    } else {
      for (int t = 0; t < nplain; ++t) {
        reduce_cols(t - 2);
        tile_body(t, std::false_type{}, fast, a1, b1, stg{});
      }
    }
    if (rem != 0) {
      reduce_cols(ntiles - 3);
      tile_body(ntiles - 1, std::true_type{}, fast, a1, b1, stg_none{});
    }
#pragma unroll
    for (int m = 0; m < MS; ++m) soft_step(accB0, accB1, m, b1, fast);
    soft_end(ntiles - 1, 1, b1, fast);
  };

  // The wave's flavour of the pipeline.  All flavours contain the same barriers in the same order.
  auto run_wave = [&](auto a1, auto b1) __attribute__((always_inline)) {
    if constexpr (PASS == 1) {
      run_chunk(std::true_type{}, a1, b1, std::false_type{});
      // a row that saw no key at all keeps the reference -1e30: its empty sum is 0, not a failure
      const bool bad = !(l_run0 <= 3.0e38f) || !(l_run1 <= 3.0e38f);     // inf or NaN: a logit outran the reference
      if (__syncthreads_or(bad)) run_chunk(std::false_type{}, a1, b1, std::true_type{});
    } else {
      run_chunk(std::false_type{}, a1, b1, std::false_type{});
    }
  };
  switch (halves1) {
    case 0: run_wave(std::false_type{}, std::false_type{}); break;
    case 1: run_wave(std::true_type{}, std::false_type{}); break;
    case 2: run_wave(std::false_type{}, std::true_type{}); break;
    default: run_wave(std::true_type{}, std::true_type{}); break;
  }

  if constexpr (PASS == 2) {
    lds_barrier();
    reduce_cols(ntiles - 2);
    reduce_cols(ntiles - 1);
  } else {
    // merge the two half-wave views of each row, then one (max*c, sum) pair per slot row and segment
    float* st = a.stats + ((int64_t)((team + lz * a.n_seqs + seq) * a.row_splits + split) * a.srows) * 2;
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
      const float m_r = sl == 0 ? m_run0 : m_run1, l_r = sl == 0 ? l_run0 : l_run1;
      const float m_o = __shfl_xor(m_r, 32);
      const float l_o = __shfl_xor(l_r, 32);
      const float M = fmaxf(m_r, m_o);
      const float L = l_r * __builtin_amdgcn_exp2f((m_r - M) * c) + l_o * __builtin_amdgcn_exp2f((m_o - M) * c);
      const int srow = (wave * 2 + sl) * 32 + l32;
      if (lane < 32 && (sl == 0 || halves1 != 0)) {
        st[srow * 2 + 0] = M * c;
        st[srow * 2 + 1] = L;
      }
    }
  }
  // the next segment reuses the LDS buffers: every wave must be done reading them
  lds_barrier();
  x += ntiles;
  }   // segments
#undef CODECOMP_GLOAD
#undef CODECOMP_SSTORE
}

// Enqueues the row merge between the two passes (defined in score.hip).
int launch_row_merge(const Plan& pl, const ScoreArgs& a, hipStream_t stream);

// Workgroups that run at once on the current device: compute units x resident workgroups per unit.  The answer
// depends on the kernel and on the device, so every kernel keeps one cached value per device ordinal (the
// occupancy query is a host-side calculation, but not a free one); 0 = not asked yet.  Two threads that ask at the
// same time both compute the same number.  This cache is the only thing the library remembers between calls.
constexpr int kMaxDevices = 64;
template <class Kernel>
int resident_workgroups(Kernel kernel, int threads, std::atomic<int>* cache) {
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (dev >= 0 && dev < kMaxDevices) {
    const int known = cache[dev].load(std::memory_order_relaxed);
    if (known > 0) return known;
  }
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess) return 0;
  if (dev >= 0 && dev < kMaxDevices) cache[dev].store(cus * per_cu, std::memory_order_relaxed);
  return cus * per_cu;
}

// Teams of one launch "wave": as many workgroups as the device holds at once (row_splits of them per team), each
// team with an equal share of the tiles (at least kMinTilesPerWorkgroup, so that small problems are not all
// prologue), unless the caller fixed the number of workgroups (codecomp_params.score_workgroups).
inline int score_teams(const Plan& pl, int resident) {
  int g = (resident > 0 ? resident : 256) / pl.row_splits;
  if (pl.grid_override > 0) g = pl.grid_override / pl.row_splits;
  else g = g < pl.real_tiles / kMinTilesPerWorkgroup ? g : pl.real_tiles / kMinTilesPerWorkgroup;
  if (g > pl.real_tiles) g = pl.real_tiles;
  if (g > kMaxScoreGrid / pl.row_splits) g = kMaxScoreGrid / pl.row_splits;
  return g < 1 ? 1 : g;
}

template <int D, int NW, bool K8>
int launch_passes(const Plan& pl, ScoreArgs a, hipStream_t stream, unsigned stages) {
  static std::atomic<int> cache1[kMaxDevices], cache2[kMaxDevices], cache2m[kMaxDevices];   // zero-initialised
  const dim3 block(NW * 64);
  a.stat_teams = score_teams(pl, resident_workgroups(score_pass_kernel<D, NW, 1, false, K8>, NW * 64, cache1));
  const bool any_tile = pl.real_tiles > 0;      // false: prefix-only softmax with no prefix anywhere
  if ((stages & CODECOMP_STAGE_ROW_STATS) && any_tile) {
    score_pass_kernel<D, NW, 1, false, K8><<<dim3(a.stat_teams * pl.row_splits), block, 0, stream>>>(a);
    if (hipError_t e = hipGetLastError()) return (int)e;
  }
  if (stages & CODECOMP_STAGE_ROW_MERGE) {
    if (int rc = launch_row_merge(pl, a, stream)) return rc;
  }
  if ((stages & CODECOMP_STAGE_MASS) && any_tile) {
    if (pl.variant & CODECOMP_VARIANT_GROUP_MAX) {
      const int g = score_teams(pl, resident_workgroups(score_pass_kernel<D, NW, 2, true, K8>, NW * 64, cache2m));
      score_pass_kernel<D, NW, 2, true, K8><<<dim3(g * pl.row_splits), block, 0, stream>>>(a);
    } else {
      const int g = score_teams(pl, resident_workgroups(score_pass_kernel<D, NW, 2, false, K8>, NW * 64, cache2));
      score_pass_kernel<D, NW, 2, false, K8><<<dim3(g * pl.row_splits), block, 0, stream>>>(a);
    }
    if (hipError_t e = hipGetLastError()) return (int)e;
  }
  return 0;
}

// The passes of one (head_dim, key type) pair; each pair is instantiated in a translation unit of its own
// (score_pass_*.hip) so that they compile side by side.
template <int D, bool K8>
int dispatch_waves(const Plan& pl, const ScoreArgs& a, hipStream_t s, unsigned st) {
  switch (pl.waves) {
    case 1: return launch_passes<D, 1, K8>(pl, a, s, st);
    case 2: return launch_passes<D, 2, K8>(pl, a, s, st);
    case 3: return launch_passes<D, 3, K8>(pl, a, s, st);
    case 4: return launch_passes<D, 4, K8>(pl, a, s, st);
    case 8: return launch_passes<D, 8, K8>(pl, a, s, st);
  }
  return CODECOMP_EINVAL_SHAPE;
}

}  // namespace codecomp
