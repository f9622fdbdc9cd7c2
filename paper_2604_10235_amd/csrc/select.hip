// Select step: per (layer, KV head, request) keep the last W tokens and the B - W best tokens
// of the prefix [0, N - W); equal scores go to the lower index; indices come out ascending
// (section "Attention-based KV Cache Compression": the best-scored context tokens are kept until the budget is used up).
//
// An MSB-first radix select over order-preserving integer images of the float scores (digits of 11, 11
// and 10 bits, LDS histograms) finds the score of the last admitted token and how many tokens tied at
// that score are admitted; one ordered pass (prefix sums of "sure" and "tied" flags) then writes the
// indices already sorted.  No float is ever added, nothing depends on the order in which workgroups run:
// the result is the same bits on every call.
//
// Requests of at most 65536 candidates in a batch with enough problems to occupy the device: one workgroup
// of 1024 threads (256 threads when all requests are short and there are a thousand problems or more) owns one
// (layer, head, request) problem; the candidates are read from memory once, all loads in flight together, and
// stay in registers through the three digit passes and the ordered pass.
// A batch with a longer request, or with few problems and long requests: every request is cut into parts
// of 8192 candidates and four kernels run one 256-thread workgroup per part (the third one per request),
// so that a problem is spread over as many compute units as it has parts and a ragged batch is not paced
// by its longest request:
//   counts  every part counts the first digit of its candidates (2048 bins) and stores the counts;
//   near    every part adds up the counts of its request, finds the bin that holds the cut, and appends its
//           candidates of that bin (keys only, in token order) to the request's list, at the place the
//           counts of the earlier parts give it; it also stores how many of its candidates lie above that bin;
//   resolve one workgroup per request finishes the radix select on the list (two more digits; the list is short
//           unless the scores crowd into one bin);
//   emit    every part counts what the earlier parts contribute and writes its own admitted indices at their
//           final places.
//
// Two selection rules share these pieces:
//   additive   : one selection on c = pooled attention + lambda * prior (the score kernel's output);
//   two-stage  : the paper's literal order - structure first, attention fills the rest
//                (sections "Span-Level Structural Protection" and "Attention-based KV Cache
//                Compression"): stage 1 keeps up to B_span = min(Bp, max(B_min, floor(rho * Bp)))
//                prefix tokens with prior > 0, largest prior first (ties: first in sequence, which for a
//                binary prior is the paper's rule for an overfull protected set: its first tokens),
//                Bp = B - W; stage 2 fills the remaining Bp - |P| slots with the best pooled-attention
//                tokens not in P.
#include "plan.h"

namespace codecomp {

// Monotone map float -> uint32 (larger float <=> larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t order_key(float x) {
  x = x + 0.0f;   // -0 -> +0
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kSelTileItems = 4;    // consecutive candidates per thread inside one ordered tile
constexpr int kHistStride = 2049;   // odd stride: equal bins of different copies sit in different banks

// The one-workgroup kernels come in two sizes.  NT = 1024 threads, up to 64 candidates per thread, 8 private copies of
// the first-digit histogram (130 KB of LDS: one workgroup per compute unit) for long requests; NT = 256 threads, up to
// 16 candidates per thread, 2 copies (21 KB: seven workgroups per compute unit) for batches of many short requests,
// where what counts is how many problems a compute unit works on at once (measured on 7168 problems of 14 .. 2185
// candidates: 270 us with the large workgroups, 132 / 105 / 108 us with the small ones and 4 / 2 / 1 copies; from
// 8192 candidates per problem on the large ones are faster).
template <int NT> struct SelectSize {
  static constexpr int kMaxItems = NT == kSelectThreads ? kSelectMaxCandidates / kSelectThreads : kSelectSmallMaxItems;
  static constexpr int kCopies = NT == kSelectThreads ? 8 : 2;     // picked by lane % kCopies
};

template <int NT> struct SelectShared {
  unsigned int hist[SelectSize<NT>::kCopies * kHistStride];
  unsigned int prefix, need;
  int wave_sure[NT / 64], wave_tie[NT / 64];
  int tile_sure, tile_tie;
  // class (0 out, 1 tied at the cut, 2 in) of every register-resident candidate, one byte each, indexed by
  // candidate: written in the load layout, read back as runs of consecutive candidates per thread
  unsigned int cls_words[NT * SelectSize<NT>::kMaxItems / 4];
};

// One candidate into the digit histogram.  CROWDED (the first digit: every candidate takes part and the scores
// crowd into a few dozen bins): LDS atomics of one instruction that hit the same address are served one after
// the other, so each lane adds to one of several private copies (lane % copies) and fewer lanes can collide;
// the copies are summed when the bin is picked.  Ballot-based aggregation was tried first: its serial
// scalar/vector control flow cost about 1000 cycles per candidate slot and workgroup.  Later digits: only the
// few candidates that share the prefix take part, one copy.
template <bool CROWDED, int NT>
__device__ __forceinline__ void hist_add(SelectShared<NT>& sh, bool match, uint32_t bin) {
  if (match) atomicAdd(&sh.hist[(CROWDED ? (threadIdx.x & (SelectSize<NT>::kCopies - 1)) * kHistStride : 0) + bin], 1u);
}

__device__ __forceinline__ int pass_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int pass_bins(int pass) { return pass == 2 ? 1024 : 2048; }
__device__ __forceinline__ uint32_t pass_himask(int pass) {
  return pass == 0 ? 0u : (0xFFFFFFFFu << (pass == 1 ? 21 : 10));
}

template <int NT>
__device__ __forceinline__ void hist_clear(SelectShared<NT>& sh, int nbins, int copies) {
  for (int b = threadIdx.x; b < (copies - 1) * kHistStride + nbins; b += NT) sh.hist[b] = 0;
  __syncthreads();
}

// After a digit pass: the bin holding the `remaining`-th largest candidate; fixes that digit in `prefix`
// and reduces `remaining` to the rank inside the bin.  All threads call it.  No step waits for an LDS
// read that depends on the previous one: the copies are summed by all threads, wave 0 finds the lane whose
// group of bins holds the rank (suffix sums over lanes), then the bin inside that group the same way.
template <int NT>
__device__ __forceinline__ void hist_pick(SelectShared<NT>& sh, int nbins, int copies, int shift, uint32_t& prefix,
                                          uint32_t& remaining) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (copies > 1) {                    // totals of the private copies into copy 0 (a thread touches only its own bins)
    for (int b = threadIdx.x; b < nbins; b += NT) {
      unsigned int c = 0;
      for (int k = 0; k < copies; ++k) c += sh.hist[k * kHistStride + b];
      sh.hist[b] = c;
    }
    __syncthreads();
  }
  if (wave == 0) {
    const int per = nbins / 64;        // lane owns bins [lane*per, lane*per+per), per <= 32
    unsigned int mine = 0;
    for (int i = 0; i < per; ++i) mine += sh.hist[lane * per + i];
    unsigned int run = mine;           // inclusive suffix sum over lanes
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const unsigned int o = __shfl_down(run, off);
      if (lane + off < 64) run += o;
    }
    const unsigned int above = run - mine;   // count in bins owned by higher lanes
    const unsigned long long hit = __ballot(above < remaining && remaining <= above + mine);   // exactly one lane
    const int owner = __ffsll(hit) - 1;
    const unsigned int above_owner = __builtin_amdgcn_readlane(above, owner);
    // the bins of the owner, one per lane
    const unsigned int c = lane < per ? sh.hist[owner * per + lane] : 0u;
    unsigned int suf = c;              // inclusive suffix sum over the owner's bins
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
      const unsigned int o = __shfl_down(suf, off);
      if (lane + off < 64) suf += o;
    }
    const unsigned int higher = above_owner + suf - c;      // candidates in bins above this one
    if (lane < per && higher < remaining && remaining <= higher + c) {   // exactly one lane
      sh.prefix = prefix | ((uint32_t)(owner * per + lane) << shift);
      sh.need = remaining - higher;    // rank inside the chosen bin
    }
  }
  __syncthreads();
  prefix = sh.prefix;
  remaining = sh.need;
}

// Exclusive prefix counts over the workgroup for one ordered tile.  In: this thread's counts.  Out: counts
// in lower threads of the tile, and the tile totals.  All threads call it.
template <int NT>
__device__ __forceinline__ void tile_scan(SelectShared<NT>& sh, int nsure, int ntie, int& before_sure, int& before_tie,
                                          int& tot_sure, int& tot_tie) {
  constexpr int NWV = NT / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int ss = nsure, st = ntie;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int os = __shfl_up(ss, off), ot = __shfl_up(st, off);
    if (lane >= off) { ss += os; st += ot; }
  }
  if (lane == 63) { sh.wave_sure[wave] = ss; sh.wave_tie[wave] = st; }
  __syncthreads();
  if (wave == 0) {
    int ws = lane < NWV ? sh.wave_sure[lane] : 0, wt = lane < NWV ? sh.wave_tie[lane] : 0;
    int is = ws, it = wt;
#pragma unroll
    for (int off = 1; off < NWV; off <<= 1) {
      const int os = __shfl_up(is, off), ot = __shfl_up(it, off);
      if (lane >= off) { is += os; it += ot; }
    }
    if (lane < NWV) { sh.wave_sure[lane] = is - ws; sh.wave_tie[lane] = it - wt; }
    if (lane == NWV - 1) { sh.tile_sure = is; sh.tile_tie = it; }
  }
  __syncthreads();
  before_sure = sh.wave_sure[wave] + ss - nsure;
  before_tie = sh.wave_tie[wave] + st - ntie;
  tot_sure = sh.tile_sure;
  tot_tie = sh.tile_tie;
  __syncthreads();                      // wave_* / tile_* are rewritten by the next tile
}

// The selection proper.  A "candidate source" gives, for index j in [0, npre):
//   key(j)      order-preserving integer image of its score,
//   eligible(j) whether it competes in the radix select,
//   forced(j)   whether it is admitted regardless (stage 2: members of the protected set).
// The candidates are loaded once into registers, ITEMS per thread (npre <= NT * ITEMS).
// emit(j, admitted, pos) is called for every j, pos = number of admitted candidates before j.
template <int NT, int ITEMS, class Source, class Emit>
__device__ __forceinline__ void select_wg(SelectShared<NT>& sh, Source src, Emit emit, int npre, int need) {
  const int tid = threadIdx.x;
  constexpr int kSelTile = NT * kSelTileItems;
  static_assert(ITEMS > 0 && ITEMS % kSelTileItems == 0 && ITEMS <= SelectSize<NT>::kMaxItems, "register-resident candidates");
  uint32_t keys[ITEMS];
  unsigned long long elig = 0, forc = 0;       // one bit per register slot
  // slot s of this thread holds candidate j = (s / 4) * kSelTile + tid * 4 + (s % 4): tiles in order, 4 consecutive
  if (npre > 0) {                              // the same for every thread
    // unconditional loads (index clamped into the row) so that all of them are in flight together
#pragma unroll
    for (int s = 0; s < ITEMS; ++s) {
      const int j = (s / kSelTileItems) * kSelTile + tid * kSelTileItems + (s % kSelTileItems);
      const int jc = j < npre ? j : npre - 1;
      const uint32_t key = src.key(jc);
      const bool el = src.eligible(jc), fo = src.forced(jc);
      keys[s] = j < npre ? key : 0u;
      if (j < npre && el) elig |= 1ull << s;
      if (j < npre && fo) forc |= 1ull << s;
    }
  } else {
#pragma unroll
    for (int s = 0; s < ITEMS; ++s) keys[s] = 0u;
  }

  uint32_t tau = 0xFFFFFFFFu;
  int ties = 0;                               // need == 0: only forced candidates are admitted
  if (need > 0) {
    uint32_t prefix = 0, remaining = (uint32_t)need;
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass_shift(pass), nbins = pass_bins(pass);
      const uint32_t himask = pass_himask(pass);
      const int copies = pass == 0 ? SelectSize<NT>::kCopies : 1;
      hist_clear(sh, nbins, copies);
#pragma unroll
      for (int s = 0; s < ITEMS; ++s) {
        const bool match = ((elig >> s) & 1ull) && (keys[s] & himask) == prefix;
        if (pass == 0) hist_add<true, NT>(sh, match, (keys[s] >> shift) & (uint32_t)(nbins - 1));
        else hist_add<false, NT>(sh, match, (keys[s] >> shift) & (uint32_t)(nbins - 1));
      }
      hist_pick(sh, nbins, copies, shift, prefix, remaining);
    }
    tau = prefix;
    ties = (int)remaining;
  }

  // ---- ordered pass.  The classes (0 out, 1 tied at the cut, 2 in) go through LDS so that every thread ends up
  // with ITEMS consecutive candidates: one workgroup prefix sum, and each thread writes its admitted indices to
  // consecutive places.
  constexpr int T4 = ITEMS / kSelTileItems;
#pragma unroll
  for (int t = 0; t < T4; ++t) {
    unsigned int word = 0;
#pragma unroll
    for (int e = 0; e < kSelTileItems; ++e) {
      const int s = t * kSelTileItems + e;
      const bool el = (elig >> s) & 1ull, fo = (forc >> s) & 1ull;
      const unsigned int c = fo ? 2u : (el ? (keys[s] > tau ? 2u : (keys[s] == tau ? 1u : 0u)) : 0u);
      word |= c << (8 * e);
    }
    sh.cls_words[t * NT + tid] = word;                   // candidates 4 * (t * NT + tid) .. + 3
  }
  __syncthreads();
  unsigned int mine[T4];
  int nsure = 0, ntie = 0;
#pragma unroll
  for (int t = 0; t < T4; ++t) {
    mine[t] = sh.cls_words[tid * T4 + t];                // candidates tid * ITEMS + 4 t .. + 3
#pragma unroll
    for (int e = 0; e < kSelTileItems; ++e) {
      const unsigned int c = (mine[t] >> (8 * e)) & 255u;
      nsure += c == 2u; ntie += c == 1u;
    }
  }
  int ps, pt, ts, tt;
  tile_scan(sh, nsure, ntie, ps, pt, ts, tt);
#pragma unroll
  for (int t = 0; t < T4; ++t) {
#pragma unroll
    for (int e = 0; e < kSelTileItems; ++e) {
      const int j = tid * ITEMS + t * kSelTileItems + e;
      const unsigned int c = (mine[t] >> (8 * e)) & 255u;
      if (j < npre) {
        const bool admitted = c == 2u || (c == 1u && pt < ties);
        emit(j, admitted, ps + min(pt, ties));
      }
      ps += c == 2u; pt += c == 1u;
    }
  }
}

struct SelectArgs {
  const float* scores;
  const float* prior;          // two-stage only
  const int32_t* cu_seqlens;
  const int32_t* cu_budgets;
  int32_t* idx;
  uint8_t* member;             // two-stage only: [T] 1 = token kept by stage 1
  int32_t* member_count;       // two-stage only: [n_seqs]
  int n_seqs, T, TB, W;
  float span_ratio;
  int span_min;
};

struct ScoreSource {            // additive rule: every prefix token competes on its fused score
  const float* sc;
  __device__ uint32_t key(int j) const { return order_key(sc[j]); }
  __device__ bool eligible(int) const { return true; }
  __device__ bool forced(int) const { return false; }
};
struct PriorSource {            // two-stage, stage 1: marked tokens compete on their prior
  const float* p;
  __device__ uint32_t key(int j) const { return order_key(p[j]); }
  __device__ bool eligible(int j) const { return p[j] > 0.f; }
  __device__ bool forced(int) const { return false; }
};
struct FillSource {             // two-stage, stage 2: protected tokens are in, the others compete on attention
  const float* sc;
  const uint8_t* member;
  __device__ uint32_t key(int j) const { return order_key(sc[j]); }
  __device__ bool eligible(int j) const { return member[j] == 0; }
  __device__ bool forced(int j) const { return member[j] != 0; }
};

// additive rule: one selection on the fused scores
template <int NT, int ITEMS>
__global__ __launch_bounds__(NT) void select_kernel(SelectArgs a) {
  __shared__ SelectShared<NT> sh;
  const int tid = threadIdx.x;
  const int seq = blockIdx.x;
  const int lz = blockIdx.y;
  const int s0 = a.cu_seqlens[seq];
  const int n = a.cu_seqlens[seq + 1] - s0;
  const int o0 = a.cu_budgets[seq];
  const int budget = a.cu_budgets[seq + 1] - o0;
  const int npre = n - a.W;              // candidates
  const int need = budget - a.W;         // how many of them are kept
  int32_t* out = a.idx + (int64_t)lz * a.TB + o0;

  // the observation window is always kept
  for (int t = tid; t < a.W; t += NT) out[need + t] = npre + t;
  if (need <= 0) return;                 // uniform
  if (need >= npre) {                    // everything is kept
    for (int j = tid; j < npre; j += NT) out[j] = j;
    return;
  }
  if (npre > NT * ITEMS) return;         // the host picks ITEMS from the longest request: cannot happen
  ScoreSource src = {a.scores + (int64_t)lz * a.T + s0};
  select_wg<NT, ITEMS>(sh, src, [&](int j, bool admitted, int pos) { if (admitted) out[pos] = j; }, npre, need);
}

// two-stage rule, stage 1: once per request (the prior is shared by layers and heads)
template <int NT, int ITEMS>
__global__ __launch_bounds__(NT) void select_stage1_kernel(SelectArgs a) {
  __shared__ SelectShared<NT> sh;
  __shared__ int sh_flagged;
  const int tid = threadIdx.x;
  const int seq = blockIdx.x;
  const int s0 = a.cu_seqlens[seq];
  const int n = a.cu_seqlens[seq + 1] - s0;
  const int budget = a.cu_budgets[seq + 1] - a.cu_budgets[seq];
  const int npre = n - a.W;
  const int bp = budget - a.W;           // slots of the prefix
  const float* p = a.prior + s0;
  uint8_t* member = a.member + s0;

  for (int t = tid; t < a.W; t += NT) member[npre + t] = 0;
  // number of structurally marked prefix tokens
  if (tid == 0) sh_flagged = 0;
  __syncthreads();
  int mine = 0;
  for (int j = tid; j < npre; j += NT) mine += p[j] > 0.f;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off);
  if ((tid & 63) == 0 && mine) atomicAdd(&sh_flagged, mine);
  __syncthreads();
  const int flagged = sh_flagged;
  int bspan = max(a.span_min, (int)floor((double)a.span_ratio * (double)bp));
  bspan = min(bp, bspan);
  const int need = min(bspan, flagged);
  if (tid == 0) a.member_count[seq] = need;
  if (need <= 0 || npre > NT * ITEMS) {
    for (int j = tid; j < npre; j += NT) member[j] = 0;
    return;
  }
  PriorSource src = {p};
  select_wg<NT, ITEMS>(sh, src, [&](int j, bool admitted, int) { member[j] = admitted ? 1 : 0; }, npre, need);
}

// two-stage rule, stage 2: attention fills what stage 1 left
template <int NT, int ITEMS>
__global__ __launch_bounds__(NT) void select_stage2_kernel(SelectArgs a) {
  __shared__ SelectShared<NT> sh;
  const int tid = threadIdx.x;
  const int seq = blockIdx.x;
  const int lz = blockIdx.y;
  const int s0 = a.cu_seqlens[seq];
  const int n = a.cu_seqlens[seq + 1] - s0;
  const int o0 = a.cu_budgets[seq];
  const int budget = a.cu_budgets[seq + 1] - o0;
  const int npre = n - a.W;
  const int bp = budget - a.W;
  const int need = bp - a.member_count[seq];   // slots left for attention (>= 0)
  int32_t* out = a.idx + (int64_t)lz * a.TB + o0;

  for (int t = tid; t < a.W; t += NT) out[bp + t] = npre + t;
  if (bp <= 0) return;
  if (bp >= npre) {
    for (int j = tid; j < npre; j += NT) out[j] = j;
    return;
  }
  if (npre > NT * ITEMS) return;
  FillSource src = {a.scores + (int64_t)lz * a.T + s0, a.member + s0};
  select_wg<NT, ITEMS>(sh, src, [&](int j, bool admitted, int pos) { if (admitted) out[pos] = j; }, npre, need);
}

// ---------------------------------------------------------------------------------------------------------
// Selection by parts: several workgroups per problem, four kernels (see the head of this file).
// ---------------------------------------------------------------------------------------------------------

struct PartArgs {
  uint16_t* hist;        // [lz][part][2048] first-digit counts of each part (at most kPartChunk each)
  int32_t* sure;         // [lz][part] candidates of the part admitted whatever the cut: bins above the cut's, forced ones
  uint32_t* head;        // [lz][request][8]: mode, first digit of the cut, rank of the cut inside that bin, size of that bin,
                         //                   number of competing candidates admitted, key of the cut, ties admitted, 1 if `before` is filled in
  uint32_t* list;        // [lz][T] keys of the candidates in the cut's bin, per request from its first token on, in token order
  int32_t* before;       // [lz][part][2] candidates of the earlier parts in the cut's bin that lie above the cut / are tied at it
  int parts;             // parts of all requests together
};

enum { kModeNone = 0, kModeAll = 1, kModeSelect = 2 };   // no competing candidate admitted / all of them / a real selection

constexpr int kPartCopies = 4;       // private copies of a histogram (lane % 4)
constexpr int kPartHistWords = 8 * (kFirstDigitBins / 2 + 1);   // 8 packed copies of the first-digit counts, or 4 plain copies of a digit
static_assert(kPartHistWords >= kPartCopies * kHistStride, "histogram storage of the part kernels");

struct PartShared {
  unsigned int hist[kPartHistWords];
  unsigned int prefix, need;
  int red[4][16];          // up to 16 waves (the resolve kernel)
  int found[4];
};

// The three rules as seen by the part kernels: where the candidates come from, how many of them are admitted, what
// is written for a candidate and for the window.
struct RuleAdditive {
  using Src = ScoreSource;
  __device__ static Src source(const SelectArgs& a, int lz, int s0) { return {a.scores + (int64_t)lz * a.T + s0}; }
  __device__ static int need(const SelectArgs& a, int, int budget, int npre, int, int& mode) {
    const int need = budget - a.W;
    mode = need <= 0 ? kModeNone : (need >= npre ? kModeAll : kModeSelect);
    return need;
  }
  __device__ static void emit(const SelectArgs& a, int lz, int, int o0, int j, bool admitted, int pos, int limit) {
    if (admitted && (unsigned)pos < (unsigned)limit) a.idx[(int64_t)lz * a.TB + o0 + pos] = j;   // pos < limit always: belt and braces
  }
  __device__ static void window(const SelectArgs& a, int lz, int, int, int o0, int budget, int npre, int, int t) {
    a.idx[(int64_t)lz * a.TB + o0 + (budget - a.W) + t] = npre + t;
  }
};
struct RuleStage1 {     // once per request: which marked tokens the span budget keeps
  using Src = PriorSource;
  __device__ static Src source(const SelectArgs& a, int, int s0) { return {a.prior + s0}; }
  __device__ static int need(const SelectArgs& a, int, int budget, int, int marked, int& mode) {
    const int bp = budget - a.W;
    int bspan = max(a.span_min, (int)floor((double)a.span_ratio * (double)bp));
    bspan = min(bp, bspan);
    const int need = min(bspan, marked);
    mode = need <= 0 ? kModeNone : kModeSelect;       // need == marked: the selection admits every marked token
    return need;
  }
  __device__ static void emit(const SelectArgs& a, int, int s0, int, int j, bool admitted, int, int) {
    a.member[s0 + j] = admitted ? 1 : 0;
  }
  __device__ static void window(const SelectArgs& a, int, int seq, int s0, int, int, int npre, int need, int t) {
    a.member[s0 + npre + t] = 0;
    if (t == 0) a.member_count[seq] = need > 0 ? need : 0;
  }
};
struct RuleStage2 {     // per (layer, head, request): attention fills what stage 1 left
  using Src = FillSource;
  __device__ static Src source(const SelectArgs& a, int lz, int s0) { return {a.scores + (int64_t)lz * a.T + s0, a.member + s0}; }
  __device__ static int need(const SelectArgs& a, int seq, int budget, int npre, int, int& mode) {
    const int bp = budget - a.W;
    if (bp <= 0) { mode = kModeNone; return 0; }
    if (bp >= npre) { mode = kModeAll; return bp; }
    const int need = bp - a.member_count[seq];
    mode = need > 0 ? kModeSelect : kModeNone;
    return need;
  }
  __device__ static void emit(const SelectArgs& a, int lz, int, int o0, int j, bool admitted, int pos, int limit) {
    if (admitted && (unsigned)pos < (unsigned)limit) a.idx[(int64_t)lz * a.TB + o0 + pos] = j;   // pos < limit always: belt and braces
  }
  __device__ static void window(const SelectArgs& a, int lz, int, int, int o0, int budget, int npre, int, int t) {
    a.idx[(int64_t)lz * a.TB + o0 + (budget - a.W) + t] = npre + t;
  }
};

__device__ __forceinline__ int parts_of(int npre) { return npre > kPartChunk ? (npre + kPartChunk - 1) / kPartChunk : 1; }

// Sum of one int over the workgroup (all threads call it; `slot` picks one of four scratch rows so that
// back-to-back calls need no barrier in between).
__device__ __forceinline__ int part_sum(PartShared& sh, int v, int slot) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  if ((threadIdx.x & 63) == 0) sh.red[slot][threadIdx.x >> 6] = v;
  __syncthreads();
  int t = 0;
#pragma unroll
  for (int w = 0; w < kPartThreads / 64; ++w) t += sh.red[slot][w];
  return t;
}

// Exclusive prefix over the threads of the workgroup of two counts, and their totals (all threads call it).
__device__ __forceinline__ void part_scan2(PartShared& sh, int a, int b, int& before_a, int& before_b, int& tot_a, int& tot_b) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int sa = a, sb = b;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int oa = __shfl_up(sa, off), ob = __shfl_up(sb, off);
    if (lane >= off) { sa += oa; sb += ob; }
  }
  __syncthreads();                                 // the scratch rows may still be read from an earlier call
  if (lane == 63) { sh.red[0][wave] = sa; sh.red[1][wave] = sb; }
  __syncthreads();
  before_a = sa - a; before_b = sb - b; tot_a = 0; tot_b = 0;
#pragma unroll
  for (int w = 0; w < kPartThreads / 64; ++w) {
    if (w < wave) { before_a += sh.red[0][w]; before_b += sh.red[1][w]; }
    tot_a += sh.red[0][w]; tot_b += sh.red[1][w];
  }
}

// Which request and which of its parts workgroup `gp` of a launch works on; `first` = number of the request's first
// part.  All threads call it (two barriers): every thread adds up the parts of a share of the requests, a prefix sum
// over the threads finds the share that holds gp, its owner walks it.
__device__ __forceinline__ void locate_part(PartShared& sh, const int32_t* cu, int n_seqs, int W, int gp, int& seq, int& part, int& first) {
  const int tid = threadIdx.x;
  const int per = (n_seqs + kPartThreads - 1) / kPartThreads;
  const int r0 = min(tid * per, n_seqs), r1 = min(r0 + per, n_seqs);
  int mine = 0;
  for (int r = r0; r < r1; ++r) mine += parts_of(cu[r + 1] - cu[r] - W);
  int before, dummy_b, total, dummy_t;
  part_scan2(sh, mine, 0, before, dummy_b, total, dummy_t);
  if (tid == 0) { sh.found[0] = n_seqs - 1; sh.found[1] = 0; }      // gp past the end never happens (grid = total parts)
  __syncthreads();
  if (gp >= before && gp < before + mine) {                         // exactly one thread
    int pos = before, r = r0;
    for (;; ++r) {
      const int np = parts_of(cu[r + 1] - cu[r] - W);
      if (gp < pos + np) break;
      pos += np;
    }
    sh.found[0] = r; sh.found[1] = pos;
  }
  __syncthreads();
  seq = sh.found[0]; first = sh.found[1]; part = gp - first;
  __syncthreads();                                                  // found[] and the scratch rows are reused
}

// Candidate in slot s of this thread: the part is cut into tiles of 4 * kPartThreads candidates, a thread holds 4
// consecutive candidates of every tile (the loads of a wave cover whole cache lines).
constexpr int kPartTile = 4 * kPartThreads;
constexpr int kPartTiles = kPartItems / 4;
__device__ __forceinline__ int part_index(int part, int s) {
  return part * kPartChunk + (s >> 2) * kPartTile + (int)threadIdx.x * 4 + (s & 3);
}

template <class Src>
__device__ __forceinline__ void part_load(const Src& src, int npre, int part, uint32_t (&keys)[kPartItems], unsigned& elig, unsigned& forc) {
  static_assert(kPartItems <= 32 && kPartItems % 4 == 0, "one flag bit per candidate, whole tiles");
  elig = 0; forc = 0;
  if (npre > 0) {
#pragma unroll
    for (int s = 0; s < kPartItems; ++s) {                          // unconditional, clamped: all loads in flight together
      const int j = part_index(part, s), jc = j < npre ? j : npre - 1;
      const uint32_t key = src.key(jc);
      const bool el = src.eligible(jc), fo = src.forced(jc);
      keys[s] = j < npre ? key : 0u;
      if (j < npre && el) elig |= 1u << s;
      if (j < npre && fo) forc |= 1u << s;
    }
  } else {
#pragma unroll
    for (int s = 0; s < kPartItems; ++s) keys[s] = 0u;
  }
}

// Places in token order.  In: per tile, a count (or two counts below 2^16 packed into the halves of a word) over this
// thread's 4 candidates of the tile.  Out: per tile, the same count(s) over all candidates of the part that come before
// them.  All threads call it.  The counts go through LDS as a [tile][thread] table, which is token order when read flat.
__device__ __forceinline__ void part_order(PartShared& sh, const unsigned int (&cnt)[kPartTiles], unsigned int (&before)[kPartTiles]) {
  unsigned int* table = sh.hist;                         // free at this point in both callers
  const int tid = threadIdx.x;
  __syncthreads();
#pragma unroll
  for (int t = 0; t < kPartTiles; ++t) table[t * kPartThreads + tid] = cnt[t];
  __syncthreads();
  unsigned int loc[kPartTiles], run = 0;
#pragma unroll
  for (int i = 0; i < kPartTiles; ++i) { loc[i] = run; run += table[tid * kPartTiles + i]; }
  int ba, bb, ta, tb;
  part_scan2(sh, (int)(run & 0xFFFFu), (int)(run >> 16), ba, bb, ta, tb);
  const unsigned int base = (unsigned int)ba | ((unsigned int)bb << 16);
#pragma unroll
  for (int i = 0; i < kPartTiles; ++i) table[tid * kPartTiles + i] = base + loc[i];
  __syncthreads();
#pragma unroll
  for (int t = 0; t < kPartTiles; ++t) before[t] = table[t * kPartThreads + tid];
  __syncthreads();
}

template <int NT = kPartThreads>
__device__ __forceinline__ void part_hist_clear(PartShared& sh, int nbins) {
  for (int b = threadIdx.x; b < (kPartCopies - 1) * kHistStride + nbins; b += NT) sh.hist[b] = 0;
  __syncthreads();
}

// counts: first digit of the part's competing candidates.  Every bin is stored, so nothing has to be cleared beforehand.
template <class Rule>
__global__ __launch_bounds__(kPartThreads) void part_counts_kernel(SelectArgs a, PartArgs c) {
  __shared__ PartShared sh;
  const int tid = threadIdx.x, gp = blockIdx.x, lz = blockIdx.y;
  int seq, part, first;
  locate_part(sh, a.cu_seqlens, a.n_seqs, a.W, gp, seq, part, first);
  const int s0 = a.cu_seqlens[seq];
  const int npre = a.cu_seqlens[seq + 1] - s0 - a.W;
  uint32_t keys[kPartItems];
  unsigned elig, forc;
  part_load(Rule::source(a, lz, s0), npre, part, keys, elig, forc);
  // A part holds at most kPartChunk < 2^16 candidates: two bins share a word, and there is room for 8 private copies
  // (lane % 8) of the table, which matters because the scores crowd into a few dozen bins.
  constexpr int COPIES = 8, STRIDE = kFirstDigitBins / 2 + 1;
  static_assert(COPIES * STRIDE <= kPartHistWords && kPartChunk < 65536, "packed first-digit counts");
  for (int b = tid; b < COPIES * STRIDE; b += kPartThreads) sh.hist[b] = 0;
  __syncthreads();
#pragma unroll
  for (int s = 0; s < kPartItems; ++s) {
    const uint32_t bin = keys[s] >> 21;
    if ((elig >> s) & 1u) atomicAdd(&sh.hist[(tid & (COPIES - 1)) * STRIDE + (bin >> 1)], 1u << (16 * (bin & 1u)));
  }
  __syncthreads();
  uint32_t* out = reinterpret_cast<uint32_t*>(c.hist + ((int64_t)lz * c.parts + gp) * kFirstDigitBins);
  for (int w = tid; w < kFirstDigitBins / 2; w += kPartThreads) {       // a sum below 2^16 per half: no carry between them
    unsigned int t = 0;
#pragma unroll
    for (int k = 0; k < COPIES; ++k) t += sh.hist[k * STRIDE + w];
    out[w] = t;
  }
}

// near: the bin that holds the cut, and the request's list of the candidates in that bin.
template <class Rule>
__global__ __launch_bounds__(kPartThreads) void part_near_kernel(SelectArgs a, PartArgs c) {
  __shared__ PartShared sh;
  const int tid = threadIdx.x, gp = blockIdx.x, lz = blockIdx.y;
  int seq, part, first;
  locate_part(sh, a.cu_seqlens, a.n_seqs, a.W, gp, seq, part, first);
  const int s0 = a.cu_seqlens[seq];
  const int npre = a.cu_seqlens[seq + 1] - s0 - a.W;
  const int budget = a.cu_budgets[seq + 1] - a.cu_budgets[seq];
  const int nparts = parts_of(npre);
  uint32_t keys[kPartItems];
  unsigned elig, forc;
  part_load(Rule::source(a, lz, s0), npre, part, keys, elig, forc);

  // counts of the 8 bins this thread owns (bins 8 * tid ...), over all parts of the request and in this part alone
  constexpr int OWN = kFirstDigitBins / kPartThreads;
  static_assert(OWN == 8, "one 16-byte load per part and thread");
  unsigned int tot[OWN], own[OWN];
#pragma unroll
  for (int i = 0; i < OWN; ++i) { tot[i] = 0; own[i] = 0; }
  const uint16_t* hp = c.hist + ((int64_t)lz * c.parts + first) * kFirstDigitBins + tid * OWN;
  constexpr int BATCH = 8;                                // loads in flight
  for (int q0 = 0; q0 < nparts; q0 += BATCH) {
    uint4 v[BATCH];
#pragma unroll
    for (int u = 0; u < BATCH; ++u)
      v[u] = *reinterpret_cast<const uint4*>(hp + (int64_t)min(q0 + u, nparts - 1) * kFirstDigitBins);
#pragma unroll
    for (int u = 0; u < BATCH; ++u) {
      if (q0 + u >= nparts) continue;
      const unsigned int w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int i = 0; i < OWN; ++i) {
        const unsigned int x = (w[i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
        tot[i] += x;
        if (q0 + u == part) own[i] = x;
      }
    }
  }
  int mine = 0;
#pragma unroll
  for (int i = 0; i < OWN; ++i) mine += (int)tot[i];
  // candidates in the bins of higher threads (higher bins hold larger keys), and all competing candidates
  int below, dummy_b, total, dummy_t;
  part_scan2(sh, mine, 0, below, dummy_b, total, dummy_t);
  const int above = total - below - mine;
  int mode;
  const int need = Rule::need(a, seq, budget, npre, total, mode);
  if (tid == 0) { sh.found[0] = 0; sh.found[1] = 0; sh.found[2] = 0; }
  __syncthreads();
  if (mode == kModeSelect && above < need && need <= above + mine) {   // exactly one thread: the cut lies in one of its bins
    int higher = above;
    for (int i = OWN - 1; i >= 0; --i) {
      if (need <= higher + (int)tot[i]) { sh.found[0] = tid * OWN + i; sh.found[1] = need - higher; sh.found[2] = (int)tot[i]; break; }
      higher += (int)tot[i];
    }
  }
  __syncthreads();
  const int b0 = sh.found[0];
  if (part == 0 && tid == 0) {
    uint32_t* h = c.head + ((int64_t)lz * a.n_seqs + seq) * 8;
    h[0] = (uint32_t)mode; h[1] = (uint32_t)b0; h[2] = (uint32_t)sh.found[1]; h[3] = (uint32_t)sh.found[2];
    h[4] = (uint32_t)need;
  }
  // candidates of this part admitted whatever the cut: its bins above b0 (none when nothing is selected), forced ones
  int sure = __popc(forc);
  if (mode == kModeSelect) {
#pragma unroll
    for (int i = 0; i < OWN; ++i) sure += tid * OWN + i > b0 ? (int)own[i] : 0;
  }
  sure = part_sum(sh, sure, 2);
  if (tid == 0) c.sure[(int64_t)lz * c.parts + gp] = sure;
  if (mode != kModeSelect) return;                                     // the same for every thread
  // where this part's share of the list begins: candidates of the earlier parts in bin b0
  int off = 0;
  for (int q = tid; q < part; q += kPartThreads) off += c.hist[((int64_t)lz * c.parts + first + q) * kFirstDigitBins + b0];
  off = part_sum(sh, off, 3);
  unsigned int cnt[kPartTiles], before[kPartTiles];
#pragma unroll
  for (int t = 0; t < kPartTiles; ++t) {
    cnt[t] = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) cnt[t] += ((elig >> (4 * t + e)) & 1u) && (int)(keys[4 * t + e] >> 21) == b0;
  }
  part_order(sh, cnt, before);
  uint32_t* list = c.list + (int64_t)lz * a.T + s0 + off;              // at most npre entries per request: inside its tokens
#pragma unroll
  for (int t = 0; t < kPartTiles; ++t) {
    unsigned int pos = before[t];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (((elig >> (4 * t + e)) & 1u) && (int)(keys[4 * t + e] >> 21) == b0) list[pos++] = keys[4 * t + e];
  }
}

// One more digit of the radix select over the request's list (all NT threads of the workgroup call it).  Entries whose
// bits above the digit equal `prefix` take part; afterwards `prefix` has the digit filled in and `remaining` is the
// rank inside it.
template <int NT>
__device__ __forceinline__ void part_digit(PartShared& sh, const uint32_t* list, int m, int shift, int nbins, uint32_t himask,
                                           uint32_t& prefix, uint32_t& remaining) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  part_hist_clear<NT>(sh, nbins);
  constexpr int UNR = 8;                                  // loads in flight per thread
  for (int i0 = tid; i0 < m; i0 += NT * UNR) {
    uint32_t k[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) k[u] = list[min(i0 + u * NT, m - 1)];
#pragma unroll
    for (int u = 0; u < UNR; ++u)
      if (i0 + u * NT < m && (k[u] & himask) == prefix)
        atomicAdd(&sh.hist[(tid & (kPartCopies - 1)) * kHistStride + ((k[u] >> shift) & (uint32_t)(nbins - 1))], 1u);
  }
  __syncthreads();
  for (int b = tid; b < nbins; b += NT) {
    unsigned int t = 0;
#pragma unroll
    for (int k = 0; k < kPartCopies; ++k) t += sh.hist[k * kHistStride + b];
    sh.hist[b] = t;
  }
  __syncthreads();
  if (wave == 0) {                       // lane owns bins [lane * per, lane * per + per); higher bins hold larger keys
    const int per = nbins / 64;
    unsigned int mine = 0;
    for (int i = 0; i < per; ++i) mine += sh.hist[lane * per + i];
    unsigned int run = mine;             // inclusive suffix sum over lanes
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const unsigned int o = __shfl_down(run, off);
      if (lane + off < 64) run += o;
    }
    const unsigned int above = run - mine;
    if (above < remaining && remaining <= above + mine) {        // exactly one lane
      unsigned int higher = above;
      for (int i = per - 1; i >= 0; --i) {
        const unsigned int cbin = sh.hist[lane * per + i];
        if (remaining <= higher + cbin) { sh.prefix = prefix | ((uint32_t)(lane * per + i) << shift); sh.need = remaining - higher; break; }
        higher += cbin;
      }
    }
  }
  __syncthreads();
  prefix = sh.prefix;
  remaining = sh.need;
  __syncthreads();
}

// resolve: one workgroup per problem finishes the radix select on the request's list (two more digits) and leaves
// the key of the cut and the number of candidates tied at it that are admitted.
constexpr int kResolveThreads = 1024;     // the list is read with 8 loads in flight per thread: many threads, few rounds
__global__ __launch_bounds__(kResolveThreads) void part_resolve_kernel(SelectArgs a, PartArgs c) {
  __shared__ PartShared sh;
  const int seq = blockIdx.x, lz = blockIdx.y;
  uint32_t* h = c.head + ((int64_t)lz * a.n_seqs + seq) * 8;
  if ((int)h[0] != kModeSelect) return;                      // the same for every thread
  const uint32_t* list = c.list + (int64_t)lz * a.T + a.cu_seqlens[seq];
  const int m = (int)h[3];
  uint32_t prefix = h[1] << 21, remaining = h[2];
  part_digit<kResolveThreads>(sh, list, m, 10, 2048, 0xFFE00000u, prefix, remaining);
  part_digit<kResolveThreads>(sh, list, m, 0, 1024, 0xFFFFFC00u, prefix, remaining);
  const uint32_t tau = prefix;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // How many list entries of each part lie above the cut / are tied at it, as running totals over the parts: an
  // emitting part then knows what the earlier parts contribute without reading their stretch of the list again.
  const int npre = a.cu_seqlens[seq + 1] - a.cu_seqlens[seq] - a.W;
  const int nparts = parts_of(npre);
  const bool fits = 3 * nparts <= kPartHistWords;            // else the emitting parts count for themselves
  if (tid == 0) { h[5] = tau; h[6] = remaining; h[7] = fits ? 1u : 0u; }
  if (!fits) return;                                         // the same for every thread
  int mine = 0;                                              // number of this request's first part
  for (int r = tid; r < seq; r += kResolveThreads) mine += parts_of(a.cu_seqlens[r + 1] - a.cu_seqlens[r] - a.W);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off);
  if (lane == 0) sh.red[0][wave] = mine;
  __syncthreads();
  int first = 0;
#pragma unroll
  for (int w = 0; w < kResolveThreads / 64; ++w) first += sh.red[0][w];
  unsigned int* seg_end = sh.hist;                           // end of each part's stretch of the list
  unsigned int* n_above = sh.hist + nparts;
  unsigned int* n_tied = sh.hist + 2 * nparts;
  const int b0 = (int)h[1];
  for (int q = tid; q < nparts; q += kResolveThreads) {
    seg_end[q] = c.hist[((int64_t)lz * c.parts + first + q) * kFirstDigitBins + b0];
    n_above[q] = 0; n_tied[q] = 0;
  }
  __syncthreads();
  // running totals over the parts, 64 at a time, by the first wave: seg_end becomes the end offsets
  auto running = [&](unsigned int* v, bool exclusive) __attribute__((always_inline)) {
    if (wave == 0) {
      unsigned int carry = 0;
      for (int base = 0; base < nparts; base += 64) {
        const unsigned int x = base + lane < nparts ? v[base + lane] : 0u;
        unsigned int incl = x;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const unsigned int o = __shfl_up(incl, off);
          if (lane >= off) incl += o;
        }
        if (base + lane < nparts) v[base + lane] = carry + (exclusive ? incl - x : incl);
        carry += __shfl(incl, 63);
      }
    }
    __syncthreads();
  };
  running(seg_end, false);
  constexpr int UNR = 8;
  for (int i0 = tid; i0 < m; i0 += kResolveThreads * UNR) {
    uint32_t k[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) k[u] = list[min(i0 + u * kResolveThreads, m - 1)];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int i = i0 + u * kResolveThreads;
      if (i >= m || k[u] < tau) continue;
      int lo = 0, hi = nparts - 1;                           // first part whose stretch ends beyond i
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (seg_end[mid] > (unsigned int)i) hi = mid; else lo = mid + 1;
      }
      atomicAdd(k[u] > tau ? &n_above[lo] : &n_tied[lo], 1u);
    }
  }
  __syncthreads();
  running(n_above, true);
  running(n_tied, true);
  for (int q = tid; q < nparts; q += kResolveThreads) {
    int32_t* out = c.before + ((int64_t)lz * c.parts + first + q) * 2;
    out[0] = (int32_t)n_above[q]; out[1] = (int32_t)n_tied[q];
  }
}

// emit: every part writes its admitted candidates at their final places.
template <class Rule>
__global__ __launch_bounds__(kPartThreads) void part_emit_kernel(SelectArgs a, PartArgs c) {
  __shared__ PartShared sh;
  const int tid = threadIdx.x, gp = blockIdx.x, lz = blockIdx.y;
  int seq, part, first;
  locate_part(sh, a.cu_seqlens, a.n_seqs, a.W, gp, seq, part, first);
  const int s0 = a.cu_seqlens[seq];
  const int npre = a.cu_seqlens[seq + 1] - s0 - a.W;
  const int o0 = a.cu_budgets[seq];
  const int budget = a.cu_budgets[seq + 1] - o0;
  uint32_t keys[kPartItems];
  unsigned elig, forc;
  part_load(Rule::source(a, lz, s0), npre, part, keys, elig, forc);
  const uint32_t* h = c.head + ((int64_t)lz * a.n_seqs + seq) * 8;
  const int mode = (int)h[0], b0 = (int)h[1], need = (int)h[4];
  if (part == 0)
    for (int t = tid; t < a.W; t += kPartThreads) Rule::window(a, lz, seq, s0, o0, budget, npre, need, t);
  if (mode == kModeAll) {                                    // every candidate is kept at its own place
#pragma unroll
    for (int s = 0; s < kPartItems; ++s) {
      const int j = part_index(part, s);
      if (j < npre) Rule::emit(a, lz, s0, o0, j, true, j, budget - a.W);
    }
    return;
  }
  uint32_t tau = 0xFFFFFFFFu;
  int ties = 0, above_before = 0, ties_before = 0;
  if (mode == kModeSelect) {
    const uint32_t* list = c.list + (int64_t)lz * a.T + s0;
    tau = h[5];
    ties = (int)h[6];
    int ab = 0, tb = 0;
    if (h[7] != 0u) {                                     // the resolve kernel has counted for every part
      const int32_t* bf = c.before + ((int64_t)lz * c.parts + gp) * 2;
      if (tid == 0) { ab = bf[0]; tb = bf[1]; }
    } else {
      // what the earlier parts hold of the list: their entries come first
      int off = 0;
      for (int q = tid; q < part; q += kPartThreads) off += c.hist[((int64_t)lz * c.parts + first + q) * kFirstDigitBins + b0];
      off = part_sum(sh, off, 2);
      constexpr int UNR = 8;
      for (int i0 = tid; i0 < off; i0 += kPartThreads * UNR) {
        uint32_t k[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) k[u] = list[min(i0 + u * kPartThreads, off - 1)];
#pragma unroll
        for (int u = 0; u < UNR; ++u)
          if (i0 + u * kPartThreads < off) { ab += k[u] > tau; tb += k[u] == tau; }
      }
      __syncthreads();
    }
    above_before = part_sum(sh, ab, 3);
    __syncthreads();
    ties_before = part_sum(sh, tb, 2);
  }
  int sure_before = 0;
  for (int q = tid; q < part; q += kPartThreads) sure_before += c.sure[(int64_t)lz * c.parts + first + q];
  __syncthreads();
  sure_before = part_sum(sh, sure_before, 3) + above_before;
  // classes of this thread's candidates: in whatever the cut / tied at the cut / out
  unsigned in2 = 0, in1 = 0;
  unsigned int cnt[kPartTiles], before[kPartTiles];
#pragma unroll
  for (int s = 0; s < kPartItems; ++s) {
    const bool el = (elig >> s) & 1u, fo = (forc >> s) & 1u;
    const bool two = fo || (el && mode == kModeSelect && keys[s] > tau);
    const bool one = !fo && el && mode == kModeSelect && keys[s] == tau;
    if (two) in2 |= 1u << s;
    if (one) in1 |= 1u << s;
  }
#pragma unroll
  for (int t = 0; t < kPartTiles; ++t) cnt[t] = __popc((in2 >> (4 * t)) & 15u) | (__popc((in1 >> (4 * t)) & 15u) << 16);
  part_order(sh, cnt, before);
#pragma unroll
  for (int t = 0; t < kPartTiles; ++t) {
    int ps = sure_before + (int)(before[t] & 0xFFFFu), pt = ties_before + (int)(before[t] >> 16);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int s = 4 * t + e, j = part_index(part, s);
      const bool two = (in2 >> s) & 1u, one = (in1 >> s) & 1u;
      if (j < npre) Rule::emit(a, lz, s0, o0, j, two || (one && pt < ties), ps + min(pt, ties), budget - a.W);
      ps += two; pt += one;
    }
  }
}

// Which one-workgroup kernel: 256 threads when every request fits 256 x 16 candidates and the batch has enough
// problems to keep several such workgroups on every compute unit, else 1024 threads.
static bool small_workgroups(const Plan& pl, int64_t problems) {
  return pl.max_n - pl.W <= kSelectSmallThreads * kSelectSmallMaxItems && problems >= kSelectSmallProblems;
}
// candidates kept in registers per thread, chosen from the longest request
static int items_for(const Plan& pl, int threads) {
  const int npre = pl.max_n - pl.W;
  for (int items : {8, 16, 32, 48}) if (npre <= threads * items) return items;
  return 64;
}

#define CODECOMP_DISPATCH_ITEMS(KERNEL, GRID, PROBLEMS, ARGS)                                              \
  if (small_workgroups(pl, PROBLEMS)) {                                                                    \
    switch (items_for(pl, kSelectSmallThreads)) {                                                          \
      case 8: KERNEL<kSelectSmallThreads, 8><<<GRID, dim3(kSelectSmallThreads), 0, stream>>>(ARGS); break;   \
      default: KERNEL<kSelectSmallThreads, 16><<<GRID, dim3(kSelectSmallThreads), 0, stream>>>(ARGS); break; \
    }                                                                                                      \
  } else {                                                                                                 \
    switch (items_for(pl, kSelectThreads)) {                                                               \
      case 8: KERNEL<kSelectThreads, 8><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;           \
      case 16: KERNEL<kSelectThreads, 16><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;         \
      case 32: KERNEL<kSelectThreads, 32><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;         \
      case 48: KERNEL<kSelectThreads, 48><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;         \
      default: KERNEL<kSelectThreads, 64><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;         \
    }                                                                                                      \
  }

static PartArgs part_args(const Plan& pl, void* workspace) {
  char* ws = static_cast<char*>(workspace);
  PartArgs c;
  c.hist = reinterpret_cast<uint16_t*>(ws + pl.off_part_hist);
  c.sure = reinterpret_cast<int32_t*>(ws + pl.off_part_sure);
  c.head = reinterpret_cast<uint32_t*>(ws + pl.off_part_head);
  c.list = reinterpret_cast<uint32_t*>(ws + pl.off_uraw);       // the raw attention mass is dead once the scores exist
  c.before = reinterpret_cast<int32_t*>(ws + pl.off_part_before);
  c.parts = pl.sel_parts;
  return c;
}

template <class Rule>
static int launch_parts(const Plan& pl, const SelectArgs& a, const PartArgs& c, int lzs, hipStream_t stream) {
  const dim3 grid(pl.sel_parts, lzs), block(kPartThreads);
  part_counts_kernel<Rule><<<grid, block, 0, stream>>>(a, c);
  if (hipError_t e = hipGetLastError()) return (int)e;
  part_near_kernel<Rule><<<grid, block, 0, stream>>>(a, c);
  if (hipError_t e = hipGetLastError()) return (int)e;
  part_resolve_kernel<<<dim3(pl.n_seqs, lzs), dim3(kResolveThreads), 0, stream>>>(a, c);
  if (hipError_t e = hipGetLastError()) return (int)e;
  part_emit_kernel<Rule><<<grid, block, 0, stream>>>(a, c);
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

int launch_select(const Plan& pl, const float* scores, int32_t* idx, void* workspace, hipStream_t stream) {
  SelectArgs a = {};
  a.scores = scores; a.cu_seqlens = pl.cu_seqlens_dev; a.cu_budgets = pl.cu_budgets_dev; a.idx = idx;
  a.n_seqs = pl.n_seqs; a.T = pl.T; a.TB = pl.TB; a.W = pl.W;
  if (pl.sel_parts > 0) return launch_parts<RuleAdditive>(pl, a, part_args(pl, workspace), pl.L * pl.Hkv, stream);
  CODECOMP_DISPATCH_ITEMS(select_kernel, dim3(pl.n_seqs, pl.L * pl.Hkv), (int64_t)pl.n_seqs * pl.L * pl.Hkv, a)
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

int launch_select_two_stage(const Plan& pl, const float* scores, const float* prior, int32_t* idx, void* workspace,
                            hipStream_t stream) {
  char* ws = static_cast<char*>(workspace);
  SelectArgs a = {};
  a.scores = scores; a.prior = prior; a.cu_seqlens = pl.cu_seqlens_dev; a.cu_budgets = pl.cu_budgets_dev; a.idx = idx;
  a.member = reinterpret_cast<uint8_t*>(ws + pl.off_member);
  a.member_count = reinterpret_cast<int32_t*>(ws + pl.off_member_count);
  a.n_seqs = pl.n_seqs; a.T = pl.T; a.TB = pl.TB; a.W = pl.W;
  a.span_ratio = pl.span_ratio; a.span_min = pl.span_min;
  if (pl.sel_parts > 0) {
    const PartArgs c = part_args(pl, workspace);
    if (int rc = launch_parts<RuleStage1>(pl, a, c, 1, stream)) return rc;
    return launch_parts<RuleStage2>(pl, a, c, pl.L * pl.Hkv, stream);
  }
  CODECOMP_DISPATCH_ITEMS(select_stage1_kernel, dim3(pl.n_seqs), (int64_t)pl.n_seqs, a)
  if (hipError_t e = hipGetLastError()) return (int)e;
  CODECOMP_DISPATCH_ITEMS(select_stage2_kernel, dim3(pl.n_seqs, pl.L * pl.Hkv), (int64_t)pl.n_seqs * pl.L * pl.Hkv, a)
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

}  // namespace codecomp
