// Select step: per (layer, KV head, request) keep the last W tokens and the B - W best tokens
// of the prefix [0, N - W); equal scores go to the lower index; indices come out ascending
// (section "Attention-based KV Cache Compression": the best-scored context tokens are kept until the budget is used up).
//
// One workgroup of 1024 threads owns one problem.  An MSB-first radix select over order-preserving
// integer images of the float scores (digits of 11, 11 and 10 bits, LDS histogram) finds the score
// of the last admitted token and how many tokens tied at that score are admitted; one ordered pass
// (workgroup prefix sums of "sure" and "tied" flags) then writes the indices already sorted.
// The candidates are read from memory ONCE, all loads in flight together, and stay in registers
// through the three digit passes and the ordered pass (up to 64 per thread, N - W <= 65536); longer
// requests fall back to re-reading the score row, which then lives in L2.
//
// Two selection rules share these pieces:
//   additive   : one selection on c = pooled attention + lambda * prior (the score kernel's output);
//   two-stage  : the paper's literal order - structure first, attention fills the rest
//                (sections "Span-Level Structural Protection" and "Attention-based KV Cache
//                Compression"): stage 1 keeps up to B_span = min(Bp, max(B_min, floor(rho * Bp)))
//                prefix tokens with prior > 0, largest prior first (ties: first in sequence, which for a
//                binary prior is the paper's rule for an overfull protected set: its first tokens), Bp = B - W; stage 2 fills the remaining
//                Bp - |P| slots with the best pooled-attention tokens not in P.
#include "plan.h"

namespace codecomp {

// Monotone map float -> uint32 (larger float <=> larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t order_key(float x) {
  x = x + 0.0f;   // -0 -> +0
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kSelTileItems = 4;    // consecutive candidates per thread inside one ordered tile
constexpr int kSelTile = kSelectThreads * kSelTileItems;

constexpr int kHistCopies = 8;      // private copies of the first-digit histogram, picked by lane % 8
constexpr int kHistStride = 2049;   // odd stride: equal bins of different copies sit in different banks

struct SelectShared {
  unsigned int hist[kHistCopies * kHistStride];
  unsigned int prefix, need;
  int wave_sure[kSelectThreads / 64], wave_tie[kSelectThreads / 64];
  int tile_sure, tile_tie;
  // class (0 out, 1 tied at the cut, 2 in) of every register-resident candidate, one byte each, indexed by
  // candidate: written in the load layout, read back as runs of consecutive candidates per thread
  unsigned int cls_words[kSelectThreads * 64 / 4];
};

// One candidate into the digit histogram.  CROWDED (the first digit: every candidate takes part and the scores
// crowd into a few dozen bins): LDS atomics of one instruction that hit the same address are served one after
// the other, so each lane adds to one of kHistCopies private copies (lane % 8) and at most 8 lanes can collide;
// the copies are summed when the bin is picked.  Ballot-based aggregation was tried first: its serial
// scalar/vector control flow cost about 1000 cycles per candidate slot and workgroup.  Later digits: only the
// few candidates that share the prefix take part, one copy.
template <bool CROWDED>
__device__ __forceinline__ void hist_add(SelectShared& sh, bool match, uint32_t bin) {
  if (match) atomicAdd(&sh.hist[(CROWDED ? (threadIdx.x & (kHistCopies - 1)) * kHistStride : 0) + bin], 1u);
}

__device__ __forceinline__ int pass_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int pass_bins(int pass) { return pass == 2 ? 1024 : 2048; }
__device__ __forceinline__ uint32_t pass_himask(int pass) {
  return pass == 0 ? 0u : (0xFFFFFFFFu << (pass == 1 ? 21 : 10));
}

__device__ __forceinline__ void hist_clear(SelectShared& sh, int nbins, int copies) {
  for (int b = threadIdx.x; b < (copies - 1) * kHistStride + nbins; b += kSelectThreads) sh.hist[b] = 0;
  __syncthreads();
}

// After a digit pass: the bin holding the `remaining`-th largest candidate; fixes that digit in `prefix`
// and reduces `remaining` to the rank inside the bin.  All threads call it.  No step waits for an LDS
// read that depends on the previous one: the copies are summed by all threads, wave 0 finds the lane whose
// group of bins holds the rank (suffix sums over lanes), then the bin inside that group the same way.
__device__ __forceinline__ void hist_pick(SelectShared& sh, int nbins, int copies, int shift, uint32_t& prefix,
                                          uint32_t& remaining) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (copies > 1) {                    // totals of the private copies into copy 0 (a thread touches only its own bins)
    for (int b = threadIdx.x; b < nbins; b += kSelectThreads) {
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
__device__ __forceinline__ void tile_scan(SelectShared& sh, int nsure, int ntie, int& before_sure, int& before_tie,
                                          int& tot_sure, int& tot_tie) {
  constexpr int NWV = kSelectThreads / 64;
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
// ITEMS > 0: candidates are loaded once into registers (npre <= kSelectThreads * ITEMS);
// ITEMS == 0: every pass re-reads them.
// emit(j, admitted, pos) is called for every j, pos = number of admitted candidates before j.
template <int ITEMS, class Source, class Emit>
__device__ __forceinline__ void select_wg(SelectShared& sh, Source src, Emit emit, int npre, int need) {
  constexpr int NT = kSelectThreads;
  const int tid = threadIdx.x;
  constexpr int NREG = ITEMS > 0 ? ITEMS : 1;
  uint32_t keys[NREG];
  unsigned long long elig = 0, forc = 0;       // one bit per register slot
  // slot s of this thread holds candidate j = (s / 4) * kSelTile + tid * 4 + (s % 4): tiles in order, 4 consecutive
  if constexpr (ITEMS > 0) {
    if (npre > 0) {                            // the same for every thread
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
  }

  uint32_t tau = 0xFFFFFFFFu;
  int ties = 0;                               // need == 0: only forced candidates are admitted
  if (need > 0) {
    uint32_t prefix = 0, remaining = (uint32_t)need;
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
      const int shift = pass_shift(pass), nbins = pass_bins(pass);
      const uint32_t himask = pass_himask(pass);
      const int copies = pass == 0 ? kHistCopies : 1;
      hist_clear(sh, nbins, copies);
      if constexpr (ITEMS > 0) {
#pragma unroll
        for (int s = 0; s < ITEMS; ++s) {
          const bool match = ((elig >> s) & 1ull) && (keys[s] & himask) == prefix;
          if (pass == 0) hist_add<true>(sh, match, (keys[s] >> shift) & (uint32_t)(nbins - 1));
          else hist_add<false>(sh, match, (keys[s] >> shift) & (uint32_t)(nbins - 1));
        }
      } else {
        const int npad = (npre + NT - 1) / NT * NT;   // uniform trip counts: every lane takes part in the ballots
        constexpr int UNR = 8;                        // loads in flight per thread
        for (int j0 = tid; j0 < npad; j0 += NT * UNR) {
          uint32_t k8[UNR];
          bool v8[UNR];
#pragma unroll
          for (int u = 0; u < UNR; ++u) {
            const int j = j0 + u * NT;
            k8[u] = 0u; v8[u] = false;
            if (j < npre) { k8[u] = src.key(j); v8[u] = src.eligible(j); }
          }
#pragma unroll
          for (int u = 0; u < UNR; ++u)
            if (pass == 0) hist_add<true>(sh, v8[u] && (k8[u] & himask) == prefix, (k8[u] >> shift) & (uint32_t)(nbins - 1));
            else hist_add<false>(sh, v8[u] && (k8[u] & himask) == prefix, (k8[u] >> shift) & (uint32_t)(nbins - 1));
        }
      }
      hist_pick(sh, nbins, copies, shift, prefix, remaining);
    }
    tau = prefix;
    ties = (int)remaining;
  }

  // ---- ordered pass
  int carry_sure = 0, carry_tie = 0;
  const int ntiles = (npre + kSelTile - 1) / kSelTile;
  auto do_tile = [&](int t, const int (&cls)[kSelTileItems]) __attribute__((always_inline)) {
    int nsure = 0, ntie = 0;
#pragma unroll
    for (int e = 0; e < kSelTileItems; ++e) { nsure += cls[e] == 2; ntie += cls[e] == 1; }
    int bs, bt, ts, tt;
    tile_scan(sh, nsure, ntie, bs, bt, ts, tt);
    int ps = carry_sure + bs, pt = carry_tie + bt;
#pragma unroll
    for (int e = 0; e < kSelTileItems; ++e) {
      const int j = t * kSelTile + tid * kSelTileItems + e;
      if (j < npre) {
        const bool admitted = cls[e] == 2 || (cls[e] == 1 && pt < ties);
        emit(j, admitted, ps + min(pt, ties));
      }
      ps += cls[e] == 2; pt += cls[e] == 1;
    }
    carry_sure += ts; carry_tie += tt;
  };
  if constexpr (ITEMS > 0) {
    // The classes go through LDS so that every thread ends up with ITEMS consecutive candidates: one workgroup
    // prefix sum instead of one per tile, and each thread writes its admitted indices to consecutive places.
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
      sh.cls_words[t * kSelectThreads + tid] = word;       // candidates 4 * (t * 1024 + tid) .. + 3
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
  } else {
    for (int t = 0; t < ntiles; ++t) {
      int cls[kSelTileItems];
#pragma unroll
      for (int e = 0; e < kSelTileItems; ++e) {
        const int j = t * kSelTile + tid * kSelTileItems + e;
        cls[e] = 0;
        if (j < npre) {
          if (src.forced(j)) cls[e] = 2;
          else if (src.eligible(j)) { const uint32_t key = src.key(j); cls[e] = key > tau ? 2 : (key == tau ? 1 : 0); }
        }
      }
      do_tile(t, cls);
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
template <int ITEMS>
__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectArgs a) {
  constexpr int NT = kSelectThreads;
  __shared__ SelectShared sh;
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
  if (ITEMS > 0 && npre > NT * ITEMS) return;   // the host picks ITEMS from the longest request: cannot happen
  ScoreSource src = {a.scores + (int64_t)lz * a.T + s0};
  select_wg<ITEMS>(sh, src, [&](int j, bool admitted, int pos) { if (admitted) out[pos] = j; }, npre, need);
}

// two-stage rule, stage 1: once per request (the prior is shared by layers and heads)
template <int ITEMS>
__global__ __launch_bounds__(kSelectThreads) void select_stage1_kernel(SelectArgs a) {
  constexpr int NT = kSelectThreads;
  __shared__ SelectShared sh;
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
  if (need <= 0 || (ITEMS > 0 && npre > NT * ITEMS)) {
    for (int j = tid; j < npre; j += NT) member[j] = 0;
    return;
  }
  PriorSource src = {p};
  select_wg<ITEMS>(sh, src, [&](int j, bool admitted, int) { member[j] = admitted ? 1 : 0; }, npre, need);
}

// two-stage rule, stage 2: attention fills what stage 1 left
template <int ITEMS>
__global__ __launch_bounds__(kSelectThreads) void select_stage2_kernel(SelectArgs a) {
  constexpr int NT = kSelectThreads;
  __shared__ SelectShared sh;
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
  if (ITEMS > 0 && npre > NT * ITEMS) return;
  FillSource src = {a.scores + (int64_t)lz * a.T + s0, a.member + s0};
  select_wg<ITEMS>(sh, src, [&](int j, bool admitted, int pos) { if (admitted) out[pos] = j; }, npre, need);
}

// candidates kept in registers per thread, chosen from the longest request
static int items_for(const Plan& pl) {
  const int npre = pl.max_n - pl.W;
  for (int items : {8, 16, 32, 48, 64})
    if (npre <= kSelectThreads * items) return items;
  return 0;
}

#define CODECOMP_DISPATCH_ITEMS(KERNEL, GRID, ARGS)                                        \
  switch (items_for(pl)) {                                                                 \
    case 8: KERNEL<8><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;             \
    case 16: KERNEL<16><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;           \
    case 32: KERNEL<32><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;           \
    case 48: KERNEL<48><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;           \
    case 64: KERNEL<64><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;           \
    default: KERNEL<0><<<GRID, dim3(kSelectThreads), 0, stream>>>(ARGS); break;            \
  }

int launch_select(const Plan& pl, const float* scores, int32_t* idx, hipStream_t stream) {
  SelectArgs a = {};
  a.scores = scores; a.cu_seqlens = pl.cu_seqlens_dev; a.cu_budgets = pl.cu_budgets_dev; a.idx = idx;
  a.n_seqs = pl.n_seqs; a.T = pl.T; a.TB = pl.TB; a.W = pl.W;
  CODECOMP_DISPATCH_ITEMS(select_kernel, dim3(pl.n_seqs, pl.L * pl.Hkv), a)
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
  CODECOMP_DISPATCH_ITEMS(select_stage1_kernel, dim3(pl.n_seqs), a)
  if (hipError_t e = hipGetLastError()) return (int)e;
  CODECOMP_DISPATCH_ITEMS(select_stage2_kernel, dim3(pl.n_seqs, pl.L * pl.Hkv), a)
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

}  // namespace codecomp
