// Select step: per (layer, KV head, request) keep the last W tokens and the B - W best tokens
// of the prefix [0, N - W); equal scores go to the lower index; indices come out ascending
// ("retain the top-ranked context tokens ... up to the remaining chunk budget").
//
// One workgroup owns one problem.  An MSB-first radix select over order-preserving integer
// images of the float scores (digits of 11, 11 and 10 bits, LDS histogram) finds the score of
// the last admitted token and how many tokens tied at that score are admitted; one ordered
// pass (workgroup prefix sums of "sure" and "tied" flags) then writes the indices already
// sorted.  The score row (<= 512 KB) stays in L2 between passes.
//
// Two selection rules share these pieces:
//   additive   : one selection on c = pooled attention + lambda * prior (the score kernel's output);
//   two-stage  : the paper's literal order - structure first, attention fills the rest
//                (sections "Span-Level Structural Protection" and "Attention-based KV Cache
//                Compression"): stage 1 keeps up to B_span = min(Bp, max(B_min, floor(rho * Bp)))
//                prefix tokens with prior > 0, largest prior first (ties: first in sequence, which for a
//                binary prior is "the first tokens of P"), Bp = B - W; stage 2 fills the remaining
//                Bp - |P| slots with the best pooled-attention tokens not in P.
#include "plan.h"

namespace codecomp {

// Monotone map float -> uint32 (larger float <=> larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t order_key(float x) {
  x = x + 0.0f;   // -0 -> +0
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct SelectShared {
  unsigned int hist[2048];
  unsigned int prefix, need;
  int wave_sure[kSelectThreads / 64], wave_tie[kSelectThreads / 64];
  int tile_sure, tile_tie;
};

// Key of the `need`-th largest candidate among j in [0, npre) with key_at(j, key) == true, and how many
// candidates equal to it are admitted.  Requires 1 <= need <= number of candidates.  All threads call it.
template <class KeyAt>
__device__ __forceinline__ void radix_select_wg(SelectShared& sh, KeyAt key_at, int npre, int need, uint32_t& tau,
                                                int& ties) {
  constexpr int NT = kSelectThreads;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t prefix = 0;                   // high bits fixed so far
  uint32_t remaining = (uint32_t)need;   // rank still to be located inside the current bucket
  const int npad = (npre + NT - 1) / NT * NT;   // uniform trip counts: every lane takes part in the ballots
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const int nbins = pass == 2 ? 1024 : 2048;
    for (int b = tid; b < nbins; b += NT) sh.hist[b] = 0;
    __syncthreads();
    const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (pass == 1 ? 21 : 10));
    constexpr int UNR = 8;                // loads in flight per thread: the pass is latency bound otherwise
    for (int j0 = tid; j0 < npad; j0 += NT * UNR) {
      uint32_t keys[UNR];
      bool valid[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int j = j0 + u * NT;
        keys[u] = 0u;
        valid[u] = j < npre && key_at(j, keys[u]);
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const uint32_t key = keys[u];
        const bool match = valid[u] && (key & himask) == prefix;
        const uint32_t bin = (key >> shift) & (uint32_t)(nbins - 1);
        // score distributions are concentrated: lanes that share a bin are counted with one atomic
        // (two rounds of leader election), whatever is left falls back to one atomic per lane
        unsigned long long pend = __ballot(match);
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          if (pend != 0) {
            const int leader = __ffsll(pend) - 1;
            const uint32_t lb = __shfl(bin, leader);
            const unsigned long long same = __ballot(match && bin == lb) & pend;
            if (lane == leader) atomicAdd(&sh.hist[lb], (unsigned int)__popcll(same));
            pend &= ~same;
          }
        }
        if ((pend >> lane) & 1ull) atomicAdd(&sh.hist[bin], 1u);
      }
    }
    __syncthreads();
    if (wave == 0) {
      // lane owns bins [lane*per, lane*per+per); walk from the top bin down until `remaining` is covered
      const int per = nbins / 64;
      unsigned int mine = 0;
      for (int i = 0; i < per; ++i) mine += sh.hist[lane * per + i];
      unsigned int run = mine;           // inclusive suffix sum over lanes
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const unsigned int o = __shfl_down(run, off);
        if (lane + off < 64) run += o;
      }
      const unsigned int above = run - mine;   // count in bins owned by higher lanes
      if (above < remaining && remaining <= above + mine) {   // exactly one lane
        unsigned int acc = above;
        int bin = per - 1;
        for (; bin > 0; --bin) {
          const unsigned int cnt = sh.hist[lane * per + bin];
          if (acc + cnt >= remaining) break;
          acc += cnt;
        }
        sh.prefix = prefix | ((uint32_t)(lane * per + bin) << shift);
        sh.need = remaining - acc;       // rank inside the chosen bin
      }
    }
    __syncthreads();
    prefix = sh.prefix;
    remaining = sh.need;
  }
  tau = prefix;
  ties = (int)remaining;
}

// Ordered pass over j in [0, npre): classify(j) returns 2 (admitted for sure), 1 (tied at the cut: admitted
// while fewer than `ties` tied candidates precede it) or 0.  emit(j, admitted, pos) is called for every j
// with pos = number of admitted candidates before j.  All threads call it.
template <class Classify, class Emit>
__device__ __forceinline__ void ordered_pass_wg(SelectShared& sh, Classify classify, Emit emit, int npre, int ties) {
  constexpr int NT = kSelectThreads;
  constexpr int NWV = NT / 64;
  constexpr int PER = 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int carry_sure = 0, carry_tie = 0;
  for (int base = 0; base < npre; base += NT * PER) {
    const int j0 = base + tid * PER;
    int cls[PER];
    int nsure = 0, ntie = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int j = j0 + e;
      cls[e] = j < npre ? classify(j) : 0;
      nsure += cls[e] == 2; ntie += cls[e] == 1;
    }
    // exclusive scan over the workgroup of (nsure, ntie)
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
    int ps = carry_sure + sh.wave_sure[wave] + ss - nsure;   // sure candidates before this thread's first
    int pt = carry_tie + sh.wave_tie[wave] + st - ntie;      // tied candidates before it
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int j = j0 + e;
      if (j < npre) {
        const bool admitted = cls[e] == 2 || (cls[e] == 1 && pt < ties);
        emit(j, admitted, ps + min(pt, ties));
      }
      ps += cls[e] == 2; pt += cls[e] == 1;
    }
    carry_sure += sh.tile_sure;
    carry_tie += sh.tile_tie;
    __syncthreads();                      // wave_* / tile_* are rewritten by the next tile
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

// additive rule: one selection on the fused scores
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
  const float* sc = a.scores + (int64_t)lz * a.T + s0;
  int32_t* out = a.idx + (int64_t)lz * a.TB + o0;

  // the observation window is always kept
  for (int t = tid; t < a.W; t += NT) out[need + t] = npre + t;
  if (need <= 0) return;                 // uniform
  if (need >= npre) {                    // everything is kept
    for (int j = tid; j < npre; j += NT) out[j] = j;
    return;
  }
  uint32_t tau; int ties;
  radix_select_wg(sh, [&](int j, uint32_t& key) { key = order_key(sc[j]); return true; }, npre, need, tau, ties);
  ordered_pass_wg(sh,
                  [&](int j) { const uint32_t key = order_key(sc[j]); return key > tau ? 2 : (key == tau ? 1 : 0); },
                  [&](int j, bool admitted, int pos) { if (admitted) out[pos] = j; }, npre, ties);
}

// two-stage rule, stage 1: once per request (the prior is shared by layers and heads)
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
  if (need <= 0) {
    for (int j = tid; j < npre; j += NT) member[j] = 0;
    return;
  }
  uint32_t tau; int ties;
  radix_select_wg(sh, [&](int j, uint32_t& key) { const float x = p[j]; key = order_key(x); return x > 0.f; }, npre,
                  need, tau, ties);
  ordered_pass_wg(sh,
                  [&](int j) {
                    const float x = p[j];
                    if (!(x > 0.f)) return 0;
                    const uint32_t key = order_key(x);
                    return key > tau ? 2 : (key == tau ? 1 : 0);
                  },
                  [&](int j, bool admitted, int) { member[j] = admitted ? 1 : 0; }, npre, ties);
}

// two-stage rule, stage 2: attention fills what stage 1 left
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
  const float* sc = a.scores + (int64_t)lz * a.T + s0;
  const uint8_t* member = a.member + s0;
  int32_t* out = a.idx + (int64_t)lz * a.TB + o0;

  for (int t = tid; t < a.W; t += NT) out[bp + t] = npre + t;
  if (bp <= 0) return;
  if (bp >= npre) {
    for (int j = tid; j < npre; j += NT) out[j] = j;
    return;
  }
  uint32_t tau = 0xFFFFFFFFu; int ties = 0;    // need == 0: nothing beyond stage 1 is admitted
  if (need > 0)
    radix_select_wg(sh, [&](int j, uint32_t& key) { key = order_key(sc[j]); return member[j] == 0; }, npre, need, tau,
                    ties);
  ordered_pass_wg(sh,
                  [&](int j) {
                    if (member[j]) return 2;
                    if (need <= 0) return 0;
                    const uint32_t key = order_key(sc[j]);
                    return key > tau ? 2 : (key == tau ? 1 : 0);
                  },
                  [&](int j, bool admitted, int pos) { if (admitted) out[pos] = j; }, npre, ties);
}

int launch_select(const Plan& pl, const float* scores, int32_t* idx, hipStream_t stream) {
  SelectArgs a = {};
  a.scores = scores; a.cu_seqlens = pl.cu_seqlens_dev; a.cu_budgets = pl.cu_budgets_dev; a.idx = idx;
  a.n_seqs = pl.n_seqs; a.T = pl.T; a.TB = pl.TB; a.W = pl.W;
  select_kernel<<<dim3(pl.n_seqs, pl.L * pl.Hkv), dim3(kSelectThreads), 0, stream>>>(a);
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
  select_stage1_kernel<<<dim3(pl.n_seqs), dim3(kSelectThreads), 0, stream>>>(a);
  if (hipError_t e = hipGetLastError()) return (int)e;
  select_stage2_kernel<<<dim3(pl.n_seqs, pl.L * pl.Hkv), dim3(kSelectThreads), 0, stream>>>(a);
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

}  // namespace codecomp
