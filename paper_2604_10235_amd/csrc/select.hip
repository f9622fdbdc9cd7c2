// Select step: per (layer, KV head, request) keep the last W tokens and the B - W best-scored
// tokens of the prefix [0, N - W); equal scores go to the lower index; indices come out
// ascending ("retain the top-ranked context tokens ... up to the remaining chunk budget").
//
// One workgroup owns one problem.  An MSB-first radix select over order-preserving integer
// images of the float scores (digits of 11, 11 and 10 bits, LDS histogram) finds the score of
// the last admitted token and how many tokens tied at that score are admitted; one ordered
// pass (workgroup prefix sums of "greater" and "equal" flags) then writes the indices already
// sorted.  The score row (<= 512 KB) stays in L2 between passes.
#include "plan.h"

namespace codecomp {

struct SelectArgs {
  const float* scores;
  const int32_t* cu_seqlens;
  const int32_t* cu_budgets;
  int32_t* idx;
  int n_seqs, T, TB, W;
};

// Monotone map float -> uint32 (larger float <=> larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t order_key(float x) {
  x = x + 0.0f;   // -0 -> +0
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectArgs a) {
  constexpr int NT = kSelectThreads;
  constexpr int NWV = NT / 64;
  __shared__ unsigned int hist[2048];
  __shared__ unsigned int sh_prefix, sh_need;
  __shared__ int wave_gt[NWV], wave_eq[NWV];
  __shared__ int tile_gt, tile_eq;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
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

  // ---- radix select: key of the need-th largest candidate (digits of 11, 11, 10 bits, MSB first)
  uint32_t prefix = 0;                   // high bits fixed so far
  uint32_t remaining = (uint32_t)need;   // rank still to be located inside the current bucket
  const int npad = (npre + NT - 1) / NT * NT;   // uniform trip counts: every lane takes part in the ballots
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const int nbins = pass == 2 ? 1024 : 2048;
    for (int b = tid; b < nbins; b += NT) hist[b] = 0;
    __syncthreads();
    const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (pass == 1 ? 21 : 10));
    constexpr int UNR = 8;                // loads in flight per thread: the pass is latency bound otherwise
    for (int j0 = tid; j0 < npad; j0 += NT * UNR) {
      uint32_t keys[UNR];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int j = j0 + u * NT;
        keys[u] = j < npre ? order_key(sc[j]) : 0u;
      }
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const int j = j0 + u * NT;
        const uint32_t key = keys[u];
        const bool match = j < npre && (key & himask) == prefix;
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
            if (lane == leader) atomicAdd(&hist[lb], (unsigned int)__popcll(same));
            pend &= ~same;
          }
        }
        if ((pend >> lane) & 1ull) atomicAdd(&hist[bin], 1u);
      }
    }
    __syncthreads();
    if (wave == 0) {
      // lane owns bins [lane*per, lane*per+per); walk from the top bin down until `remaining` is covered
      const int per = nbins / 64;
      unsigned int mine = 0;
      for (int i = 0; i < per; ++i) mine += hist[lane * per + i];
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
          const unsigned int cnt = hist[lane * per + bin];
          if (acc + cnt >= remaining) break;
          acc += cnt;
        }
        sh_prefix = prefix | ((uint32_t)(lane * per + bin) << shift);
        sh_need = remaining - acc;       // rank inside the chosen bin
      }
    }
    __syncthreads();
    prefix = sh_prefix;
    remaining = sh_need;
  }
  const uint32_t tau = prefix;           // key of the last admitted candidate
  const int ties = (int)remaining;       // candidates with key == tau admitted (lowest indices first)

  // ---- ordered compaction
  int carry_gt = 0, carry_eq = 0;
  constexpr int PER = 4;
  for (int base = 0; base < npre; base += NT * PER) {
    const int j0 = base + tid * PER;
    int gt[PER], eq[PER];
    int ngt = 0, neq = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int j = j0 + e;
      uint32_t key = 0;
      const bool in = j < npre;
      if (in) key = order_key(sc[j]);
      gt[e] = in && key > tau;
      eq[e] = in && key == tau;
      ngt += gt[e]; neq += eq[e];
    }
    // exclusive scan over the workgroup of (ngt, neq)
    int sg = ngt, se = neq;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int og = __shfl_up(sg, off), oe = __shfl_up(se, off);
      if (lane >= off) { sg += og; se += oe; }
    }
    if (lane == 63) { wave_gt[wave] = sg; wave_eq[wave] = se; }
    __syncthreads();
    if (wave == 0) {
      int wg = lane < NWV ? wave_gt[lane] : 0, we = lane < NWV ? wave_eq[lane] : 0;
      int ig = wg, ie = we;
#pragma unroll
      for (int off = 1; off < NWV; off <<= 1) {
        const int og = __shfl_up(ig, off), oe = __shfl_up(ie, off);
        if (lane >= off) { ig += og; ie += oe; }
      }
      if (lane < NWV) { wave_gt[lane] = ig - wg; wave_eq[lane] = ie - we; }
      if (lane == NWV - 1) { tile_gt = ig; tile_eq = ie; }
    }
    __syncthreads();
    int pg = carry_gt + wave_gt[wave] + sg - ngt;     // "greater" candidates before this thread's first
    int pe = carry_eq + wave_eq[wave] + se - neq;     // "equal" candidates before it
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (gt[e]) out[pg + min(pe, ties)] = j0 + e;
      else if (eq[e] && pe < ties) out[pg + pe] = j0 + e;
      pg += gt[e]; pe += eq[e];
    }
    carry_gt += tile_gt;
    carry_eq += tile_eq;
    __syncthreads();                      // wave_* / tile_* are rewritten by the next tile
  }
}

int launch_select(const Plan& pl, const float* scores, int32_t* idx, hipStream_t stream) {
  SelectArgs a;
  a.scores = scores; a.cu_seqlens = pl.cu_seqlens_dev; a.cu_budgets = pl.cu_budgets_dev; a.idx = idx;
  a.n_seqs = pl.n_seqs; a.T = pl.T; a.TB = pl.TB; a.W = pl.W;
  select_kernel<<<dim3(pl.n_seqs, pl.L * pl.Hkv), dim3(kSelectThreads), 0, stream>>>(a);
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

}  // namespace codecomp
