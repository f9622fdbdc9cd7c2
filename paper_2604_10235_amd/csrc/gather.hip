// Gather step: copy the retained K and V rows into the compact per-layer cache (the
// compressed chunk of section "Position Encoding": rows keep their original order).
// Pure data movement: a row of d elements (bf16, or one-byte FP8 codes) is moved as 16-byte pieces
// by consecutive lanes, so both the reads and the writes of a row are one contiguous segment.
#include "plan.h"

namespace codecomp {

struct GatherArgs {
  const unsigned char* k;
  const unsigned char* v;
  const int32_t* idx;
  const int32_t* cu_seqlens;
  const int32_t* cu_budgets;
  unsigned char* k_out;
  unsigned char* v_out;
  int n_seqs, Hkv, TB, pieces_log2;    // 16-byte pieces per row = d * element size / 16 (4, 8 or 16)
  int64_t kv_sl, kv_sh, kv_st, o_sl, o_sh, o_st;     // in bytes
};

constexpr int kGatherThreads = 256;
constexpr int kGatherRowsPerThread = 2;     // rows of K and of V a thread has in flight
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 ld16(const unsigned char* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ void st16(unsigned char* p, u32x4 v) { *reinterpret_cast<u32x4*>(p) = v; }

__global__ __launch_bounds__(kGatherThreads) void gather_kernel(GatherArgs a) {
  const int pieces = 1 << a.pieces_log2;
  const int rows_per_pass = kGatherThreads >> a.pieces_log2;
  const int piece = threadIdx.x & (pieces - 1);
  const int rsub = threadIdx.x >> a.pieces_log2;
  const int lz = blockIdx.y;
  const int layer = lz / a.Hkv, head = lz - layer * a.Hkv;
  const int32_t* idx = a.idx + (int64_t)lz * a.TB;
  const unsigned char* kb = a.k + layer * a.kv_sl + head * a.kv_sh;
  const unsigned char* vb = a.v + layer * a.kv_sl + head * a.kv_sh;
  unsigned char* ko = a.k_out + layer * a.o_sl + head * a.o_sh;
  unsigned char* vo = a.v_out + layer * a.o_sl + head * a.o_sh;
  const int first_slot = blockIdx.x * rows_per_pass * kGatherRowsPerThread;
  const int slot0 = first_slot + rsub;

  // Request that owns the workgroup's first output slot: a 256-way search by the whole workgroup (thread t
  // probes the t-th of 256 evenly spaced candidates; the probes that are not beyond the slot form a prefix),
  // one round per factor of 256 in n_seqs instead of one dependent load per factor of 2.  The rows of the
  // workgroup then walk forward from there (they lie within a few dozen slots of the first).
  int r_first = 0;
  for (int span = a.n_seqs; span > 1;) {
    const int step = (span + kGatherThreads - 1) / kGatherThreads;
    const int r = r_first + (int)threadIdx.x * step;
    const int hits = __syncthreads_count(r < r_first + span && a.cu_budgets[r] <= first_slot);   // >= 1: cu_budgets[r_first] <= first_slot
    const int next = r_first + (hits - 1) * step;
    span = min(step, r_first + span - next);
    r_first = next;
  }

  u32x4 kv[kGatherRowsPerThread], vv[kGatherRowsPerThread];
#pragma unroll
  for (int i = 0; i < kGatherRowsPerThread; ++i) {
    const int slot = slot0 + i * rows_per_pass;
    if (slot < a.TB) {
      int lo = r_first;                   // request owning this output slot
      while (lo + 1 < a.n_seqs && a.cu_budgets[lo + 1] <= slot) ++lo;
      // indices are clamped into the request so that a corrupt idx can never read out of bounds
      const int s0 = a.cu_seqlens[lo], n = a.cu_seqlens[lo + 1] - s0;
      const int64_t tok = (int64_t)s0 + min(max(idx[slot], 0), n - 1);
      kv[i] = ld16(kb + tok * a.kv_st + piece * 16);
      vv[i] = ld16(vb + tok * a.kv_st + piece * 16);
    }
  }
#pragma unroll
  for (int i = 0; i < kGatherRowsPerThread; ++i) {
    const int slot = slot0 + i * rows_per_pass;
    if (slot < a.TB) {
      st16(ko + (int64_t)slot * a.o_st + piece * 16, kv[i]);
      st16(vo + (int64_t)slot * a.o_st + piece * 16, vv[i]);
    }
  }
}

int launch_gather(const Plan& pl, const void* k, const void* v, const int32_t* idx, void* k_out, void* v_out,
                  hipStream_t stream) {
  GatherArgs a;
  a.k = static_cast<const unsigned char*>(k); a.v = static_cast<const unsigned char*>(v); a.idx = idx;
  a.cu_seqlens = pl.cu_seqlens_dev; a.cu_budgets = pl.cu_budgets_dev;
  a.k_out = static_cast<unsigned char*>(k_out); a.v_out = static_cast<unsigned char*>(v_out);
  const int esz = pl.kv_fp8 ? 1 : 2;
  a.n_seqs = pl.n_seqs; a.Hkv = pl.Hkv; a.TB = pl.TB;
  a.pieces_log2 = (pl.d == 128 ? 4 : 3) - (pl.kv_fp8 ? 1 : 0);
  a.kv_sl = pl.kv_sl * esz; a.kv_sh = pl.kv_sh * esz; a.kv_st = pl.kv_st * esz;
  a.o_sl = pl.o_sl * esz; a.o_sh = pl.o_sh * esz; a.o_st = pl.o_st * esz;
  const int rows_per_block = (kGatherThreads >> a.pieces_log2) * kGatherRowsPerThread;
  gather_kernel<<<dim3((pl.TB + rows_per_block - 1) / rows_per_block, pl.L * pl.Hkv), dim3(kGatherThreads), 0,
                  stream>>>(a);
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

}  // namespace codecomp
