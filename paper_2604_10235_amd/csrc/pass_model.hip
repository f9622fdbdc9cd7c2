// libcodecomp_peaks, second measurement: a synthetic loop with the structure of the score passes (score_pass.h) whose
// features are switched on one by one, to show where a pass loses time against its bare instruction mix.  512 threads
// (eight waves, two per SIMD), two row blocks of 32 rows per wave, 64-key tiles, accumulators in VGPRs; per MFMA two
// logits per lane of (fma, exp2, add).  Results mean nothing; only the time counts.  Not part of the hot path and not
// from the paper.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "codecomp_peaks.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define BC(a) __builtin_bit_cast(bf16x8, a)

constexpr int kModelThreads = 512;
constexpr int kRing = 1, kStage = 2, kLoads = 4, kUneven = 8, kDirect = 16;   // feature bits

// FLAGS: kRing    K fragments come from LDS through a four-entry register ring, one workgroup barrier per tile;
//        kStage   every thread parks 32 bytes per tile in the other LDS buffer (the next tile);
//        kLoads   those bytes come from global memory (16 KB per tile and workgroup, streamed from a region of
//                 `big` of the workgroup's own), asked for NSETS tiles before they are parked;
//        kUneven  waves 4..7 (the second wave of every SIMD) skip their second row block in the second half of
//                 every tile: three (block, half-tile) units against four, as with 14 row blocks over eight waves;
//        kDirect  (instead of kStage | kLoads) the 16 KB of a tile go from global memory straight into LDS
//                 (global_load_lds_dwordx4: lane i's 16 bytes land at base + 16 i, so rows cannot be padded; the
//                 16-byte pieces of a row are XOR-swizzled with the row number instead), into a ring of four tile
//                 buffers, NSETS tiles ahead of their use; no staging registers, no LDS stores.
template <int FLAGS, int NSETS>
__global__ __launch_bounds__(kModelThreads, 2) void pass_model_kernel(const u32x4* __restrict__ rnd, const u32x4* __restrict__ big,
                                                                      size_t big_n16, float* out, long long* clk, int tiles) {
  constexpr int NT = kModelThreads;
  constexpr bool DIRECT = (FLAGS & kDirect) != 0;
  constexpr int ROW = DIRECT ? 16 : 17;             // 16-byte pieces per key row in LDS (272-byte rows, or 256 swizzled)
  constexpr int NBUF = DIRECT ? (NSETS > 3 ? 8 : 4) : 2;      // LDS tile buffers (128 KB with eight: dynamic shared memory)
  extern __shared__ u32x4 tile_mem[];
  u32x4 (*tile)[64 * ROW] = reinterpret_cast<u32x4 (*)[64 * ROW]>(tile_mem);
  u32x4 q[2][8], ring[4], stage[4][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hf = lane >> 5;
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) q[s][i] = rnd[((s * 8 + i) * NT + tid + 29 * s) & 4095];   // the two blocks differ (equal ones would be merged)
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int i = 0; i < 2; ++i) stage[k][i] = rnd[(i * NT + tid + 33 * k + 7) & 4095];
  for (int i = tid; i < NBUF * 64 * ROW; i += NT) (&tile[0][0])[i] = rnd[i & 4095];
  __syncthreads();
  // where this lane finds the fragment of k-step ks inside a 32-key half tile (in 16-byte pieces)
  int frag_at[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) frag_at[ks] = DIRECT ? l32 * 16 + ((2 * ks + hf) ^ (l32 & 7)) : l32 * 17 + hf + ks * 2;
#pragma unroll
  for (int i = 0; i < 4; ++i) ring[i] = tile[0][frag_at[i]];
  f32x16 accA[2], accB[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) { accA[s] = f32x16{0}; accB[s] = f32x16{0}; }
  float nl[2][16];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int v = 0; v < 16; ++v) nl[s][v] = -30.f - v * 0.3f - s;
  float tot = 0.f;
  const float c = 0.1275f;
  const f32x16 zero = {0};
  const size_t per_wg = big_n16 / gridDim.x;        // >= 2 * NT (checked by the host)
  const u32x4* src = big + (size_t)blockIdx.x * per_wg;
  size_t pos = 0;
  const long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  auto body = [&](auto light_t) __attribute__((always_inline)) {
    constexpr bool LIGHT = decltype(light_t)::value;
    auto one_tile = [&](int t, u32x4 (&stg)[2]) __attribute__((always_inline)) {
      const int buf = t & (NBUF - 1);
      auto phase = [&](auto ph_t) __attribute__((always_inline)) {
        constexpr int ph = decltype(ph_t)::value;
        f32x16* nn = ph == 0 ? accA : accB;
        const f32x16* pp = ph == 0 ? accB : accA;
        constexpr bool s1_new = !(LIGHT && ph == 1);      // the second row block computes this half tile
        constexpr bool s1_old = !(LIGHT && ph == 0);      // ... has logits of the previous half tile to consume
        constexpr int PER = s1_old ? 2 : 1;               // logits per gap (one gap after every MFMA position)
        float sum0 = 0.f, sum1 = 0.f;
        if (ph == 0 && DIRECT) {
          // tile t + NSETS: this thread's two pieces, the global piece chosen so that it lands swizzled
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const int chunk = wave * 2 + i;                          // 4 key rows = 64 pieces = one instruction of a wave
            const int r = 4 * chunk + (lane >> 4);
            const u32x4* from = src + pos + r * 16 + ((lane & 15) ^ (r & 7));
            const unsigned to = (unsigned)(size_t)(&tile[(t + NSETS) & (NBUF - 1)][chunk * 64]);   // LDS byte address, the same in every lane
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(__builtin_amdgcn_readfirstlane(to)), "v"(from) : "memory", "m0");
          }
          pos += 2 * NT;
          if (pos + 2 * NT > per_wg) pos = 0;
        }
        if (ph == 0 && !DIRECT) {
          if (FLAGS & kStage) {
#pragma unroll
            for (int i = 0; i < 2; ++i) { const int cidx = tid + i * NT; tile[buf ^ 1][(cidx >> 4) * 17 + (cidx & 15)] = stg[i]; }
          }
          if (FLAGS & kLoads) {
#pragma unroll
            for (int i = 0; i < 2; ++i) stg[i] = src[pos + tid + i * NT];      // pos + 2 * NT <= per_wg
            pos += 2 * NT;
            if (pos + 2 * NT > per_wg) pos = 0;
          }
        }
        auto soft = [&](int gap) __attribute__((always_inline)) {
#pragma unroll
          for (int u = 0; u < PER; ++u) {
            const int e = gap * PER + u;
            if (s1_old) {
              if (e & 1) sum1 += __builtin_amdgcn_exp2f(__builtin_fmaf(pp[1][e >> 1], c, nl[1][e >> 1]));
              else sum0 += __builtin_amdgcn_exp2f(__builtin_fmaf(pp[0][e >> 1], c, nl[0][e >> 1]));
            } else {
              sum0 += __builtin_amdgcn_exp2f(__builtin_fmaf(pp[0][e], c, nl[0][e]));
            }
          }
        };
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          if ((FLAGS & kRing) && ph == 1 && ks == 4) {
            // tile t + 1 must be whole: its two loads of this thread are the oldest of 2 * NSETS in flight
            if (DIRECT) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * (NSETS - 1)) : "memory");
            else asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
          }
          nn[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(BC(q[0][ks]), BC(ring[ks & 3]), ks == 0 ? zero : nn[0], 0, 0, 0);
          soft(2 * ks);
          if (s1_new) nn[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(BC(q[1][ks]), BC(ring[ks & 3]), ks == 0 ? zero : nn[1], 0, 0, 0);
          if (FLAGS & kRing) {
            const int from_buf = (ks + 4 < 8 || ph == 0) ? buf : (buf + 1) & (NBUF - 1);
            ring[ks & 3] = tile[from_buf][(ph ^ (ks + 4 >= 8)) * 32 * ROW + frag_at[(ks + 4) & 7]];
          }
          soft(2 * ks + 1);
        }
#pragma unroll
        for (int m = 0; m < 16; ++m) {
          if (!(m & 1) || s1_new) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if ((FLAGS & kRing) && (m & 1)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);
          __builtin_amdgcn_sched_group_barrier(0x400, PER, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, PER, 0);
        }
        tot += sum0 + sum1;
      };
      phase(std::integral_constant<int, 0>{});
      phase(std::integral_constant<int, 1>{});
    };
    // register set t % NSETS holds tile t + 1 and is refilled for tile t + 1 + NSETS (tiles is a multiple of 12)
    if constexpr (NSETS == 2) { for (int t = 0; t < tiles; t += 2) { one_tile(t, stage[0]); one_tile(t + 1, stage[1]); } }
    else if constexpr (NSETS == 3) { for (int t = 0; t < tiles; t += 3) { one_tile(t, stage[0]); one_tile(t + 1, stage[1]); one_tile(t + 2, stage[2]); } }
    else { for (int t = 0; t < tiles; t += 4) { one_tile(t, stage[0]); one_tile(t + 1, stage[1]); one_tile(t + 2, stage[2]); one_tile(t + 3, stage[3]); } }   // also the direct variants further ahead (no register sets)
  };
  if ((FLAGS & kUneven) && wave >= 4) body(std::true_type{}); else body(std::false_type{});
  if (DIRECT) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // no load into LDS is left in flight when the wave ends
  const long long c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
  float s = tot;
#pragma unroll
  for (int k = 0; k < 4; ++k) s += __builtin_bit_cast(float, stage[k][0].x) + __builtin_bit_cast(float, stage[k][1].y);
#pragma unroll
  for (int i = 0; i < 2; ++i) s += accA[i][0] + accB[i][5];
  if (s == 12345.678f) out[0] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) { clk[0] = c1 - c0; clk[1] = r1 - r0; }
}

template <int FLAGS, int NSETS>
int run_variant(const u32x4* rnd, const u32x4* big, size_t big_n16, float* sink, long long* clk, int cus, hipStream_t s,
                hipEvent_t e0, hipEvent_t e1, codecomp_pass_model_row* row) {
  constexpr int tiles = 3000;                       // a multiple of 12; ~5 ms
  int occ = 0;
  hipError_t e;
  constexpr bool DIRECT = (FLAGS & kDirect) != 0;
  constexpr size_t lds = (size_t)(DIRECT ? (NSETS > 3 ? 8 : 4) : 2) * 64 * (DIRECT ? 16 : 17) * sizeof(u32x4);   // as in the kernel
  if (lds > 65536 && (e = hipFuncSetAttribute(reinterpret_cast<const void*>(pass_model_kernel<FLAGS, NSETS>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds))) return (int)e;
  if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, pass_model_kernel<FLAGS, NSETS>, kModelThreads, lds))) return (int)e;
  if (occ < 1) return -2;
  const int g = cus;                                // one workgroup per compute unit, as the eight-wave passes
  pass_model_kernel<FLAGS, NSETS><<<g, kModelThreads, lds, s>>>(rnd, big, big_n16, sink, clk, tiles);   // warm-up
  if ((e = hipEventRecord(e0, s))) return (int)e;
  pass_model_kernel<FLAGS, NSETS><<<g, kModelThreads, lds, s>>>(rnd, big, big_n16, sink, clk, tiles);
  if ((e = hipEventRecord(e1, s)) || (e = hipEventSynchronize(e1)) || (e = hipGetLastError())) return (int)e;
  float ms = 0.f;
  if ((e = hipEventElapsedTime(&ms, e0, e1))) return (int)e;
  long long cyc[2] = {0, 0};
  if ((e = hipMemcpyAsync(cyc, clk, 16, hipMemcpyDeviceToHost, s)) || (e = hipStreamSynchronize(s))) return (int)e;
  const double units = (FLAGS & kUneven) ? 3.5 : 4.0;                     // (block, half tile) units per wave and tile
  const double mfmas_per_simd = (double)tiles * 8.0 * units * 2.0;        // two waves per SIMD
  const double clock_hz = cyc[1] > 0 ? (double)cyc[0] / ((double)cyc[1] * 1e-8) : 0.0;
  row->features = FLAGS;
  row->tiles_ahead = (FLAGS & (kLoads | kDirect)) ? NSETS : 0;
  row->logits_per_s = mfmas_per_simd * 4.0 * cus * 128.0 / (ms * 1e-3);
  row->clock_mhz = clock_hz / 1e6;
  row->cycles_per_mfma = ms * 1e-3 * clock_hz / mfmas_per_simd;
  row->hbm_gbs = (FLAGS & (kLoads | kDirect)) ? (double)g * tiles * 16384.0 / (ms * 1e-3) / 1e9 : 0.0;
  return 0;
}

}  // namespace

extern "C" int codecomp_measure_pass_model(const void* rnd, const void* big, size_t big_bytes, void* small,
                                           codecomp_pass_model* out, void* hip_stream) {
  if (!rnd || !big || !small || !out || (big_bytes & 15)) return -1;
  hipStream_t s = (hipStream_t)hip_stream;
  int dev = 0, cus = 0;
  hipError_t e;
  if ((e = hipGetDevice(&dev)) || (e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev))) return out->status = (int)e;
  // every workgroup streams through a region of its own of at least two loads per thread
  if (cus < 1 || big_bytes / 16 / (size_t)cus < 2 * (size_t)kModelThreads) return out->status = -1;
  hipEvent_t e0, e1;
  if ((e = hipEventCreate(&e0)) || (e = hipEventCreate(&e1))) return out->status = (int)e;
  float* sink = static_cast<float*>(small);
  long long* clk = reinterpret_cast<long long*>(static_cast<char*>(small) + 32);
  const u32x4* r = static_cast<const u32x4*>(rnd);
  const u32x4* b = static_cast<const u32x4*>(big);
  const size_t n16 = big_bytes / 16;
  int rc = 0, i = 0;
  out->compute_units = cus;
  if ((rc = run_variant<kRing, 2>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kStage, 2>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kStage | kLoads, 2>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kStage | kLoads, 3>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kStage | kLoads, 4>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kStage | kLoads | kUneven, 2>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kStage | kLoads | kUneven, 4>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kLoads, 2>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kDirect, 2>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kDirect, 3>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kDirect, 6>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
  if ((rc = run_variant<kRing | kDirect | kUneven, 6>(r, b, n16, sink, clk, cus, s, e0, e1, &out->rows[i++]))) goto done;
done:
  out->n_rows = i;
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  return out->status = rc;
}
