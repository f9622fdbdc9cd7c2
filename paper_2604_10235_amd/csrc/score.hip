// Score step, small kernels and entry: row merge between the two MFMA passes, pooling + prior, and the
// launch sequence.  The passes themselves live in score_pass.h and are instantiated per (head_dim, key
// type) in score_pass_*.hip.
#include "score_pass.h"

namespace codecomp {

extern template int dispatch_waves<128, false>(const Plan&, const ScoreArgs&, hipStream_t, unsigned);
extern template int dispatch_waves<128, true>(const Plan&, const ScoreArgs&, hipStream_t, unsigned);
extern template int dispatch_waves<64, false>(const Plan&, const ScoreArgs&, hipStream_t, unsigned);
extern template int dispatch_waves<64, true>(const Plan&, const ScoreArgs&, hipStream_t, unsigned);

// One thread per (layer*head, request, row): log2-sum-exp over the segments (of the teams) that cover the request and
// over the (at most two) wave slots that hold a share of the row's keys.
__global__ __launch_bounds__(256) void score_merge_kernel(ScoreArgs a) {
  __shared__ int part[256 / 64];
  const int seq = blockIdx.y;
  const int lz = blockIdx.z;
  // positions of the earlier requests in a problem's sequence: summed by the whole workgroup
  int mine = 0;
  for (int r = threadIdx.x; r < seq; r += 256)
    mine += a.lead + (a.cu_seqlens[r + 1] - a.cu_seqlens[r] - a.key_trim + kTileKeys - 1) / kTileKeys;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mine;
  __syncthreads();
  const int tile_off = a.lead + part[0] + part[1] + part[2] + part[3];
  // a launch with many problems has one workgroup per problem (the rows in turns), else one per 256 rows
  for (int row = blockIdx.x * blockDim.x + threadIdx.x; row < a.lrows; row += gridDim.x * blockDim.x) {
  const int split = row / (a.nb * 32);
  const int rb = (row - split * a.nb * 32) >> 5;
  const int nt = (a.cu_seqlens[seq + 1] - a.cu_seqlens[seq] - a.key_trim + kTileKeys - 1) / kTileKeys;
  if (nt == 0) {                           // no key to attend to: nothing reads this normaliser
    a.lse[((int64_t)lz * a.n_seqs + seq) * a.lrows + row] = 0.f;
    continue;
  }
  const int x0 = lz * a.tiles_per_problem + tile_off;
  const int g0 = wg_of_tile(x0, a.total_tiles, a.stat_teams), g1 = wg_of_tile(x0 + nt - 1, a.total_tiles, a.stat_teams);
  const int p = lz * a.n_seqs + seq;
  float M = NEG_BIG, L = 0.f;
  for (int h = 0; h < 2; ++h) {
    const int holder = a.rb_holder[rb][h];
    if (holder == 255) continue;
    // the segment of team g in this problem and row split sits in slot (g + p) * row_splits + split
    const float* sh = a.stats + (((int64_t)p * a.row_splits + split) * a.srows + holder * 32 + (row & 31)) * 2;
    for (int g = g0; g <= g1; ++g) {
      const int64_t at = (int64_t)g * a.row_splits * a.srows * 2;
      const float m = sh[at], l = sh[at + 1];
      const float Mn = fmaxf(M, m);
      L = L * __builtin_amdgcn_exp2f(M - Mn) + l * __builtin_amdgcn_exp2f(m - Mn);
      M = Mn;
    }
  }
  a.lse[((int64_t)lz * a.n_seqs + seq) * a.lrows + row] = M + log2f(L);
  }
}

struct FinishArgs {
  const float* uraw;
  const float* prior;
  const int32_t* cu_seqlens;
  float* scores;
  int n_seqs, T, LH, row_splits, pool;
  int mass_trim;      // window positions at the end of every request that hold no attention mass (prefix-only softmax)
  int pool_trim;      // window positions at the end of every request that pooling leaves out (prefix-only pooling)
  int pool_max;       // 1: max pooling
  float lambda, inv_pool;
};

constexpr int kFinishTile = 2048;     // tokens per workgroup of the finish kernel (one round of workgroups at the bench size)
constexpr int kFinishHalo = 512;      // largest supported (pool_kernel - 1) / 2

__device__ __forceinline__ int request_of(const int32_t* cu, int n_seqs, int j) {
  int lo = 0, hi = n_seqs;              // cu[lo] <= j < cu[lo+1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= j) lo = mid; else hi = mid;
  }
  return lo;
}

// scores[lz][j] = pool_{|delta| <= (k-1)/2, inside the request (or its prefix)} u[lz][j+delta] + lambda * prior[j],
// pool = sum / k (zero padding, divisor always k) or max.
// One workgroup stages its tokens of u (+ halo, row splits added) in LDS; every output is a direct sum.
// Everything that comes from memory (request bounds, prior, u) is asked for before the one barrier, so
// that a workgroup pays one memory round trip.  A tile that lies inside one request (the common case)
// takes that request's bounds once; otherwise every token looks its request up.
__global__ __launch_bounds__(256) void score_finish_kernel(FinishArgs a) {
  constexpr int PER = kFinishTile / 256;
  __shared__ float tile[kFinishTile + 2 * kFinishHalo];
  const int tid = threadIdx.x;
  const int lz = blockIdx.y;
  const int base = blockIdx.x * kFinishTile;
  const int half = (a.pool - 1) >> 1;
  const int last = min(base + kFinishTile, a.T) - 1;
  const int r_first = request_of(a.cu_seqlens, a.n_seqs, base), r_last = request_of(a.cu_seqlens, a.n_seqs, last);
  const bool one_request = r_first == r_last;
  int lo_[PER], hi_[PER];               // request bounds [lo, hi) of each of this thread's tokens
  float pr[PER];
  // A tile that meets fewer than 64 requests: every wave takes their upper bounds into one register (lane q: request
  // r_first + q) and each token counts the bounds at or below it - one load per wave instead of a binary search per token.
  const bool few_requests = !one_request && r_last - r_first < 64;
  const int bound = few_requests ? a.cu_seqlens[min(r_first + 1 + (tid & 63), a.n_seqs)] : 0;
  const int first_lo = a.cu_seqlens[r_first];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int j = base + e * 256 + tid;
    if (few_requests) {
      int k = 0;                          // requests of the tile that end at or before token j
      if (j < a.T)
        for (int q = 0; q < r_last - r_first; ++q) k += j >= __builtin_amdgcn_readlane(bound, q);
      hi_[e] = __shfl(bound, k);
      const int below = __shfl(bound, max(k - 1, 0));       // every lane takes part: a lane reads from lanes that are not in its request
      lo_[e] = k == 0 ? first_lo : below;
    } else {
      const int r = one_request || j >= a.T ? r_first : request_of(a.cu_seqlens, a.n_seqs, j);
      lo_[e] = a.cu_seqlens[r]; hi_[e] = a.cu_seqlens[r + 1];
    }
    pr[e] = j < a.T ? a.prior[j] : 0.f;
  }
  // the tile's own tokens: PER independent loads per thread (per row split), all in flight together
  float body[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) body[e] = 0.f;
  for (int sp = 0; sp < a.row_splits; ++sp) {
    const float* u = a.uraw + ((int64_t)sp * a.LH + lz) * a.T;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int j = base + e * 256 + tid;
      // the load does not wait for the request bounds (clamped: always in bounds); window positions were never
      // written by the mass pass when the softmax leaves them out, whatever they hold is dropped
      const float val = u[min(j, a.T - 1)];
      body[e] += j < min(a.T, hi_[e] - a.mass_trim) ? val : 0.f;
    }
  }
  // the halo on both sides: 2 * half tokens that belong to the neighbouring tiles
  for (int i = tid; i < 2 * half; i += 256) {
    const int x = i < half ? base - half + i : base + kFinishTile + (i - half);
    float val = 0.f;
    bool has_mass = x >= 0 && x < a.T;
    if (has_mass && a.mass_trim > 0)
      has_mass = x < a.cu_seqlens[request_of(a.cu_seqlens, a.n_seqs, x) + 1] - a.mass_trim;
    if (has_mass)
      for (int sp = 0; sp < a.row_splits; ++sp) val += a.uraw[((int64_t)sp * a.LH + lz) * a.T + x];
    tile[x - base + half] = val;
  }
#pragma unroll
  for (int e = 0; e < PER; ++e) tile[half + e * 256 + tid] = body[e];
  __syncthreads();
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int j = base + e * 256 + tid;
    if (j >= a.T) continue;
    const int s0 = lo_[e], s1 = hi_[e] - a.pool_trim;     // pooling domain [s0, s1)
    const int b0 = max(s0, j - half), b1 = min(s1 - 1, j + half);
    float pooled = 0.f;
    if (j < s1) {
      if (a.pool_max) {
        for (int x = b0; x <= b1; ++x) pooled = fmaxf(pooled, tile[x - base + half]);      // masses are >= 0
      } else {
        for (int x = b0; x <= b1; ++x) pooled += tile[x - base + half];
        pooled *= a.inv_pool;
      }
    }
    a.scores[(int64_t)lz * a.T + j] = __builtin_fmaf(a.lambda, pr[e], pooled);
  }
}

int launch_row_merge(const Plan& pl, const ScoreArgs& a, hipStream_t stream) {
  const bool many = (int64_t)pl.n_seqs * pl.L * pl.Hkv >= 2048;     // enough workgroups for the device as it is
  const dim3 mgrid(many ? 1 : (a.lrows + 255) / 256, pl.n_seqs, pl.L * pl.Hkv);
  score_merge_kernel<<<mgrid, dim3(256), 0, stream>>>(a);
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

int launch_score(const Plan& pl, const void* q, const void* k, const float* prior, float* scores,
                 void* workspace, hipStream_t stream, unsigned stages) {
  char* ws = static_cast<char*>(workspace);
  ScoreArgs a;
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const unsigned char*>(k);
  a.cu_seqlens = pl.cu_seqlens_dev;
  a.stats = reinterpret_cast<float*>(ws + pl.off_stats);
  a.lse = reinterpret_cast<float*>(ws + pl.off_lse);
  a.uraw = reinterpret_cast<float*>(ws + pl.off_uraw);
  a.n_seqs = pl.n_seqs; a.Hkv = pl.Hkv; a.G = pl.G; a.W = pl.W; a.R = pl.R;
  a.row_splits = pl.row_splits; a.nb = pl.row_blocks; a.srows = pl.waves * kRowsPerWave;
  a.lrows = pl.row_splits * pl.row_blocks * 32;
  for (int w = 0; w < kMaxWaves; ++w) a.wave_desc[w] = pl.wave_desc[w];
  for (int b = 0; b < 2 * kMaxWaves; ++b) { a.rb_holder[b][0] = pl.rb_holder[b][0]; a.rb_holder[b][1] = pl.rb_holder[b][1]; }
  a.lead = pl.lead_tiles; a.tiles_per_problem = pl.tiles_per_problem; a.total_tiles = pl.total_tiles; a.stat_teams = 0; a.T = pl.T;
  a.LH = pl.L * pl.Hkv;
  a.q_sl = pl.q_sl; a.q_ss = pl.q_ss; a.q_sh = pl.q_sh; a.q_st = pl.q_st;
  a.kv_sl = pl.kv_sl; a.kv_sh = pl.kv_sh; a.kv_st = pl.kv_st;
  a.c = pl.scale * 1.4426950408889634f;
  a.inv_g = (pl.variant & CODECOMP_VARIANT_GROUP_SUM) ? 1.0f : 1.0f / (float)pl.G;
  a.key_trim = pl.key_trim;
  a.blocks_per_head = (pl.variant & CODECOMP_VARIANT_GROUP_MAX) ? pl.W / 32 : 1;
  int rc;
  if (pl.kv_fp8) rc = pl.d == 128 ? dispatch_waves<128, true>(pl, a, stream, stages) : dispatch_waves<64, true>(pl, a, stream, stages);
  else rc = pl.d == 128 ? dispatch_waves<128, false>(pl, a, stream, stages) : dispatch_waves<64, false>(pl, a, stream, stages);
  if (rc) return rc;
  if (!(stages & CODECOMP_STAGE_FINISH)) return 0;

  FinishArgs f;
  f.uraw = a.uraw; f.prior = prior; f.cu_seqlens = pl.cu_seqlens_dev; f.scores = scores;
  f.n_seqs = pl.n_seqs; f.T = pl.T; f.LH = pl.L * pl.Hkv; f.row_splits = pl.row_splits; f.pool = pl.pool;
  f.lambda = pl.lambda; f.inv_pool = 1.0f / (float)pl.pool;
  f.mass_trim = pl.key_trim;
  f.pool_trim = (pl.variant & CODECOMP_VARIANT_POOL_PREFIX) ? pl.W : 0;
  f.pool_max = (pl.variant & CODECOMP_VARIANT_POOL_MAX) ? 1 : 0;
  score_finish_kernel<<<dim3((pl.T + kFinishTile - 1) / kFinishTile, pl.L * pl.Hkv), dim3(256), 0, stream>>>(f);
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

}  // namespace codecomp
