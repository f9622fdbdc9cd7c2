// Score step: window attention mass -> group mean -> average pool -> + lambda * prior.
//
// For one (layer, KV head, request) the R = G*W observation rows are soft-maxed over all N_r
// keys and summed per key (the equation of section "Attention-based KV Cache Compression").
// A column sum of a row softmax needs every row normaliser first, so the logits are formed
// twice on the matrix cores:
//   pass 1  S^T tile = K Q^T   (lane = query row)  -> per-row running (max, sum) -> per-chunk stats
//   merge   per-row log2-sum-exp over the chunks of a request
//   pass 2  S tile   = Q K^T   (lane = key)        -> exp2(s*c - lse) summed over rows -> u
//   finish  average pool over pool_kernel neighbours inside the request, add lambda * prior
// Both passes keep the wave's 64 query rows as MFMA fragments in registers for the whole
// workgroup lifetime and stream 64-key tiles of K through LDS (double buffered, one barrier
// per tile).  v_mfma_f32_32x32x16_bf16: the A and B fragments have the same lane layout
// (lane%32 = row/column, lane/32 = which 8 of the 16 k values), so swapping the operands
// transposes the output tile without touching the loads.
#include "plan.h"

namespace codecomp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct ScoreArgs {
  const uint16_t* q;
  const uint16_t* k;
  const int32_t* cu_seqlens;
  float* stats;   // [L*Hkv][total_chunks][rpad][2] : (max * c, sum of exp2(s*c - max*c))
  float* lse;     // [L*Hkv][n_seqs][rpad]          : log2 sum_j exp2(s_j * c)
  float* uraw;    // [row_splits][L*Hkv][T]         : (1/G) * sum over this split's rows of A
  int n_seqs, Hkv, G, W, R, rows_per_split, rpad, chunk_keys, total_chunks, T;
  int64_t q_sl, q_ss, q_sh, q_st, kv_sl, kv_sh, kv_st;
  float c;        // softmax_scale * log2(e)
  float inv_g;
};

#define NEG_BIG (-1.0e30f)

__device__ __forceinline__ bf16x8 frag(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ bool locate_chunk(const int32_t* cu, int n_seqs, int chunk_keys, int item,
                                             int& seq, int& tok0, int& n, int& local, int& chunk_base) {
  int acc = 0;
  for (int r = 0; r < n_seqs; ++r) {
    int a = cu[r], b = cu[r + 1];
    int nch = (b - a + chunk_keys - 1) / chunk_keys;
    if (item < acc + nch) {
      seq = r; tok0 = a; n = b - a; local = item - acc; chunk_base = acc;
      return true;
    }
    acc += nch;
  }
  return false;
}

template <int D, int NW, int PASS>
__global__ __launch_bounds__(NW * 64) void score_pass_kernel(ScoreArgs a) {
  constexpr int NT = NW * 64;
  constexpr int KS = D / 16;                   // MFMA k-steps per logit
  constexpr int ROWB = D * 2 + 16;             // LDS bytes per key row (+16: spreads rows over banks)
  constexpr int CH_PER_ROW = D / 8;            // 16-byte pieces per key row
  constexpr int NCH = kTileKeys * CH_PER_ROW;  // pieces per tile
  constexpr int LD = (NCH + NT - 1) / NT;      // pieces staged per thread

  __shared__ __attribute__((aligned(16))) unsigned char ktile[2][kTileKeys * ROWB];
  __shared__ float colbuf[PASS == 2 ? 2 : 1][PASS == 2 ? NW : 1][kTileKeys];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hf = lane >> 5;
  const int split = blockIdx.y;
  const int lz = blockIdx.z;               // layer * Hkv + head
  const int layer = lz / a.Hkv;
  const int head = lz - layer * a.Hkv;

  int seq, tok0, n, local, chunk_base;
  if (!locate_chunk(a.cu_seqlens, a.n_seqs, a.chunk_keys, blockIdx.x, seq, tok0, n, local, chunk_base)) return;
  const int kstart = local * a.chunk_keys;
  const int kend = min(n, kstart + a.chunk_keys);
  const int ntiles = (kend - kstart + kTileKeys - 1) / kTileKeys;

  // ---- this wave's 64 query rows as MFMA fragments
  const int row0 = split * a.rows_per_split + wave * kRowsPerWave;
  uint4 qf[2][KS];
  {
    const uint16_t* qb = a.q + (int64_t)layer * a.q_sl + (int64_t)seq * a.q_ss;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const int row = row0 + rb * 32 + l32;
      const bool ok = row < a.R;
      const int g = ok ? row / a.W : 0;
      const int t = ok ? row - g * a.W : 0;
      const uint16_t* p = qb + (int64_t)(head * a.G + g) * a.q_sh + (int64_t)t * a.q_st + hf * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (ok) v = *reinterpret_cast<const uint4*>(p + ks * 16);
        qf[rb][ks] = v;
      }
    }
  }

  const uint16_t* kb = a.k + (int64_t)layer * a.kv_sl + (int64_t)head * a.kv_sh + (int64_t)tok0 * a.kv_st;
  uint4 stage[LD];
  auto gload = [&](int key0) {
#pragma unroll
    for (int i = 0; i < LD; ++i) {
      const int cidx = tid + i * NT;
      const int row = cidx / CH_PER_ROW, col = cidx - row * CH_PER_ROW;
      const int key = key0 + row;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (cidx < NCH && key < kend) v = *reinterpret_cast<const uint4*>(kb + (int64_t)key * a.kv_st + col * 8);
      stage[i] = v;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LD; ++i) {
      const int cidx = tid + i * NT;
      const int row = cidx / CH_PER_ROW, col = cidx - row * CH_PER_ROW;
      if (cidx < NCH) *reinterpret_cast<uint4*>(&ktile[buf][row * ROWB + col * 16]) = stage[i];
    }
  };

  const float c = a.c;

  // pass 1 state: running (max, sum) of this lane's row over the keys this lane sees
  float m_run[2] = {NEG_BIG, NEG_BIG};
  float l_run[2] = {0.f, 0.f};
  // pass 2 state: -lse of the 32 rows this lane holds in the S tile
  float nl[2][16];
  if constexpr (PASS == 2) {
    const float* lse = a.lse + ((int64_t)lz * a.n_seqs + seq) * a.rpad;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = row0 + rb * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
        nl[rb][v] = row < a.R ? -lse[row] : -INFINITY;
      }
  }

  auto reduce_cols = [&](int buf, int key0) {
    // sum the per-wave column partials of one finished tile and store the attention mass
    if constexpr (PASS == 2) {
      if (tid < kTileKeys) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += colbuf[buf][w][tid];
        const int key = key0 + tid;
        if (key < kend) a.uraw[((int64_t)split * gridDim.z + lz) * a.T + tok0 + key] = s * a.inv_g;
      }
    }
  };

  gload(kstart);
  sstore(0);
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const int buf = t & 1;
    const int key0 = kstart + t * kTileKeys;
    if (t + 1 < ntiles) gload(key0 + kTileKeys);
    if constexpr (PASS == 2) {
      if (t > 0) reduce_cols(buf ^ 1, key0 - kTileKeys);
    }
    const int nvalid = min(kTileKeys, kend - key0);

#pragma unroll
    for (int kh = 0; kh < 2; ++kh) {
      f32x16 acc0 = {0}, acc1 = {0};
      const unsigned char* kp = &ktile[buf][(kh * 32 + l32) * ROWB + hf * 16];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const uint4 kf = *reinterpret_cast<const uint4*>(kp + ks * 32);
        if constexpr (PASS == 1) {
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(kf), frag(qf[0][ks]), acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(kf), frag(qf[1][ks]), acc1, 0, 0, 0);
        } else {
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(qf[0][ks]), frag(kf), acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(qf[1][ks]), frag(kf), acc1, 0, 0, 0);
        }
      }
      if constexpr (PASS == 1) {
        // lane = query row (l32 of row block rb); register v = key 8*(v/4) + 4*hf + v%4 of this half tile
        if (nvalid < kTileKeys) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key_local = kh * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
            if (key_local >= nvalid) { acc0[v] = -INFINITY; acc1[v] = -INFINITY; }
          }
        }
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          const f32x16& acc = rb == 0 ? acc0 : acc1;
          float tmax = acc[0];
#pragma unroll
          for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, acc[v]);
          const float m_new = fmaxf(m_run[rb], tmax);
          const float alpha = __builtin_amdgcn_exp2f((m_run[rb] - m_new) * c);
          const float mc = m_new * c;
          float s0 = 0.f, s1 = 0.f;
#pragma unroll
          for (int v = 0; v < 16; v += 2) {
            s0 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[v], c, -mc));
            s1 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[v + 1], c, -mc));
          }
          l_run[rb] = l_run[rb] * alpha + (s0 + s1);
          m_run[rb] = m_new;
        }
      } else {
        // lane = key l32 of this half tile; register v of row block rb = query row 8*(v/4) + 4*hf + v%4
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          s0 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc0[v], c, nl[0][v]));
          s1 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc1[v], c, nl[1][v]));
        }
        float col = s0 + s1;
        col += __shfl_xor(col, 32);
        if (lane < 32) colbuf[buf][wave][kh * 32 + lane] = col;
      }
    }

    if (t + 1 < ntiles) sstore(buf ^ 1);
    __syncthreads();
  }

  if constexpr (PASS == 2) {
    reduce_cols((ntiles - 1) & 1, kstart + (ntiles - 1) * kTileKeys);
  } else {
    // merge the two half-wave views of each row, then one (max*c, sum) pair per row and chunk
    float* st = a.stats + (((int64_t)lz * a.total_chunks + chunk_base + local) * a.rpad) * 2;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const float m_o = __shfl_xor(m_run[rb], 32);
      const float l_o = __shfl_xor(l_run[rb], 32);
      const float M = fmaxf(m_run[rb], m_o);
      const float L = l_run[rb] * __builtin_amdgcn_exp2f((m_run[rb] - M) * c) +
                      l_o * __builtin_amdgcn_exp2f((m_o - M) * c);
      const int row = row0 + rb * 32 + l32;
      if (lane < 32) {
        st[row * 2 + 0] = M * c;
        st[row * 2 + 1] = L;
      }
    }
  }
}

// One thread per (layer*head, request, row): log2-sum-exp over that request's chunks.
__global__ __launch_bounds__(256) void score_merge_kernel(ScoreArgs a) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  const int seq = blockIdx.y;
  const int lz = blockIdx.z;
  if (row >= a.rpad) return;
  int chunk_base = 0;
  for (int r = 0; r < seq; ++r)
    chunk_base += (a.cu_seqlens[r + 1] - a.cu_seqlens[r] + a.chunk_keys - 1) / a.chunk_keys;
  const int nch = (a.cu_seqlens[seq + 1] - a.cu_seqlens[seq] + a.chunk_keys - 1) / a.chunk_keys;
  const float* st = a.stats + (((int64_t)lz * a.total_chunks + chunk_base) * a.rpad + row) * 2;
  float M = NEG_BIG;
  for (int ch = 0; ch < nch; ++ch) M = fmaxf(M, st[(int64_t)ch * a.rpad * 2]);
  float L = 0.f;
  for (int ch = 0; ch < nch; ++ch)
    L += st[(int64_t)ch * a.rpad * 2 + 1] * __builtin_amdgcn_exp2f(st[(int64_t)ch * a.rpad * 2] - M);
  a.lse[((int64_t)lz * a.n_seqs + seq) * a.rpad + row] = M + log2f(L);
}

struct FinishArgs {
  const float* uraw;
  const float* prior;
  const int32_t* cu_seqlens;
  float* scores;
  int n_seqs, T, LH, row_splits, pool;
  float lambda, inv_pool;
};

// scores[lz][j] = (1/k) * sum_{|delta| <= (k-1)/2, inside the request} u[lz][j+delta] + lambda * prior[j]
__global__ __launch_bounds__(256) void score_finish_kernel(FinishArgs a) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int lz = blockIdx.y;
  if (j >= a.T) return;
  int lo = 0, hi = a.n_seqs;            // request containing token j: cu[lo] <= j < cu[lo+1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.cu_seqlens[mid] <= j) lo = mid; else hi = mid;
  }
  const int s0 = a.cu_seqlens[lo], s1 = a.cu_seqlens[lo + 1];
  const int half = (a.pool - 1) >> 1;
  const int b0 = max(s0, j - half), b1 = min(s1 - 1, j + half);
  float sum = 0.f;
  for (int sp = 0; sp < a.row_splits; ++sp) {
    const float* u = a.uraw + ((int64_t)sp * a.LH + lz) * a.T;
    for (int x = b0; x <= b1; ++x) sum += u[x];
  }
  a.scores[(int64_t)lz * a.T + j] = __builtin_fmaf(a.lambda, a.prior[j], sum * a.inv_pool);
}

template <int D, int NW>
static int launch_passes(const Plan& pl, const ScoreArgs& a, hipStream_t stream, unsigned stages) {
  const dim3 grid(pl.total_chunks, pl.row_splits, pl.L * pl.Hkv);
  const dim3 block(NW * 64);
  if (stages & CODECOMP_STAGE_ROW_STATS) {
    score_pass_kernel<D, NW, 1><<<grid, block, 0, stream>>>(a);
    if (hipError_t e = hipGetLastError()) return (int)e;
  }
  if (stages & CODECOMP_STAGE_ROW_MERGE) {
    const dim3 mgrid((a.rpad + 255) / 256, pl.n_seqs, pl.L * pl.Hkv);
    score_merge_kernel<<<mgrid, dim3(256), 0, stream>>>(a);
    if (hipError_t e = hipGetLastError()) return (int)e;
  }
  if (stages & CODECOMP_STAGE_MASS) {
    score_pass_kernel<D, NW, 2><<<grid, block, 0, stream>>>(a);
    if (hipError_t e = hipGetLastError()) return (int)e;
  }
  return 0;
}

template <int D>
static int dispatch_waves(const Plan& pl, const ScoreArgs& a, hipStream_t s, unsigned st) {
  switch (pl.waves) {
    case 1: return launch_passes<D, 1>(pl, a, s, st);
    case 2: return launch_passes<D, 2>(pl, a, s, st);
    case 3: return launch_passes<D, 3>(pl, a, s, st);
    case 4: return launch_passes<D, 4>(pl, a, s, st);
    case 5: return launch_passes<D, 5>(pl, a, s, st);
    case 6: return launch_passes<D, 6>(pl, a, s, st);
    case 7: return launch_passes<D, 7>(pl, a, s, st);
    case 8: return launch_passes<D, 8>(pl, a, s, st);
  }
  return CODECOMP_EINVAL_SHAPE;
}

int launch_score(const Plan& pl, const void* q, const void* k, const float* prior, float* scores,
                 void* workspace, hipStream_t stream, unsigned stages) {
  char* ws = static_cast<char*>(workspace);
  ScoreArgs a;
  a.q = static_cast<const uint16_t*>(q);
  a.k = static_cast<const uint16_t*>(k);
  a.cu_seqlens = pl.cu_seqlens_dev;
  a.stats = reinterpret_cast<float*>(ws + pl.off_stats);
  a.lse = reinterpret_cast<float*>(ws + pl.off_lse);
  a.uraw = reinterpret_cast<float*>(ws + pl.off_uraw);
  a.n_seqs = pl.n_seqs; a.Hkv = pl.Hkv; a.G = pl.G; a.W = pl.W; a.R = pl.R;
  a.rows_per_split = pl.rows_per_split; a.rpad = pl.row_splits * pl.rows_per_split;
  a.chunk_keys = pl.chunk_keys; a.total_chunks = pl.total_chunks; a.T = pl.T;
  a.q_sl = pl.q_sl; a.q_ss = pl.q_ss; a.q_sh = pl.q_sh; a.q_st = pl.q_st;
  a.kv_sl = pl.kv_sl; a.kv_sh = pl.kv_sh; a.kv_st = pl.kv_st;
  a.c = pl.scale * 1.4426950408889634f;
  a.inv_g = 1.0f / (float)pl.G;
  int rc = pl.d == 128 ? dispatch_waves<128>(pl, a, stream, stages) : dispatch_waves<64>(pl, a, stream, stages);
  if (rc) return rc;
  if (!(stages & CODECOMP_STAGE_FINISH)) return 0;

  FinishArgs f;
  f.uraw = a.uraw; f.prior = prior; f.cu_seqlens = pl.cu_seqlens_dev; f.scores = scores;
  f.n_seqs = pl.n_seqs; f.T = pl.T; f.LH = pl.L * pl.Hkv; f.row_splits = pl.row_splits; f.pool = pl.pool;
  f.lambda = pl.lambda; f.inv_pool = 1.0f / (float)pl.pool;
  score_finish_kernel<<<dim3((pl.T + 255) / 256, pl.L * pl.Hkv), dim3(256), 0, stream>>>(f);
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

}  // namespace codecomp
