// Structure-side helpers around the hot path.
//  * Host arithmetic of the paper's sections "Structural Feature Extraction" (log normalisation,
//    chunk score sigma_i) and "Structure-Aware Budget Allocation" (normalised score, capacity
//    multiplier, token budget B_i): scalar work on a handful of chunks, done on the host in double.
//  * Str. Score on the device: the fraction of structurally critical tokens (prior > 0) that survive
//    compression, per (layer, KV head, request) - the paper's own quality proxy.
#include <math.h>

#include "plan.h"

namespace codecomp {

struct StrArgs {
  const int32_t* idx;
  const float* prior;
  const int32_t* cu_seqlens;
  const int32_t* cu_budgets;
  float* out;      // [L*Hkv][n_seqs]
  int n_seqs, TB;
};

__global__ __launch_bounds__(256) void structure_score_kernel(StrArgs a) {
  __shared__ int red[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int seq = blockIdx.x, lz = blockIdx.y;
  const int s0 = a.cu_seqlens[seq], n = a.cu_seqlens[seq + 1] - s0;
  const int o0 = a.cu_budgets[seq], b = a.cu_budgets[seq + 1] - o0;
  const float* p = a.prior + s0;
  const int32_t* idx = a.idx + (int64_t)lz * a.TB + o0;
  int total = 0, kept = 0;
  for (int j = tid; j < n; j += 256) total += p[j] > 0.f;
  for (int i = tid; i < b; i += 256) {
    const int j = min(max(idx[i], 0), n - 1);     // clamped: a corrupt index cannot read out of bounds
    kept += p[j] > 0.f;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { total += __shfl_xor(total, off); kept += __shfl_xor(kept, off); }
  if (lane == 0) { red[0][wave] = total; red[1][wave] = kept; }
  __syncthreads();
  if (tid == 0) {
    const int t = red[0][0] + red[0][1] + red[0][2] + red[0][3];
    const int k = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    a.out[(int64_t)lz * a.n_seqs + seq] = t > 0 ? (float)k / (float)t : __builtin_nanf("");
  }
}

int launch_structure_score(const Plan& pl, const int32_t* idx, const float* prior, float* out, hipStream_t stream) {
  StrArgs a;
  a.idx = idx; a.prior = prior; a.cu_seqlens = pl.cu_seqlens_dev; a.cu_budgets = pl.cu_budgets_dev; a.out = out;
  a.n_seqs = pl.n_seqs; a.TB = pl.TB;
  structure_score_kernel<<<dim3(pl.n_seqs, pl.L * pl.Hkv), dim3(256), 0, stream>>>(a);
  if (hipError_t e = hipGetLastError()) return (int)e;
  return 0;
}

}  // namespace codecomp

using namespace codecomp;

extern "C" {

int codecomp_chunk_structure_scores(const double* features_host, const double* tau_host, const double* weights_host,
                                    int32_t n_chunks, int32_t n_features, double* sigma_host) {
  if (!features_host || !tau_host || !weights_host || !sigma_host) return CODECOMP_EINVAL_NULL;
  if (n_chunks < 1 || n_features < 1) return CODECOMP_EINVAL_SHAPE;
  for (int k = 0; k < n_features; ++k)
    if (!(tau_host[k] > 0.0)) return CODECOMP_EINVAL_SHAPE;
  for (int i = 0; i < n_chunks; ++i) {
    double s = 0.0;
    for (int k = 0; k < n_features; ++k) {
      const double x = features_host[(size_t)i * n_features + k];
      if (!(x >= 0.0)) return CODECOMP_EINVAL_SHAPE;
      const double nrm = fmin(1.0, log1p(x) / log1p(tau_host[k]));
      s += weights_host[k] * nrm;
    }
    sigma_host[i] = s;
  }
  return CODECOMP_OK;
}

int codecomp_chunk_budgets(const double* sigma_host, const int32_t* chunk_len_host, int32_t n_chunks, double ratio,
                           double m_min, double m_max, double r_max, double eps, int32_t window,
                           int32_t* budgets_host) {
  if (!sigma_host || !chunk_len_host || !budgets_host) return CODECOMP_EINVAL_NULL;
  if (n_chunks < 1 || !(ratio >= 0.0) || !(m_max >= m_min) || !(r_max >= 0.0) || !(eps > 0.0) || window < 0)
    return CODECOMP_EINVAL_SHAPE;
  double lo = sigma_host[0], hi = sigma_host[0];
  for (int i = 1; i < n_chunks; ++i) { lo = fmin(lo, sigma_host[i]); hi = fmax(hi, sigma_host[i]); }
  for (int i = 0; i < n_chunks; ++i) {
    if (chunk_len_host[i] < 1) return CODECOMP_EINVAL_SEQLENS;
    if (window > chunk_len_host[i]) return CODECOMP_EINVAL_WINDOW;
    double s = 0.5;
    if (hi != lo) s = (sigma_host[i] - lo) / fmax(eps, hi - lo);
    s = fmin(1.0, fmax(0.0, s));
    const double m = m_min + (m_max - m_min) * s;
    double b = floor((double)chunk_len_host[i] * fmin(r_max, ratio * m));
    // the hot path always keeps the observation window and can keep at most the whole chunk
    b = fmin((double)chunk_len_host[i], fmax((double)window, b));
    budgets_host[i] = (int32_t)b;
  }
  return CODECOMP_OK;
}

int codecomp_structure_score(const int32_t* idx, const float* prior, const codecomp_params* params, float* retained,
                             void* hip_stream) {
  if (!idx || !prior || !params || !retained) return CODECOMP_EINVAL_NULL;
  Plan pl;
  if (int rc = make_plan(params, &pl)) return rc;
  return launch_structure_score(pl, idx, prior, retained, (hipStream_t)hip_stream);
}

}  // extern "C"
