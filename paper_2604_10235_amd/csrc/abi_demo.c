/* A C99 program that uses the library through its C ABI alone (no Python, no PyTorch): device memory from the HIP
 * runtime, one fused codecomp_compress call, and checks of what the header promises about its outputs - exactly B
 * ascending request-local indices per (layer, KV head), the observation window kept, and k_out / v_out equal to the
 * rows of K / V that the indices name, bit for bit.  Prints "abi_demo: ok" and returns 0, or says what failed. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "codecomp.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "abi_demo: %s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)

static uint32_t lcg(uint32_t* s) { *s = *s * 1664525u + 1013904223u; return *s; }
/* a bf16 bit pattern with magnitude in [0.5, 2) and a random sign */
static uint16_t some_bf16(uint32_t* s) { const uint32_t r = lcg(s); return (uint16_t)(0x3f00u + ((r >> 16) & 0xffu) + ((r >> 31) << 15)); }

int main(void) {
  enum { L = 2, HQ = 8, HKV = 2, D = 128, N = 5000, W = 64, B = 700 };
  const size_t nq = (size_t)L * HQ * W * D, nkv = (size_t)L * HKV * N * D, nout = (size_t)L * HKV * B * D;
  uint16_t* q = malloc(nq * 2); uint16_t* k = malloc(nkv * 2); uint16_t* v = malloc(nkv * 2);
  float* prior = malloc(N * sizeof(float));
  int32_t* idx = malloc((size_t)L * HKV * B * sizeof(int32_t));
  uint16_t* ko = malloc(nout * 2); uint16_t* vo = malloc(nout * 2);
  if (!q || !k || !v || !prior || !idx || !ko || !vo) return 3;
  uint32_t seed = 20260410u;
  for (size_t i = 0; i < nq; ++i) q[i] = some_bf16(&seed);
  for (size_t i = 0; i < nkv; ++i) { k[i] = some_bf16(&seed); v[i] = some_bf16(&seed); }
  for (int j = 0; j < N; ++j) prior[j] = (j / 40) % 5 == 0 ? 1.0f : 0.0f;      /* every fifth span of 40 tokens is marked */

  int32_t cu_seqlens[2] = {0, N}, cu_budgets[2] = {0, B};
  void *dq, *dk, *dv, *dprior, *dscores, *didx, *dko, *dvo, *dws, *dcu, *dcb;
  CHECK_HIP(hipMalloc(&dq, nq * 2)); CHECK_HIP(hipMalloc(&dk, nkv * 2)); CHECK_HIP(hipMalloc(&dv, nkv * 2));
  CHECK_HIP(hipMalloc(&dprior, N * sizeof(float))); CHECK_HIP(hipMalloc(&dscores, (size_t)L * HKV * N * sizeof(float)));
  CHECK_HIP(hipMalloc(&didx, (size_t)L * HKV * B * sizeof(int32_t)));
  CHECK_HIP(hipMalloc(&dko, nout * 2)); CHECK_HIP(hipMalloc(&dvo, nout * 2));
  CHECK_HIP(hipMalloc(&dcu, sizeof cu_seqlens)); CHECK_HIP(hipMalloc(&dcb, sizeof cu_budgets));
  CHECK_HIP(hipMemcpy(dq, q, nq * 2, hipMemcpyHostToDevice)); CHECK_HIP(hipMemcpy(dk, k, nkv * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dv, v, nkv * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dprior, prior, N * sizeof(float), hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dcu, cu_seqlens, sizeof cu_seqlens, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dcb, cu_budgets, sizeof cu_budgets, hipMemcpyHostToDevice));

  codecomp_params p;
  memset(&p, 0, sizeof p);                       /* strides 0 = dense layouts, scale 0 = 1/sqrt(d), additive rule, bf16 cache */
  p.n_layers = L; p.n_q_heads = HQ; p.n_kv_heads = HKV; p.head_dim = D; p.window = W; p.pool_kernel = 7;
  p.prior_weight = 1.0f; p.n_seqs = 1;
  p.cu_seqlens_host = cu_seqlens; p.cu_budgets_host = cu_budgets;
  p.cu_seqlens_dev = (const int32_t*)dcu; p.cu_budgets_dev = (const int32_t*)dcb;
  int rc = codecomp_validate(&p);
  if (rc != CODECOMP_OK) { fprintf(stderr, "abi_demo: validate: %s\n", codecomp_status_string(rc)); return 4; }
  const size_t ws_bytes = codecomp_workspace_bytes(&p);
  CHECK_HIP(hipMalloc(&dws, ws_bytes ? ws_bytes : 256));
  rc = codecomp_compress(dq, dk, dv, (const float*)dprior, &p, (float*)dscores, (int32_t*)didx, dko, dvo, dws, ws_bytes, NULL);
  if (rc != CODECOMP_OK) { fprintf(stderr, "abi_demo: compress: %d %s\n", rc, codecomp_status_string(rc)); return 5; }
  CHECK_HIP(hipDeviceSynchronize());
  CHECK_HIP(hipMemcpy(idx, didx, (size_t)L * HKV * B * sizeof(int32_t), hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(ko, dko, nout * 2, hipMemcpyDeviceToHost)); CHECK_HIP(hipMemcpy(vo, dvo, nout * 2, hipMemcpyDeviceToHost));

  long marked_kept = 0;
  for (int lz = 0; lz < L * HKV; ++lz) {
    const int32_t* row = idx + (size_t)lz * B;
    for (int i = 0; i < B; ++i) {
      if (row[i] < 0 || row[i] >= N || (i > 0 && row[i] <= row[i - 1])) { fprintf(stderr, "abi_demo: indices of (layer, head) %d not ascending in range at %d\n", lz, i); return 6; }
      if (i >= B - W && row[i] != N - B + i) { fprintf(stderr, "abi_demo: window token missing at %d\n", i); return 7; }
      if (memcmp(ko + ((size_t)lz * B + i) * D, k + ((size_t)lz * N + row[i]) * D, D * 2) ||
          memcmp(vo + ((size_t)lz * B + i) * D, v + ((size_t)lz * N + row[i]) * D, D * 2)) { fprintf(stderr, "abi_demo: gathered row %d of %d differs\n", i, lz); return 8; }
      marked_kept += prior[row[i]] > 0.0f;
    }
  }
  /* keys of magnitude ~1 spread the attention thinly, so with weight 1 the marked tokens (1000 of 5000) fill all 636 prefix slots */
  if (marked_kept < (long)L * HKV * (B - W)) { fprintf(stderr, "abi_demo: only %ld marked tokens kept\n", marked_kept); return 9; }
  printf("abi_demo: ok (%d layers x %d KV heads, %d of %d tokens kept, workspace %zu bytes, library version %d)\n", L, HKV, B, N, ws_bytes, codecomp_version());
  return 0;
}
