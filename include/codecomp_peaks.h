/*
 * codecomp_peaks.h - C ABI of libcodecomp_peaks: what the GPU sustains on the ingredients of the score passes of
 * codecomp.h (the two logit passes behind the attention equation of section "Attention-based KV Cache
 * Compression").  A measurement aid for the benchmark, not part of the hot path and not from the paper: the
 * roofline fractions of a run are printed against the published peaks and against these measured ones.
 */
#ifndef CODECOMP_PEAKS_H
#define CODECOMP_PEAKS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct codecomp_peaks {
  double mfma_bf16_tflops;      /* v_mfma_f32_32x32x16_bf16 only, random bf16 operands, whole chip          */
  double mfma_clock_mhz;        /* shader clock during that run                                              */
  double exp_per_s;             /* v_exp_f32 results per second, whole chip                                  */
  double fma_per_s;             /* v_fma_f32 results per second, whole chip                                  */
  double mix_logits_per_s;      /* logits per second through (half an MFMA at head_dim 128) + fma + exp2 + add:
                                   the instruction mix of a score pass without memory                        */
  double mix_clock_mhz;         /* shader clock during that run                                              */
  double copy_gbs;              /* (bytes read + bytes written) / time of a copy pass over `bytes`           */
  double read_gbs;              /* bytes read / time of a read-only pass                                     */
  int32_t mix_waves_per_simd;   /* waves per SIMD the mix ran with (2, as the score passes, where it fits)   */
  int32_t compute_units;
  int32_t status;               /* 0, -1 (bad argument), -2 (a kernel does not fit the device) or a hipError_t */
} codecomp_peaks;

/* All pointers are DEVICE pointers except `out` (host).  rnd: at least 64 KiB of bf16 bit patterns of random numbers
 * (operands of the MFMA runs), 16-byte aligned.  buf_a, buf_b: `bytes` bytes each, the copy's source and destination
 * (bytes a multiple of 16 and at least 1 MiB; several times the 256 MB memory-side cache for a figure that means HBM).
 * small: at least 64 bytes.  Launches a handful of short kernels on `hip_stream` (NULL = default stream), each twice
 * (the second launch is timed with events), and SYNCHRONISES the stream: a measurement, not a hot-path call.
 * Allocates nothing on the device.  Returns `out->status`. */
int codecomp_measure_peaks(const void* rnd, void* buf_a, void* buf_b, size_t bytes, void* small, codecomp_peaks* out,
                           void* hip_stream);

/* A synthetic loop with the structure of the score passes (eight waves, two row blocks per wave, 64-key tiles,
 * accumulators in VGPRs), its features switched on one by one; one row per variant. */
#define CODECOMP_PASS_MODEL_RING 1      /* K fragments from LDS through a register ring, one workgroup barrier per tile */
#define CODECOMP_PASS_MODEL_STAGE 2     /* every thread parks 32 bytes per tile in LDS (the next tile)                  */
#define CODECOMP_PASS_MODEL_LOADS 4     /* ... that come from global memory, 16 KB per tile and workgroup               */
#define CODECOMP_PASS_MODEL_UNEVEN 8    /* the second wave of every SIMD carries three units per tile against four      */
#define CODECOMP_PASS_MODEL_DIRECT 16   /* the tile's bytes go from global memory straight into LDS (no registers)      */
#define CODECOMP_PASS_MODEL_MAX_ROWS 12

typedef struct codecomp_pass_model_row {
  int32_t features;             /* CODECOMP_PASS_MODEL_* bits                                                */
  int32_t tiles_ahead;          /* tiles between sending for a tile's bytes and parking them (0: no loads)   */
  double logits_per_s;          /* whole chip                                                                */
  double clock_mhz;             /* shader clock during the run                                               */
  double cycles_per_mfma;       /* shader cycles per MFMA and SIMD                                           */
  double hbm_gbs;               /* bytes streamed from `big` per second                                      */
} codecomp_pass_model_row;

typedef struct codecomp_pass_model {
  codecomp_pass_model_row rows[CODECOMP_PASS_MODEL_MAX_ROWS];
  int32_t n_rows;
  int32_t compute_units;
  int32_t status;               /* as codecomp_peaks.status                                                  */
  int32_t reserved_;
} codecomp_pass_model;

/* All pointers are DEVICE pointers except `out` (host).  rnd: at least 64 KiB of bf16 bit patterns, 16-byte aligned.
 * big: `big_bytes` bytes that the loop streams through (a multiple of 16; at least 16 KiB per compute unit, several
 * times the 256 MB memory-side cache for a figure that means HBM); small: at least 64 bytes.  Launches every variant
 * twice on `hip_stream` (the second launch is timed) and SYNCHRONISES the stream.  Allocates nothing on the device.
 * Returns `out->status`; `out->n_rows` rows are valid. */
int codecomp_measure_pass_model(const void* rnd, const void* big, size_t big_bytes, void* small,
                                codecomp_pass_model* out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CODECOMP_PEAKS_H */
