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

#ifdef __cplusplus
}
#endif
#endif /* CODECOMP_PEAKS_H */
