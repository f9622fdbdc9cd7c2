"""What this GPU sustains on the ingredients of the score passes (libcodecomp_peaks.so, csrc/peaks.hip):
MFMA-only rate with random bf16 operands, v_exp_f32 and v_fma_f32 issue rates, the MFMA + softmax instruction
mix of a score pass without memory, copy and read bandwidth.  Measurement only; bench.py prints these next to
the published peaks.

  python -m paper_2604_10235_amd.peaks [--repeat 3]
"""
from __future__ import annotations

import ctypes as C
import json
import os
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcodecomp_peaks.so")


class codecomp_peaks(C.Structure):
    _fields_ = [("mfma_bf16_tflops", C.c_double), ("mfma_clock_mhz", C.c_double), ("exp_per_s", C.c_double),
                ("fma_per_s", C.c_double), ("mix_logits_per_s", C.c_double), ("mix_clock_mhz", C.c_double),
                ("copy_gbs", C.c_double), ("read_gbs", C.c_double),
                ("mix_waves_per_simd", C.c_int32), ("compute_units", C.c_int32), ("status", C.c_int32)]


_state = {}


def measure(copy_bytes: int = 1 << 30) -> dict:
    """One measurement on cuda:0 (about 0.1 s of GPU time).  Raises if the library is missing or a launch fails."""
    import numpy as np
    import torch
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2604_10235_amd.build)")
    if "lib" not in _state:
        lib = C.CDLL(LIB_PATH)
        lib.codecomp_measure_peaks.restype = C.c_int
        lib.codecomp_measure_peaks.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p,
                                               C.POINTER(codecomp_peaks), C.c_void_p]
        dev = torch.device("cuda:0")
        g = np.random.Generator(np.random.Philox(key=[20260410235, 7]))
        rnd = torch.from_numpy(g.standard_normal(1 << 15).astype(np.float32)).to(dev).to(torch.bfloat16)   # 64 KiB
        _state.update(lib=lib, rnd=rnd, a=torch.full((copy_bytes,), 7, dtype=torch.uint8, device=dev),
                      b=torch.empty(copy_bytes, dtype=torch.uint8, device=dev),
                      small=torch.zeros(64, dtype=torch.uint8, device=dev))
    st = _state
    out = codecomp_peaks()
    rc = st["lib"].codecomp_measure_peaks(st["rnd"].data_ptr(), st["a"].data_ptr(), st["b"].data_ptr(), st["a"].numel(),
                                          st["small"].data_ptr(), C.byref(out), int(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError(f"codecomp_measure_peaks: status {rc}")
    return {"mfma_bf16_tflops": round(out.mfma_bf16_tflops, 1), "mfma_clock_mhz": round(out.mfma_clock_mhz),
            "exp_per_s": float(f"{out.exp_per_s:.4g}"), "fma_per_s": float(f"{out.fma_per_s:.4g}"),
            "mix_logits_per_s": float(f"{out.mix_logits_per_s:.4g}"), "mix_clock_mhz": round(out.mix_clock_mhz),
            # shader cycles a SIMD spends per MFMA and its 128 logits of softmax work, from the rate and the clock
            "mix_cycles_per_mfma": round(out.mix_clock_mhz * 1e6 * out.compute_units * 4 * 128 / out.mix_logits_per_s, 1)
            if out.mix_logits_per_s > 0 else None, "mix_waves_per_simd": out.mix_waves_per_simd,
            "copy_gb_per_s": round(out.copy_gbs, 1), "read_gb_per_s": round(out.read_gbs, 1),
            "compute_units": out.compute_units}


def release():
    _state.clear()


def main() -> int:
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--repeat", type=int, default=3)
    args = ap.parse_args()
    for i in range(args.repeat):
        print(json.dumps(measure()))
    return 0


if __name__ == "__main__":
    sys.exit(main())
