"""What this GPU sustains on the ingredients of the score passes (libcodecomp_peaks.so, csrc/peaks.hip):
MFMA-only rate with random bf16 operands, v_exp_f32 and v_fma_f32 issue rates, the MFMA + softmax instruction
mix of a score pass without memory, copy and read bandwidth.  Measurement only; bench.py prints these next to
the published peaks.

  python -m paper_2604_10235_amd.peaks [--repeat 3]
  python -m paper_2604_10235_amd.peaks --pass-model     # a loop shaped like the passes, feature by feature (csrc/pass_model.hip)
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


class codecomp_pass_model_row(C.Structure):
    _fields_ = [("features", C.c_int32), ("tiles_ahead", C.c_int32), ("logits_per_s", C.c_double),
                ("clock_mhz", C.c_double), ("cycles_per_mfma", C.c_double), ("hbm_gbs", C.c_double)]


PASS_MODEL_MAX_ROWS = 12
PASS_MODEL_FEATURES = {1: "LDS ring + barrier", 2: "staging writes", 4: "global loads", 16: "loads straight into LDS",
                       8: "uneven waves"}


class codecomp_pass_model(C.Structure):
    _fields_ = [("rows", codecomp_pass_model_row * PASS_MODEL_MAX_ROWS), ("n_rows", C.c_int32),
                ("compute_units", C.c_int32), ("status", C.c_int32), ("reserved_", C.c_int32)]


_state = {}


def _setup(copy_bytes: int) -> dict:
    """Loads the library and allocates the buffers of the measurements once."""
    import numpy as np
    import torch
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2604_10235_amd.build)")
    if "lib" not in _state:
        lib = C.CDLL(LIB_PATH)
        lib.codecomp_measure_peaks.restype = C.c_int
        lib.codecomp_measure_peaks.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p,
                                               C.POINTER(codecomp_peaks), C.c_void_p]
        lib.codecomp_measure_pass_model.restype = C.c_int
        lib.codecomp_measure_pass_model.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p,
                                                    C.POINTER(codecomp_pass_model), C.c_void_p]
        dev = torch.device("cuda:0")
        g = np.random.Generator(np.random.Philox(key=[20260410235, 7]))
        rnd = torch.from_numpy(g.standard_normal(1 << 15).astype(np.float32)).to(dev).to(torch.bfloat16)   # 64 KiB
        # the copy source doubles as the key stream of the pass model: bf16 normals, so that the MFMAs see real operands
        a = rnd.view(torch.uint8).repeat((copy_bytes + (1 << 16) - 1) >> 16)[:copy_bytes].contiguous()
        _state.update(lib=lib, rnd=rnd, a=a,
                      b=torch.empty(copy_bytes, dtype=torch.uint8, device=dev),
                      small=torch.zeros(64, dtype=torch.uint8, device=dev))
    return _state


def measure(copy_bytes: int = 1 << 30) -> dict:
    """One measurement on cuda:0 (about 0.1 s of GPU time).  Raises if the library is missing or a launch fails."""
    import torch
    st = _setup(copy_bytes)
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


def measure_pass_model(stream_bytes: int = 1 << 30) -> list:
    """The synthetic pass loop of csrc/pass_model.hip, one dict per variant (about 0.1 s of GPU time); it streams
    through the copy source of the peak measurement."""
    import torch
    st = _setup(stream_bytes)
    lib, big = st["lib"], st["a"]
    out = codecomp_pass_model()
    rc = lib.codecomp_measure_pass_model(st["rnd"].data_ptr(), big.data_ptr(), big.numel(), st["small"].data_ptr(),
                                         C.byref(out), int(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError(f"codecomp_measure_pass_model: status {rc}")
    rows = []
    for i in range(out.n_rows):
        r = out.rows[i]
        rows.append({"features": " + ".join(n for b, n in PASS_MODEL_FEATURES.items() if r.features & b),
                     "tiles_ahead": r.tiles_ahead, "logits_per_s": float(f"{r.logits_per_s:.4g}"),
                     "clock_mhz": round(r.clock_mhz), "cycles_per_mfma": round(r.cycles_per_mfma, 1),
                     "hbm_gb_per_s": round(r.hbm_gbs, 1)})
    return rows


def release():
    _state.clear()


def main() -> int:
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--repeat", type=int, default=3)
    ap.add_argument("--pass-model", action="store_true", help="run the synthetic pass loop instead of the peaks")
    args = ap.parse_args()
    for i in range(args.repeat):
        if args.pass_model:
            for row in measure_pass_model():
                print(json.dumps(row))
            print()
        else:
            print(json.dumps(measure()))
    return 0


if __name__ == "__main__":
    sys.exit(main())
