#!/usr/bin/env python3
"""Benchmark of the prefill KV-eviction hot path (score -> select -> gather) on one MI355X.

One "step" is one fused codecomp_compress call over every layer of the workload: all layers
scored, selected and gathered, inputs already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload qwen7b_32k]

value = token-layers per second = (sum of request lengths) x layers / time per step.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
# No transcendental rate is published.  v_exp_f32 issues at half the fma rate on gfx950 (measured, see
# profiles/peaks_mi355x.md): 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz / 2.
EXP_PEAK_PER_S = 256 * 4 * 16 * 2.4e9 / 2


def algorithmic_bytes(w, kv_bytes: int = 2) -> dict:
    """Bytes the method itself must move per step: K once, Q, prior, scores written and read once,
    indices written and read once, retained K and V rows read and written (kv_bytes per cache element)."""
    L, H, T, TB, d = w.n_layers, w.n_kv_heads, w.total_tokens, w.total_budget, w.head_dim
    b = {
        "k_read": L * H * T * d * kv_bytes,
        "q_read": L * w.n_seqs * w.n_q_heads * w.window * d * 2,
        "prior_read": L * T * 4,
        "scores_rw": 2 * L * H * T * 4,
        "idx_rw": 2 * L * H * TB * 4,
        "gather_rw": 2 * 2 * L * H * TB * d * kv_bytes,
    }
    b["total"] = sum(b.values())
    return b


def read_traffic(name: str):
    """Measured HBM bytes per launch of the kernels, from the committed counter summary (profiles/pmc_<workload>.txt,
    lines `key = value`; FETCH_SIZE / WRITE_SIZE cannot be read from inside this process); None when no summary
    exists.  `commit` and `date` in that file say which build the counters were read on."""
    path = os.path.join(ROOT, "profiles", f"pmc_{name}.txt")
    if not os.path.exists(path):
        return None
    vals = {"file": os.path.relpath(path, ROOT)}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            v = v.strip()
            try:
                vals[k.strip()] = float(v.split()[0])
            except (ValueError, IndexError):
                vals[k.strip()] = v
    return vals


def binding_roofline(flops_pass: float, logits_pass: float, ab: dict, k_bytes: int, ms_per_step: float, peaks):
    """Floors of one step of the two-pass design (the logits are formed twice: row normalisers, then column sums) at
    the published peaks and, when measured, at what this GPU sustained in this run.  hbm_one_read is the method's own
    traffic (K once); hbm_two_reads adds K's second read.  issue_mix is the measured instruction mix of the passes
    without memory (MFMA and softmax VALU work compete for issue slots).  frac = largest floor / time per step."""
    def floors(mfma_tflops, exp_per_s, hbm_gbs, mix_logits_per_s=None):
        f = {"mfma_two_passes": 2 * flops_pass / (mfma_tflops * 1e12) * 1e3,
             "exp_two_passes": 2 * logits_pass / exp_per_s * 1e3,
             "hbm_one_read": ab["total"] / (hbm_gbs * 1e9) * 1e3,
             "hbm_two_reads": (ab["total"] + k_bytes) / (hbm_gbs * 1e9) * 1e3}
        if mix_logits_per_s:
            f["issue_mix_two_passes"] = 2 * logits_pass / mix_logits_per_s * 1e3
        return f

    def pack(f):
        binding = max((k for k in f if k != "hbm_one_read"), key=lambda k: f[k])
        return {"floors_ms": {k: round(v, 4) for k, v in f.items()}, "binding": binding,
                "frac": round(f[binding] / ms_per_step, 4)}

    out = {"spec": pack(floors(MFMA_BF16_PEAK_TFLOPS, EXP_PEAK_PER_S, HBM_PEAK_GBS))}
    if peaks:
        out["measured"] = pack(floors(peaks["mfma_bf16_tflops"], peaks["exp_per_s"], peaks["read_gb_per_s"],
                                      peaks["mix_logits_per_s"]))
    return out


class LayerSlices:
    """The same device buffers, worked through in slices of consecutive layers: every call of the path is made once
    per slice, one slice after the other (row statistics -> merge -> mass -> finish -> select -> gather of a slice
    before the next slice starts), so that the second logit pass of a slice reads the K its first pass has just
    read.  An experiment on K's second read (--layer-slices); argument marshalling only."""

    def __init__(self, prob, binding, n_slices: int):
        w = prob.w
        L = prob.n_layers
        if n_slices < 1 or L % n_slices:
            raise ValueError(f"--layer-slices must divide the layer count {L}")
        per = L // n_slices
        self.b, self.prob, self.subs = binding, prob, []
        for s in range(n_slices):
            sl = slice(s * per, (s + 1) * per)
            p = binding.make_params(n_layers=per, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                                    window=w.window, pool_kernel=w.pool_kernel, prior_weight=w.prior_weight,
                                    cu_seqlens_host=w.cu_seqlens(), cu_budgets_host=w.cu_budgets(),
                                    cu_seqlens_dev=prob.cu_seqlens.data_ptr(), cu_budgets_dev=prob.cu_budgets.data_ptr(),
                                    kv_dtype=prob.params.kv_dtype)
            self.subs.append((p, prob.q[sl], prob.k[sl], prob.v[sl], prob.scores[sl], prob.idx[sl], prob.k_out[sl], prob.v_out[sl]))

    def compress(self):
        for p, q, k, v, sc, ix, ko, vo in self.subs:
            self.b.codecomp_compress(q, k, v, self.prob.prior, p, sc, ix, ko, vo, self.prob.workspace)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200,
                    help="timed steps; the bracketing synchronisation costs a fixed ~1.5 ms, so few steps overstate the step time")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="qwen7b_32k")
    ap.add_argument("--kv-dtype", default="bf16", choices=["bf16", "fp8_e4m3"],
                    help="storage type of the KV cache (the headline workload is bf16; fp8_e4m3 is the 8-bit variant)")
    ap.add_argument("--cpu-layers", type=int, default=0,
                    help="layers the CPU oracle is timed and compared on (always layer 0 and the last one); 0 = as many "
                         "as keep its matrix products under 1.5 TFLOP (all 28 of the bench workload: ~5 s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the micro-benchmarks of what the GPU sustains")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (experiments only)")
    ap.add_argument("--layer-slices", type=int, default=1,
                    help="experiment on K's second read: run the whole path slice by slice over this many slices of "
                         "consecutive layers (1 = all layers in one call, the product's way); only the fused loop is timed")
    ap.add_argument("--operands", default="workload", choices=["workload", "zero_keys", "one_key", "zero_queries"],
                    help="experiment on the power limit: the same launches with keys that are all zero, all equal to "
                         "key 0, or with all-zero queries (results are checked like any other, the figures belong to no workload)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain device copy of 1 GiB (reads 1 GiB, writes 1 GiB): the reference "
                         "dispatch for scaling FETCH_SIZE / WRITE_SIZE counter readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2604_10235_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU substitute", file=sys.stderr)
        return 3
    if args.calibrate_copy:
        src = torch.full((1 << 30,), 7, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": 1 << 30, "calibrate_copy_bytes_written": 1 << 30, "copies": 3}))
        return 0
    w = wl.CONFIGS[args.workload]()
    if args.layers > 0:
        w = wl.scaled(w, name=f"{w.name}_L{args.layers}", n_layers=args.layers)
    t0 = time.time()
    q, k, v, prior = wl.make_all(w, threads=min(16, os.cpu_count() or 8))
    if args.kv_dtype == "fp8_e4m3":
        k, v = wl.bf16_bits_to_fp8_codes(k), wl.bf16_bits_to_fp8_codes(v)
    if args.operands == "zero_keys":
        k = np.zeros_like(k)
    elif args.operands == "one_key":
        k = np.ascontiguousarray(np.broadcast_to(k[:, :, :1, :], k.shape))
    elif args.operands == "zero_queries":
        q = np.zeros_like(q)
    if args.operands != "workload":
        w = wl.scaled(w, name=f"{w.name} with operands {args.operands}")
    t_gen = time.time() - t0
    prob = binding.DeviceProblem(w, q, k, v, prior)
    torch.cuda.synchronize()
    if args.layer_slices > 1:
        sliced = LayerSlices(prob, binding, args.layer_slices)
        for _ in range(args.warmup):
            sliced.compress()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(args.steps):
            sliced.compress()
        ev1.record()
        torch.cuda.synchronize()
        got = [t.clone() for t in (prob.idx, prob.k_out, prob.v_out)]
        prob.compress(); torch.cuda.synchronize()
        same = all(torch.equal(a_, b_) for a_, b_ in zip(got, (prob.idx, prob.k_out, prob.v_out)))
        print(json.dumps({"experiment": "layer slices", "workload": w.name, "layer_slices": args.layer_slices,
                          "layers_per_slice": w.n_layers // args.layer_slices, "steps": args.steps,
                          "ms_per_step": round(ev0.elapsed_time(ev1) / args.steps, 4),
                          "outputs_equal_the_unsliced_call": bool(same)}))
        return 0 if same else 4

    # Order of the measurement legs: what this GPU sustains (peaks), a long window of fused calls, then the W warm-up
    # steps and the K timed steps of the fused call (the headline figure), then the per-kernel durations.  The chip's
    # shader, fabric and memory clocks come up from idle over some tens of milliseconds of load: taken on an idle chip
    # with a handful of warm-up steps, 20 timed steps read 8-10 % slower than the same steps a moment later.  With the
    # first two legs in front, every figure of the line is taken in the working state; both windows are printed.
    peaks_now = None
    if not args.no_peaks:
        from paper_2604_10235_amd import peaks
        peaks.measure()                           # the first measurement also pays for the set-up
        peaks_now = peaks.measure()
        peaks.release()
    # a long window of fused calls (reported as ms_per_step_long_window, never used for `value`)
    prob.compress()                               # first call: module load, occupancy queries
    long_steps = max(200, args.steps)
    ev_s0, ev_s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev_s0.record()
    for _ in range(long_steps):
        prob.compress()
    ev_s1.record()
    torch.cuda.synchronize()
    ms_per_step_long = ev_s0.elapsed_time(ev_s1) / long_steps
    for _ in range(args.warmup):
        prob.compress()
    torch.cuda.synchronize()
    # the timed region: K fused calls back to back, bracketed by two events on the stream the kernels run on
    # (torch's current stream) and, outside them, by the host clock around a synchronisation
    ev_begin, ev_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev_begin.record()
    for _ in range(args.steps):
        prob.compress()
    ev_end.record()
    torch.cuda.synchronize()
    ms_per_step_host = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = ev_begin.elapsed_time(ev_end) / args.steps
    # per-kernel durations: the same kernels enqueued one by one with events between them, all steps
    # back to back like the fused loop above (one synchronisation at the end: same clocks, same heat)
    names = ["score_row_stats", "score_row_merge", "score_mass", "score_finish", "select", "gather"]
    stages = [binding.STAGE_ROW_STATS, binding.STAGE_ROW_MERGE, binding.STAGE_MASS, binding.STAGE_FINISH]
    acc = dict.fromkeys(names, 0.0)
    all_ev = []
    for _ in range(args.steps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)]
        ev[0].record()
        for i, st in enumerate(stages):
            prob.score_stages(st)
            ev[i + 1].record()
        prob.select(); ev[5].record()
        prob.gather(); ev[6].record()
        all_ev.append(ev)
    torch.cuda.synchronize()
    for ev in all_ev:
        for i, nm in enumerate(names):
            acc[nm] += ev[i].elapsed_time(ev[i + 1])
    stage_ms = {nm: acc[nm] / args.steps for nm in names}

    T, L = w.total_tokens, w.n_layers
    value = T * L / (ms_per_step * 1e-3)
    ab = algorithmic_bytes(w, 1 if args.kv_dtype == "fp8_e4m3" else 2)
    hbm_gbs = ab["total"] / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: one of the two MFMA passes; flops of one launch = 2 * R * sum(N_r) * d per (layer, KV head)
    dom = max(("score_row_stats", "score_mass"), key=lambda n: stage_ms[n])
    flops = 2.0 * w.group * w.window * T * w.head_dim * w.n_kv_heads * L
    achieved = flops / (stage_ms[dom] * 1e-3) / 1e12
    traffic = read_traffic(w.name if args.kv_dtype == "bf16" else f"{w.name}_{args.kv_dtype}")
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "traffic": None if not traffic else traffic.get(f"{dom}_hbm_bytes_per_launch"),
                "traffic_source": None if not traffic else {k_: traffic.get(k_) for k_ in ("file", "commit", "date")},
                "kernel_ms": round(stage_ms[dom], 4), "flop_per_launch": flops}
    logits = float(w.group * w.window * T * w.n_kv_heads * L)

    out = {
        "metric": "KV tokens scored+selected+gathered/sec per GPU; HBM GB/s as % of peak",
        "value": round(value, 1), "unit": "token-layers/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_host": round(ms_per_step_host, 4),
        "ms_per_step_long_window": round(ms_per_step_long, 4), "long_window_steps": long_steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.kv_dtype, "data": "synthetic",
        "config": {"workload": w.name if args.kv_dtype == "bf16" else f"{w.name} with an {args.kv_dtype} cache", "n_layers": L, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "tokens": T, "n_seqs": w.n_seqs, "window": w.window,
                   "budget_total": w.total_budget, "pool_kernel": w.pool_kernel, "prior_weight": w.prior_weight},
        "tokens_per_s_whole_model": round(T / (ms_per_step * 1e-3), 1),
        "hbm": {"algorithmic_bytes": ab["total"], "gb_per_s": round(hbm_gbs, 1), "peak_gb_per_s": HBM_PEAK_GBS,
                "frac_of_peak": round(hbm_gbs / HBM_PEAK_GBS, 4)},
        "stage_ms": {k_: round(v_, 4) for k_, v_ in stage_ms.items()},
        "stage_ms_sum": round(sum(stage_ms.values()), 4),
        "roofline": roofline,
        "binding_roofline": binding_roofline(flops, logits, ab, ab["k_read"], ms_per_step, peaks_now),
        "peaks": {"spec": {"mfma_bf16_tflops": MFMA_BF16_PEAK_TFLOPS, "hbm_gb_per_s": HBM_PEAK_GBS,
                           "exp_per_s": EXP_PEAK_PER_S}, "measured": peaks_now},
        "input_generation_s": round(t_gen, 1),
    }

    if not args.no_cpu_baseline:
        from oracle import codecomp_oracle as orc
        from tests import parity_util as pu
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            blas_threads = None
        auto = int(1.5e12 // max(1.0, flops / L))
        nl = max(1, min(args.cpu_layers if args.cpu_layers > 0 else max(2, auto), L))
        layers = sorted(set(np.linspace(0, L - 1, nl).round().astype(int).tolist()))   # always layer 0 and L-1
        cu, cb = w.cu_seqlens(), w.cu_budgets()
        t0, c0 = time.perf_counter(), time.process_time()
        sc_ref, idx_ref, ko_ref, vo_ref = orc.compress_packed(q[layers], k[layers], v[layers], prior, cu, cb,
                                                             window=w.window, pool_kernel=w.pool_kernel,
                                                             prior_weight=w.prior_weight, k_format=args.kv_dtype)
        t_cpu, c_cpu = time.perf_counter() - t0, time.process_time() - c0
        # cores = CPU time / wall time of the oracle run: only its matrix products run on the BLAS thread pool, the
        # exponentials, sums and sorts are single-threaded numpy
        out["cpu_baseline"] = {"value": round(T * len(layers) / t_cpu, 1), "unit": "token-layers/s",
                               "cores": max(1, round(c_cpu / t_cpu)), "cpu_seconds": round(c_cpu, 2),
                               "blas_threads": blas_threads, "kind": "oracle", "seconds": round(t_cpu, 2),
                               "sample": f"{len(layers)} of {L} layers (all heads, all requests) of the same inputs"}
        # parity report on the sampled layers (the GPU results are those of the timed fused call)
        prob.compress(); torch.cuda.synchronize()
        sc = prob.scores[layers].cpu().numpy()
        idx = prob.idx[layers].cpu().numpy()
        worst = pu.assert_scores_close(sc, sc_ref)
        ndiff = 0
        for li in range(len(layers)):
            for h in range(w.n_kv_heads):
                for r in range(w.n_seqs):
                    ndiff += pu.assert_index_sets_match(idx[li, h, cb[r]:cb[r + 1]], idx_ref[li, h, cb[r]:cb[r + 1]],
                                                        sc_ref[li, h, cu[r]:cu[r + 1]], w.window)
        ko = binding.DeviceProblem.bits(prob.k_out[layers]); vo = binding.DeviceProblem.bits(prob.v_out[layers])
        exact = bool(np.array_equal(ko, pu.host_gather(k[layers], idx, cu, cb)) and
                     np.array_equal(vo, pu.host_gather(v[layers], idx, cu, cb)))
        out["parity"] = {"layers_checked": len(layers), "max_rel_score_err": float(f"{worst:.3e}"),
                         "tie_band_index_diffs": int(ndiff), "gather_bit_exact": exact}
        if not exact:
            print(json.dumps(out))
            return 4
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
