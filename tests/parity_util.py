"""Comparison protocol between the HIP path and the CPU oracle (used by the GPU tests, the
smoke check and the benchmark's parity report)."""
from __future__ import annotations

import numpy as np

SCORE_RTOL = 1e-3          # acceptance: scores within 1e-3 relative of the fp64 oracle
BAND_RTOL = 2e-3           # index sets may differ only among tokens this close to the cut score


def assert_scores_close(gpu: np.ndarray, ref: np.ndarray, what: str = "scores"):
    gpu = np.asarray(gpu, dtype=np.float64)
    err = np.abs(gpu - ref)
    tol = SCORE_RTOL * np.abs(ref) + 1e-30
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err / tol), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} outside {SCORE_RTOL:g} relative; worst at {i}: "
                             f"gpu={gpu[i]!r} ref={ref[i]!r}")
    return float((err / (np.abs(ref) + 1e-300)).max())


def check_index_invariants(idx_row: np.ndarray, n: int, window: int, budget: int):
    assert idx_row.shape == (budget,)
    assert idx_row.min() >= 0 and idx_row.max() < n
    assert (np.diff(idx_row.astype(np.int64)) > 0).all(), "indices must be strictly ascending"
    assert np.array_equal(idx_row[budget - window:], np.arange(n - window, n)), "window must be kept"


def assert_index_sets_match(idx_gpu: np.ndarray, idx_ref: np.ndarray, ref_scores: np.ndarray, window: int,
                            what: str = "idx"):
    """idx_* [B] for one (layer, head, request); ref_scores float64 [N] of the oracle."""
    n = ref_scores.shape[0]
    b = idx_ref.shape[0]
    check_index_invariants(idx_gpu, n, window, b)
    if b == window:
        return 0
    sg, sr = set(idx_gpu.tolist()), set(idx_ref.tolist())
    diff = sorted(sg ^ sr)
    if diff:
        pre = ref_scores[: n - window]
        tau = np.sort(pre)[::-1][b - window - 1]
        off = [j for j in diff if abs(ref_scores[j] - tau) > BAND_RTOL * abs(tau)]
        assert not off, f"{what}: {len(off)} differing indices lie outside the tie band around tau={tau!r}: {off[:8]}"
    return len(diff)


def host_gather(k_bits: np.ndarray, idx: np.ndarray, cu_seqlens, cu_budgets) -> np.ndarray:
    """Row copy with the GIVEN indices (plain numpy indexing; used to check the gather bit for bit
    against the indices the GPU itself selected)."""
    n_layers, h, _, d = k_bits.shape
    out = np.empty((n_layers, h, int(cu_budgets[-1]), d), dtype=k_bits.dtype)
    for r in range(len(cu_seqlens) - 1):
        a = int(cu_seqlens[r]); oa, ob = int(cu_budgets[r]), int(cu_budgets[r + 1])
        sel = idx[:, :, oa:ob].astype(np.int64) + a
        out[:, :, oa:ob] = np.take_along_axis(k_bits, sel[..., None], axis=2)
    return out
