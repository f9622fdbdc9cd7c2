"""The pins are only worth something if a plausible mistake in the oracle fails one of them.
Each case plants one mistake in a copy of an oracle function (on the CPU, never in the HIP path)
and checks that the pin suite notices."""
import math

import numpy as np
import pytest

from oracle import codecomp_oracle as orc
from tests import test_oracle_pins as pins


def _pins_for_mass():
    pins.test_rational_golden_fixture()
    pins.test_two_keys_is_a_logistic()
    pins.test_single_row_is_library_softmax()
    pins.test_mass_sums_to_window(6, 2, 5, 33, 16)
    pins.test_identical_or_zero_keys_give_uniform_mass()
    pins.test_shift_invariance_and_permutation()
    pins.test_group_is_mean_over_query_heads()
    pins.test_head_mapping_is_contiguous()
    pins.test_brute_force_python_loops()


def _pins_for_pool():
    pins.test_pool_matches_library_avg_pool(7, 40)
    pins.test_pool_matches_library_avg_pool(5, 6)
    pins.test_pool_uniform_edges_closed_form()
    pins.test_pool_identity_and_mass_loss()


def _pins_for_select():
    pins.test_select_invariants_random()
    pins.test_select_exhaustive_enumeration()
    pins.test_select_matches_library_topk_without_ties()
    pins.test_select_ties_go_to_lower_index()
    pins.test_binary_prior_large_weight_keeps_flagged_first()


def _mass(q_obs, k, scale, *, group_sum=False, softmax_axis=1, interleaved_heads=False, transpose=False):
    h_q, w, d = q_obs.shape
    h_kv, n, _ = k.shape
    g = h_q // h_kv
    u = np.zeros((h_kv, n))
    for hq in range(h_q):
        kv = hq % h_kv if interleaved_heads else hq // g
        s = (q_obs[hq] @ k[kv].T) * scale
        if transpose:
            s = -s
        s = s - s.max(axis=softmax_axis, keepdims=True)
        e = np.exp(s)
        a = e / e.sum(axis=softmax_axis, keepdims=True)
        u[kv] += a.sum(axis=0)
    return u if group_sum else u / g


MASS_MUTANTS = {
    "scale 1/d": lambda q, k, scale=None, **kw: _mass(q, k, 1.0 / q.shape[-1]),
    "no scale": lambda q, k, scale=None, **kw: _mass(q, k, 1.0),
    "sum over the group": lambda q, k, scale=None, **kw: _mass(q, k, 1 / math.sqrt(q.shape[-1]), group_sum=True),
    "softmax over queries": lambda q, k, scale=None, **kw: _mass(q, k, 1 / math.sqrt(q.shape[-1]), softmax_axis=0),
    "interleaved head mapping": lambda q, k, scale=None, **kw: _mass(q, k, 1 / math.sqrt(q.shape[-1]), interleaved_heads=True),
    "negated logits": lambda q, k, scale=None, **kw: _mass(q, k, 1 / math.sqrt(q.shape[-1]), transpose=True),
}


@pytest.mark.parametrize("name", sorted(MASS_MUTANTS))
def test_attention_mass_mutants_are_caught(name, monkeypatch):
    _pins_for_mass()                                   # the real oracle passes
    monkeypatch.setattr(orc, "window_attention_mass", MASS_MUTANTS[name])
    with pytest.raises(AssertionError):
        _pins_for_mass()


def _pool(u, kernel, *, divisor="k", shift=0):
    half = (kernel - 1) // 2
    n = u.shape[-1]
    out = np.zeros_like(u, dtype=np.float64)
    cnt = np.zeros(n)
    for delta in range(-half + shift, half + 1 + shift):
        lo, hi = max(0, -delta), min(n, n - delta)
        if hi > lo:
            out[..., lo:hi] += u[..., lo + delta:hi + delta]
            cnt[lo:hi] += 1
    return out / (kernel if divisor == "k" else cnt)


POOL_MUTANTS = {
    "divide by the covered count": lambda u, k, extent=None: _pool(u, k, divisor="count"),
    "window shifted by one": lambda u, k, extent=None: _pool(u, k, shift=1),
    "no pooling": lambda u, k, extent=None: u.astype(np.float64),
}


@pytest.mark.parametrize("name", sorted(POOL_MUTANTS))
def test_pool_mutants_are_caught(name, monkeypatch):
    _pins_for_pool()
    monkeypatch.setattr(orc, "average_pool", POOL_MUTANTS[name])
    with pytest.raises(AssertionError):
        _pins_for_pool()


def _select(scores, window, budget, *, ascending=False, tie_high=False, keep_window=True, unsorted=False):
    h, n = scores.shape
    take = budget - window
    out = np.empty((h, budget), dtype=np.int64)
    for i in range(h):
        pre = scores[i, : n - window] if keep_window else scores[i]
        key = pre if ascending else -pre
        if tie_high:
            order = np.argsort(key[::-1], kind="stable")
            order = len(pre) - 1 - order
        else:
            order = np.argsort(key, kind="stable")
        if keep_window:
            chosen = order[:take]
            chosen = chosen if unsorted else np.sort(chosen)
            out[i] = np.concatenate([chosen, np.arange(n - window, n)])
        else:
            out[i] = np.sort(order[:budget])
    return out


SELECT_MUTANTS = {
    "keeps the smallest": lambda s, w, b: _select(s, w, b, ascending=True),
    "ties to the higher index": lambda s, w, b: _select(s, w, b, tie_high=True),
    "window not forced": lambda s, w, b: _select(s, w, b, keep_window=False),
    "rank order instead of ascending": lambda s, w, b: _select(s, w, b, unsorted=True),
}


@pytest.mark.parametrize("name", sorted(SELECT_MUTANTS))
def test_select_mutants_are_caught(name, monkeypatch):
    _pins_for_select()
    monkeypatch.setattr(orc, "select", SELECT_MUTANTS[name])
    with pytest.raises(AssertionError):
        _pins_for_select()


def test_prior_sign_mutant_is_caught(monkeypatch):
    pins.test_prior_weight_zero_and_linearity()
    monkeypatch.setattr(orc, "fuse_prior", lambda pooled, prior, lam: pooled - lam * np.asarray(prior)[None, :])
    with pytest.raises(AssertionError):
        pins.test_prior_weight_zero_and_linearity()


_FP8_TRUE = orc.fp8_e4m3_to_f64

FP8_MUTANTS = {
    "bias 8": lambda c: _FP8_TRUE(c) / 2,
    "no subnormals": lambda c: np.where(((np.asarray(c) >> 3) & 0xF) == 0, 0.0, _FP8_TRUE(c)),
    "E5M2 layout": lambda c: np.where(np.asarray(c) & 0x80, -1.0, 1.0) *
    np.ldexp(1 + (np.asarray(c) & 3) / 4.0, ((np.asarray(c).astype(np.int64) >> 2) & 31) - 15),
    "top exponent is infinity": lambda c: np.where(((np.asarray(c) >> 3) & 0xF) == 15, np.inf, _FP8_TRUE(c)),
    "sign ignored": lambda c: np.abs(_FP8_TRUE(c)),
}


@pytest.mark.parametrize("name", sorted(FP8_MUTANTS))
def test_fp8_decoder_mutants_are_caught(name, monkeypatch):
    monkeypatch.setattr(orc, "fp8_e4m3_to_f64", FP8_MUTANTS[name])
    with pytest.raises(AssertionError):
        pins.test_fp8_e4m3_decoder_matches_library_and_format_constants()
