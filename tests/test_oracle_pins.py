"""Pins of the CPU oracle against what the paper's equations and plain mathematics fix:
closed forms, invariants, special cases that reduce to library routines, and exhaustive
search on tiny inputs.  None of these re-types the oracle's own formula."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import codecomp_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(20260410)


def rand_qk(h_q, h_kv, w, n, d, seed=0):
    g = np.random.default_rng(seed)
    return g.standard_normal((h_q, w, d)), g.standard_normal((h_kv, n, d))


# ------------------------------------------------------------------ bf16 widening

def test_bf16_widening_matches_torch():
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    ours = orc.bf16_bits_to_f64(bits)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    finite = np.isfinite(ref)
    assert np.array_equal(ours[finite], ref[finite])
    assert np.array_equal(np.isnan(ours), np.isnan(ref))


# ------------------------------------------------------------------ attention mass (eq. of the compression section)

def test_rational_golden_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "softmax_rational.txt")) if not l.startswith("#")]
    a = np.array([float(r[0]) for r in rows]); b = np.array([float(r[1]) for r in rows])
    expect = np.array([int(r[2]) / int(r[3]) for r in rows])
    q = np.zeros((1, 2, 4)); q[0, 0, 0] = 2.0; q[0, 1, 1] = 2.0
    k = np.zeros((1, 3, 4)); k[0, :, 0] = np.log(a); k[0, :, 1] = np.log(b)
    u = orc.window_attention_mass(q, k)
    np.testing.assert_allclose(u[0], expect, rtol=1e-14)


def test_two_keys_is_a_logistic():
    # N = 2, W = 1: A(1, 0) = 1 / (1 + exp(-(q.k0 - q.k1)/sqrt(d))): pins the sign and the 1/sqrt(d) scale.
    d = 16
    q = np.zeros((1, 1, d)); q[0, 0, 3] = 1.5
    k = np.zeros((1, 2, d)); k[0, 0, 3] = 2.0; k[0, 1, 3] = -1.0
    u = orc.window_attention_mass(q, k)
    p0 = 1.0 / (1.0 + math.exp(-(1.5 * 3.0) / math.sqrt(d)))
    np.testing.assert_allclose(u[0], [p0, 1 - p0], rtol=1e-14)


def test_single_row_is_library_softmax():
    # W = 1, G = 1, k = 1, lambda = 0: the score row is one textbook softmax row.
    from scipy.special import softmax
    q, k = rand_qk(1, 1, 1, 50, 8, seed=1)
    sc = orc.score(q, k, np.zeros(50), pool_kernel=1, prior_weight=0.0)
    ref = softmax((k[0] @ q[0, 0]) / math.sqrt(8))
    np.testing.assert_allclose(sc[0], ref, rtol=1e-13)


@pytest.mark.parametrize("h_q,h_kv,w,n,d", [(4, 4, 3, 17, 8), (6, 2, 5, 33, 16), (8, 1, 2, 9, 4)])
def test_mass_sums_to_window(h_q, h_kv, w, n, d):
    q, k = rand_qk(h_q, h_kv, w, n, d, seed=2)
    u = orc.window_attention_mass(q, k)
    np.testing.assert_allclose(u.sum(axis=1), np.full(h_kv, float(w)), rtol=1e-12)
    assert (u > 0).all()


def test_identical_or_zero_keys_give_uniform_mass():
    q, _ = rand_qk(6, 2, 4, 1, 8, seed=3)
    n, w = 40, 4
    row = RNG.standard_normal(8)
    for k in (np.zeros((2, n, 8)), np.tile(row, (2, n, 1))):
        u = orc.window_attention_mass(q, k)
        np.testing.assert_allclose(u, np.full((2, n), w / n), rtol=1e-13)


def test_shift_invariance_and_permutation():
    q, k = rand_qk(4, 2, 3, 21, 8, seed=4)
    u = orc.window_attention_mass(q, k)
    shift = RNG.standard_normal(8)
    np.testing.assert_allclose(orc.window_attention_mass(q, k + shift), u, rtol=1e-11)
    perm = RNG.permutation(21)
    np.testing.assert_allclose(orc.window_attention_mass(q, k[:, perm]), u[:, perm], rtol=1e-12)


def test_dominant_key_takes_whole_window():
    # every window query is q0; key 5 is strongly aligned with q0, all others are orthogonal
    d, n, w = 8, 12, 3
    q = np.zeros((1, w, d)); q[0, :, 0] = 1.0
    k = np.zeros((1, n, d)); k[0, :, 1] = RNG.standard_normal(n)
    k[0, 5, 0] = 400.0
    u = orc.window_attention_mass(q, k)
    assert abs(u[0, 5] - w) < 1e-12
    assert u[0, np.arange(n) != 5].max() < 1e-50


def test_large_logits_do_not_overflow():
    q = np.full((1, 2, 4), 300.0); k = np.full((1, 5, 4), 300.0); k[0, 2] *= 1.001
    u = orc.window_attention_mass(q, k)
    assert np.isfinite(u).all() and abs(u.sum() - 2) < 1e-12


def test_group_is_mean_over_query_heads():
    # duplicating every query head G times must not change u (mean, not sum, over the group)
    q, k = rand_qk(2, 2, 3, 19, 8, seed=5)
    u1 = orc.window_attention_mass(q, k)
    q3 = np.repeat(q, 3, axis=0)                      # heads [0,0,0,1,1,1]: contiguous grouping
    np.testing.assert_allclose(orc.window_attention_mass(q3, k), u1, rtol=1e-13)
    # and two different heads in one group average their masses
    qa, ka = rand_qk(2, 1, 3, 19, 8, seed=6)
    both = orc.window_attention_mass(qa, ka)
    sep = 0.5 * (orc.window_attention_mass(qa[:1], ka) + orc.window_attention_mass(qa[1:], ka))
    np.testing.assert_allclose(both, sep, rtol=1e-13)


def test_head_mapping_is_contiguous():
    # query head h_q must read KV head h_q // G: make KV head 1 have a dominant key only for q heads 2,3
    d, n = 4, 6
    q = np.zeros((4, 1, d)); q[:, 0, 0] = 1.0
    k = np.zeros((2, n, d)); k[0, 1, 0] = 300.0; k[1, 4, 0] = 300.0
    u = orc.window_attention_mass(q, k)
    assert abs(u[0, 1] - 1) < 1e-12 and abs(u[1, 4] - 1) < 1e-12


def test_brute_force_python_loops():
    # the defining double sum written with scalar loops and math.exp on a tiny case
    q, k = rand_qk(4, 2, 2, 7, 4, seed=7)
    u = orc.window_attention_mass(q, k)
    for h in range(2):
        for j in range(7):
            tot = 0.0
            for g in range(2):
                for t in range(2):
                    logits = [sum(q[h * 2 + g, t, c] * k[h, jj, c] for c in range(4)) / 2.0 for jj in range(7)]
                    z = sum(math.exp(x) for x in logits)
                    tot += math.exp(logits[j]) / z
            assert abs(u[h, j] - tot / 2) < 1e-13


# ------------------------------------------------------------------ pooling

@pytest.mark.parametrize("kernel", [1, 3, 5, 7, 9])
@pytest.mark.parametrize("n", [1, 2, 6, 40])
def test_pool_matches_library_avg_pool(kernel, n):
    u = RNG.random((3, n))
    ref = torch.nn.functional.avg_pool1d(torch.from_numpy(u)[None], kernel, stride=1, padding=(kernel - 1) // 2,
                                         count_include_pad=True)[0].numpy()
    np.testing.assert_allclose(orc.average_pool(u, kernel), ref, rtol=1e-13, atol=1e-16)


def test_pool_uniform_edges_closed_form():
    n, w, kernel = 50, 4, 7
    u = np.full((1, n), w / n)
    p = orc.average_pool(u, kernel)[0]
    half = 3
    np.testing.assert_allclose(p[half:n - half], w / n, rtol=1e-14)
    for e in range(half):      # e = distance from the end: k - half + e terms fall inside
        expect = (w / n) * (kernel - half + e) / kernel
        np.testing.assert_allclose([p[e], p[n - 1 - e]], expect, rtol=1e-14)


def test_pool_identity_and_mass_loss():
    u = RNG.random((2, 30))
    assert np.array_equal(orc.average_pool(u, 1), u)
    k = 5
    p = orc.average_pool(u, k)
    # every u[j] is counted once per window that covers it: k times in the interior, fewer near the ends
    cover = np.array([min(j, 2) + min(29 - j, 2) + 1 for j in range(30)])
    np.testing.assert_allclose(p.sum(axis=1), (u * cover).sum(axis=1) / k, rtol=1e-13)


# ------------------------------------------------------------------ prior fusion

def test_prior_weight_zero_and_linearity():
    q, k = rand_qk(4, 2, 3, 31, 8, seed=8)
    prior = (RNG.random(31) < 0.3).astype(np.float64) * RNG.random(31)
    base = orc.score(q, k, prior, pool_kernel=5, prior_weight=0.0)
    np.testing.assert_allclose(base, orc.average_pool(orc.window_attention_mass(q, k), 5), rtol=0, atol=0)
    for lam in (0.5, 2.0):
        c = orc.score(q, k, prior, pool_kernel=5, prior_weight=lam)
        np.testing.assert_allclose(c - base, np.tile(lam * prior, (2, 1)), rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------------ selection

def check_invariants(idx, scores, w, b):
    h, n = scores.shape
    assert idx.shape == (h, b)
    for i in range(h):
        row = idx[i]
        assert (np.diff(row) > 0).all()
        assert row[0] >= 0 and row[-1] == n - 1
        assert np.array_equal(row[b - w:], np.arange(n - w, n))
        kept = np.zeros(n, bool); kept[row] = True
        pre = scores[i, : n - w]
        if b > w and (~kept[: n - w]).any():
            assert pre[~kept[: n - w]].max() <= pre[kept[: n - w]].min()


def test_select_invariants_random():
    for seed in range(5):
        g = np.random.default_rng(seed)
        n = int(g.integers(8, 200)); w = int(g.integers(1, 8)); b = int(g.integers(w, n + 1))
        sc = g.random((3, n))
        check_invariants(orc.select(sc, w, b), sc, w, b)


def test_select_exhaustive_enumeration():
    # the chosen prefix set maximises the total score over all subsets of its size; with distinct
    # scores that maximiser is unique
    g = np.random.default_rng(11)
    n, w, b = 11, 2, 6
    sc = g.random((1, n))
    idx = orc.select(sc, w, b)[0]
    best = max(itertools.combinations(range(n - w), b - w), key=lambda s: sum(sc[0, j] for j in s))
    assert sorted(best) == list(idx[: b - w])


def test_select_matches_library_topk_without_ties():
    g = np.random.default_rng(12)
    n, w, b = 500, 16, 100
    sc = g.random((4, n))
    idx = orc.select(sc, w, b)
    top = torch.topk(torch.from_numpy(sc[:, : n - w]), b - w, dim=1).indices.numpy()
    for i in range(4):
        assert set(idx[i, : b - w]) == set(top[i])


def test_select_ties_go_to_lower_index():
    sc = np.array([[0.5, 0.7, 0.5, 0.5, 0.7, 0.5, 0.1, 0.1]])
    # W = 2 keeps {6, 7}; B - W = 4 from prefix: both 0.7 (1, 4) then the first two 0.5 (0, 2)
    assert list(orc.select(sc, 2, 6)[0]) == [0, 1, 2, 4, 6, 7]
    assert list(orc.select(sc, 2, 2)[0]) == [6, 7]                    # B == W: window only
    assert list(orc.select(sc, 2, 8)[0]) == list(range(8))           # B == N: identity


def test_binary_prior_large_weight_keeps_flagged_first():
    g = np.random.default_rng(13)
    q, k = rand_qk(2, 2, 4, 120, 8, seed=14)
    n, w = 120, 4
    prior = (g.random(n) < 0.2).astype(np.float64)
    att = orc.score(q, k, prior, pool_kernel=3, prior_weight=0.0)
    lam = 10.0 * att.max()
    sc = orc.score(q, k, prior, pool_kernel=3, prior_weight=lam)
    flagged = np.flatnonzero(prior[: n - w] > 0)
    f = len(flagged)
    # budget with room for all flagged: all flagged kept, the rest = attention top among unflagged
    b = w + f + 7
    idx = orc.select(sc, w, b)
    for h in range(2):
        chosen = set(idx[h, : b - w])
        assert set(flagged) <= chosen
        unfl = np.setdiff1d(np.arange(n - w), flagged)
        best_unfl = unfl[np.argsort(-att[h, unfl], kind="stable")[:7]]
        assert chosen - set(flagged) == set(best_unfl)
    # budget smaller than the flagged set: only flagged kept, the attention-top among them
    b2 = w + f - 3
    idx2 = orc.select(sc, w, b2)
    for h in range(2):
        chosen = set(idx2[h, : b2 - w])
        assert chosen <= set(flagged)
        best_fl = flagged[np.argsort(-att[h, flagged], kind="stable")[: f - 3]]
        assert chosen == set(best_fl)


def test_flagged_retention_monotone_in_prior_weight():
    g = np.random.default_rng(15)
    q, k = rand_qk(4, 2, 4, 200, 8, seed=16)
    prior = (g.random(200) < 0.25).astype(np.float64)
    kept_prev = np.zeros(2)
    for lam in (0.0, 0.01, 0.05, 0.2, 1.0, 100.0):
        sc = orc.score(q, k, prior, pool_kernel=5, prior_weight=lam)
        idx = orc.select(sc, 4, 40)
        kept = np.array([prior[idx[h, :36]].sum() for h in range(2)])
        assert (kept >= kept_prev).all()
        kept_prev = kept


# ------------------------------------------------------------------ gather / packed wrappers

def test_gather_is_a_row_copy():
    g = np.random.default_rng(17)
    k = g.integers(0, 1 << 16, size=(3, 20, 8), dtype=np.uint16)
    v = g.integers(0, 1 << 16, size=(3, 20, 8), dtype=np.uint16)
    idx = np.stack([np.sort(g.choice(20, 6, replace=False)) for _ in range(3)])
    ko, vo = orc.gather(k, v, idx)
    np.testing.assert_array_equal(ko, np.take_along_axis(k, idx[:, :, None], axis=1))
    np.testing.assert_array_equal(vo, np.take_along_axis(v, idx[:, :, None], axis=1))
    full = np.tile(np.arange(20), (3, 1))
    ko, vo = orc.gather(k, v, full)
    assert np.array_equal(ko, k) and np.array_equal(vo, v)


def test_packed_requests_and_layers_are_independent():
    # a ragged batch must give, per (layer, request), exactly what that request gives alone
    from paper_2604_10235_amd import workloads as wl
    w = wl.scaled(wl.ragged_agentic(), seqlens=[90, 41, 133], budgets=[20, 9, 30], window=8, n_layers=2,
                  n_q_heads=4, n_kv_heads=2, head_dim=16)
    q, k, v, prior = wl.make_all(w)
    cu, cb = w.cu_seqlens(), w.cu_budgets()
    sc, idx, ko, vo = orc.compress_packed(q, k, v, prior, cu, cb, window=w.window, pool_kernel=w.pool_kernel,
                                          prior_weight=w.prior_weight)
    for l in range(2):
        for r in range(3):
            a, b = cu[r], cu[r + 1]
            alone = orc.score(orc.bf16_bits_to_f64(q[l, r]), orc.bf16_bits_to_f64(k[l, :, a:b]), prior[a:b],
                              pool_kernel=w.pool_kernel, prior_weight=w.prior_weight)
            assert np.array_equal(alone, sc[l, :, a:b])
            sel = orc.select(alone, w.window, w.budgets[r])
            assert np.array_equal(sel, idx[l, :, cb[r]:cb[r + 1]])
            for h in range(2):
                assert np.array_equal(ko[l, h, cb[r]:cb[r + 1]], k[l, h, a:b][sel[h]])
                assert np.array_equal(vo[l, h, cb[r]:cb[r + 1]], v[l, h, a:b][sel[h]])
    # scores of the tiny synthetic recipe have the expected magnitudes: mass W per head before pooling
    u = orc.window_attention_mass(orc.bf16_bits_to_f64(q[0, 0]), orc.bf16_bits_to_f64(k[0, :, :90]))
    np.testing.assert_allclose(u.sum(axis=1), 8.0, rtol=1e-12)


# ------------------------------------------------------------------ budgets (eq. of the budget-allocation section)

def test_log_norm_closed_forms():
    # Norm(0) = 0, Norm(tau) = 1, saturates above tau, Norm(sqrt(1+tau)-1) = 1/2
    tau = 15.0
    np.testing.assert_allclose(orc.log_norm([0.0, tau, 10 * tau, math.sqrt(1 + tau) - 1], tau), [0, 1, 1, 0.5], atol=1e-15)
    s = orc.chunk_structure_score([[0, 15.0], [15.0, 0]], [15.0, 15.0], [0.25, 0.75])
    np.testing.assert_allclose(s, [0.75, 0.25], atol=1e-15)


def test_budgets_closed_forms():
    lens = np.array([1000, 2000, 512])
    # all scores equal -> normalised score 0.5 -> multiplier midway -> B = floor(len * r * 1.0)
    b = orc.chunk_budgets([3.0, 3.0, 3.0], lens, ratio=0.4, m_min=0.5, m_max=1.5, r_max=1.0, eps=1e-6)
    assert list(b) == [400, 800, 204]
    # extremes get m_min / m_max, the middle one interpolates linearly
    b = orc.chunk_budgets([0.0, 1.0, 0.5], lens, ratio=0.4, m_min=0.5, m_max=1.5, r_max=1.0, eps=1e-6)
    assert list(b) == [200, 1200, math.floor(512 * 0.4)]
    # the cap r_max binds
    b = orc.chunk_budgets([0.0, 1.0], [1000, 1000], ratio=0.6, m_min=0.5, m_max=1.5, r_max=0.8, eps=1e-6)
    assert list(b) == [300, 800]
    # a spread below eps is divided by eps, not by itself
    b = orc.chunk_budgets([0.0, 1e-9], [1000, 1000], ratio=0.5, m_min=0.5, m_max=1.5, r_max=1.0, eps=1e-6)
    assert list(b) == [250, math.floor(1000 * 0.5 * (0.5 + 1e-3))]
    # monotone in sigma
    g = np.random.default_rng(3)
    sig = g.random(20); ln = np.full(20, 4096)
    b = orc.chunk_budgets(sig, ln, ratio=0.4, m_min=0.5, m_max=1.5, r_max=1.0, eps=1e-6)
    assert (np.diff(b[np.argsort(sig)]) >= 0).all()


def test_structure_score_closed_forms():
    prior = np.array([0, 1, 1, 0, 0.5, 0, 0, 2.0])
    idx = np.array([[1, 2, 6, 7], [0, 3, 5, 6], [1, 2, 4, 7]])
    np.testing.assert_allclose(orc.structure_score(idx, prior, 8), [0.75, 0.0, 1.0])
    assert np.isnan(orc.structure_score(idx, np.zeros(8), 8)).all()


# ------------------------------------------------------------------ two-stage rule (structure first, attention fills)

def test_span_budget_closed_forms():
    assert orc.span_budget(100, 0.5, 0) == 50
    assert orc.span_budget(100, 0.5, 70) == 70        # the minimum binds
    assert orc.span_budget(100, 0.5, 170) == 100      # never more than the budget itself
    assert orc.span_budget(101, 0.5, 0) == 50         # floor
    assert orc.span_budget(100, 0.0, 0) == 0


def test_two_stage_hand_example():
    # prefix of 8 tokens + window of 2; budget 7 -> 5 prefix slots; rho = 0.6 -> span budget 3
    pooled = np.array([[0.10, 0.90, 0.20, 0.80, 0.30, 0.70, 0.40, 0.60, 0.0, 0.0]])
    prior = np.array([0.0, 0.0, 1.0, 0.0, 2.0, 0.0, 1.0, 1.0, 5.0, 0.0])   # the window's own prior is ignored
    # stage 1: largest prior 4, then the ties at 1.0 in sequence order: 2, 6 (7 does not fit)
    # stage 2: two slots by attention among {0,1,3,5,7}: 1 (0.9), 3 (0.8)
    got = orc.select_two_stage(pooled, prior, 2, 7, span_ratio=0.6, span_min=0)
    assert list(got[0]) == [1, 2, 3, 4, 6, 8, 9]
    # a zero span budget is attention only; a full one with few marked tokens keeps them all
    assert np.array_equal(orc.select_two_stage(pooled, prior, 2, 7, span_ratio=0.0, span_min=0),
                          orc.select(pooled, 2, 7))
    got = orc.select_two_stage(pooled, prior, 2, 8, span_ratio=1.0, span_min=0)
    assert list(got[0]) == [1, 2, 3, 4, 6, 7, 8, 9]


def test_two_stage_equals_additive_limit_for_binary_prior():
    # binary prior, span budget = whole budget: "protected first, attention fills the rest" is the
    # lambda -> infinity limit of the additive reading as long as the marked tokens fit
    g = np.random.default_rng(21)
    q, k = rand_qk(4, 2, 4, 150, 8, seed=22)
    n, w = 150, 4
    prior = (g.random(n) < 0.15).astype(np.float64)
    att = orc.score(q, k, prior, pool_kernel=5, prior_weight=0.0)
    f = int((prior[: n - w] > 0).sum())
    b = w + f + 11
    two = orc.select_two_stage(att, prior, w, b, span_ratio=1.0, span_min=0)
    add = orc.select(orc.fuse_prior(att, prior, 100.0 * att.max()), w, b)
    assert np.array_equal(two, add)
    # more marked tokens than slots: the paper keeps the FIRST marked tokens in sequence, not the best attended
    b2 = w + f - 5
    two = orc.select_two_stage(att, prior, w, b2, span_ratio=1.0, span_min=0)
    marked = np.flatnonzero(prior[: n - w] > 0)
    for hh in range(2):
        assert list(two[hh, : b2 - w]) == list(marked[: f - 5])


def test_two_stage_invariants_and_optimality():
    g = np.random.default_rng(23)
    for trial in range(6):
        n = int(g.integers(20, 120)); w = int(g.integers(1, 6)); b = int(g.integers(w, n + 1))
        pooled = g.random((2, n)); prior = np.where(g.random(n) < 0.3, g.random(n), 0.0)
        rho = float(g.choice([0.0, 0.25, 0.5, 1.0])); bmin = int(g.integers(0, 5))
        idx = orc.select_two_stage(pooled, prior, w, b, span_ratio=rho, span_min=bmin)
        npre, bp = n - w, b - w
        marked = set(np.flatnonzero(prior[:npre] > 0).tolist())
        bs = orc.span_budget(bp, rho, bmin)
        for hh in range(2):
            row = idx[hh]
            assert (np.diff(row) > 0).all() and np.array_equal(row[bp:], np.arange(npre, n))
            chosen = set(row[:bp].tolist())
            # some set P of min(bs, |marked|) marked tokens is inside, every marked token left out of P has a
            # prior no larger than the smallest prior in P, and the rest is the attention top of the complement
            kept_marked = sorted(chosen & marked, key=lambda j: (-prior[j], j))
            npro = min(bs, len(marked))
            assert len(kept_marked) >= npro
            best = sorted(marked, key=lambda j: (-prior[j], j))[:npro]
            assert set(best) <= chosen
            rest = sorted(set(range(npre)) - set(best), key=lambda j: (-pooled[hh, j], j))[: bp - npro]
            assert chosen == set(best) | set(rest)


# ----------------------------------------------------------------------------------------
# variants of the score tail
# ----------------------------------------------------------------------------------------

def _rand_case(seed, h_q=6, h_kv=2, w=3, n=23, d=8):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((h_q, w, d)), rng.standard_normal((h_kv, n, d)), rng.random(n)


def test_group_sum_is_g_times_mean_and_max_is_the_largest_head():
    q, k, _ = _rand_case(1)
    mean = orc.window_attention_mass(q, k)
    np.testing.assert_allclose(orc.window_attention_mass(q, k, group_reduce="sum"), 3 * mean, rtol=1e-13)
    # per-head masses from single-head calls (G = 1 on a repeated KV head), then max by hand
    heads = np.stack([orc.window_attention_mass(q[h:h + 1], k[h // 3:h // 3 + 1])[0] for h in range(6)])
    np.testing.assert_allclose(orc.window_attention_mass(q, k, group_reduce="max"),
                               np.stack([heads[:3].max(axis=0), heads[3:].max(axis=0)]), rtol=1e-13)
    # identical query heads: mean == max, sum == G * max
    qq = np.repeat(q[:2], 3, axis=0)[[0, 1, 2, 3, 4, 5]]
    qq[0:3] = q[0]; qq[3:6] = q[1]
    np.testing.assert_allclose(orc.window_attention_mass(qq, k, group_reduce="max"), orc.window_attention_mass(qq, k), rtol=1e-13)


def test_prefix_softmax_is_the_full_softmax_on_truncated_keys():
    q, k, _ = _rand_case(2)
    n, w = k.shape[1], q.shape[1]
    u = orc.window_attention_mass(q, k, softmax_keys=n - w)
    np.testing.assert_allclose(u[:, :n - w], orc.window_attention_mass(q, k[:, :n - w]), rtol=1e-13)
    assert (u[:, n - w:] == 0).all()
    np.testing.assert_allclose(u.sum(axis=1), w, rtol=1e-12)          # all the mass sits on the prefix
    # uniform keys: W / (N - W) on the prefix
    uz = orc.window_attention_mass(q, np.zeros_like(k), softmax_keys=n - w)
    np.testing.assert_allclose(uz[:, :n - w], w / (n - w), rtol=1e-13)
    # through score(): same thing with lambda = 0 and no pooling
    sc = orc.score(q, k, np.zeros(n), pool_kernel=1, prior_weight=0.0, softmax_domain="prefix")
    np.testing.assert_allclose(sc, u, rtol=1e-13)
    # no prefix at all: nothing to attend to, all zero
    assert (orc.window_attention_mass(q, k[:, :w], softmax_keys=0) == 0).all()


@pytest.mark.parametrize("kernel,n", [(1, 9), (3, 10), (5, 17), (7, 7), (9, 4)])
def test_max_pool_matches_library_max_pool(kernel, n):
    rng = np.random.default_rng(kernel * 100 + n)
    u = rng.random((3, n))                       # masses are non-negative
    ref = torch.nn.functional.max_pool1d(torch.from_numpy(u)[None], kernel, stride=1, padding=(kernel - 1) // 2)[0].numpy()
    np.testing.assert_array_equal(orc.max_pool(u, kernel), ref)
    # monotone signal: the window maximum is the value (k-1)/2 places further on
    ramp = np.arange(n, dtype=np.float64)[None]
    np.testing.assert_array_equal(orc.max_pool(ramp, kernel)[0], np.minimum(np.arange(n) + (kernel - 1) // 2, n - 1))


@pytest.mark.parametrize("mode", ["avg", "max"])
def test_prefix_pooling_is_pooling_of_the_prefix_slice(mode):
    rng = np.random.default_rng(7)
    u = rng.random((2, 31))
    pool = orc.average_pool if mode == "avg" else orc.max_pool
    for kernel, extent in [(5, 20), (7, 31), (3, 1), (9, 0)]:
        out = pool(u, kernel, extent)
        np.testing.assert_array_equal(out[:, :extent], pool(u[:, :extent], kernel))
        assert (out[:, extent:] == 0).all()
    # library pin for the average on the slice
    ref = torch.nn.functional.avg_pool1d(torch.from_numpy(u[:, :20])[None], 5, stride=1, padding=2, count_include_pad=True)[0].numpy()
    np.testing.assert_allclose(orc.average_pool(u, 5, 20)[:, :20], ref, rtol=1e-14)


def test_score_variants_compose_and_default_is_unchanged():
    q, k, p = _rand_case(3)
    n, w = k.shape[1], q.shape[1]
    base = orc.score(q, k, p, pool_kernel=5, prior_weight=0.7)
    np.testing.assert_array_equal(base, orc.score(q, k, p, pool_kernel=5, prior_weight=0.7, group_reduce="mean",
                                                  pool_mode="avg", softmax_domain="all", pool_domain="row"))
    full = orc.score(q, k, p, pool_kernel=5, prior_weight=0.7, group_reduce="sum", pool_mode="max",
                     softmax_domain="prefix", pool_domain="prefix")
    by_hand = orc.max_pool(3 * orc.window_attention_mass(q, k[:, :n - w]), 5)
    np.testing.assert_allclose(full[:, :n - w], by_hand + 0.7 * p[None, :n - w], rtol=1e-13)
    np.testing.assert_allclose(full[:, n - w:], np.broadcast_to(0.7 * p[None, n - w:], (2, w)), rtol=1e-13)
    # selection at lambda = 0 does not care about mean vs sum (a positive factor)
    a = orc.select(orc.score(q, k, p, pool_kernel=3, prior_weight=0.0), w, 9)
    b_ = orc.select(orc.score(q, k, p, pool_kernel=3, prior_weight=0.0, group_reduce="sum"), w, 9)
    np.testing.assert_array_equal(a, b_)


# ------------------------------------------------------------------ fp8 (E4M3) key storage

def test_fp8_e4m3_decoder_matches_library_and_format_constants():
    codes = np.arange(256, dtype=np.uint8)
    ours = orc.fp8_e4m3_to_f64(codes)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(ours), np.isnan(ref)) and np.isnan(ours).sum() == 2      # 0x7f and 0xff only
    ok = ~np.isnan(ref)
    assert np.array_equal(ours[ok], ref[ok])
    # constants of the format: one, largest finite, smallest subnormal, smallest normal, signed zero
    assert ours[0x38] == 1.0 and ours[0x7E] == 448.0 and ours[0x01] == 2.0 ** -9 and ours[0x08] == 2.0 ** -6
    assert ours[0x00] == 0.0 and ours[0x80] == 0.0 and np.signbit(ours[0x80])
    assert ours[0x3C] == 1.5 and ours[0xC0] == -2.0
    # magnitudes grow with the code, and the sign bit only flips the sign
    assert (np.diff(ours[:0x7F]) > 0).all()
    assert np.array_equal(ours[0x80:0xFF], -ours[0x00:0x7F])


def test_fp8_keys_score_like_the_bf16_keys_holding_the_same_numbers():
    g = np.random.default_rng(11)
    l, hq, hkv, w, d = 2, 4, 2, 3, 8
    cu = np.array([0, 9, 20])
    codes = g.integers(0, 256, size=(l, hkv, 20, d)).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x38                       # no NaN codes
    codes &= 0xBF                                              # magnitudes below 2: tame logits
    # every E4M3 number is a bf16 number: the same values as bf16 patterns, built with the library cast
    as_bf16 = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    q = g.integers(0x3C00, 0x4000, size=(l, 2, hq, w, d)).astype(np.uint16)
    prior = g.random(20)
    a = orc.score_packed(q, codes, prior, cu, pool_kernel=3, prior_weight=0.5, k_format="fp8_e4m3")
    b = orc.score_packed(q, as_bf16, prior, cu, pool_kernel=3, prior_weight=0.5)
    np.testing.assert_array_equal(a, b)
    # and the whole path copies the codes themselves
    cb = np.array([0, 5, 12])
    sc, idx, ko, vo = orc.compress_packed(q, codes, codes[::-1].copy(), prior, cu, cb, window=w, pool_kernel=3,
                                          prior_weight=0.5, k_format="fp8_e4m3")
    assert ko.dtype == np.uint8 and np.array_equal(sc, a)
    assert np.array_equal(ko[1, 0, 5:], codes[1, 0, 9:][idx[1, 0, 5:]])
    assert np.array_equal(vo[0, 1, :5], codes[1, 1, :9][idx[0, 1, :5]])
