"""Selection at the sizes and in the modes the benchmark configurations use.

* codecomp_select on crafted fp32 score rows uploaded straight into `scores` (no score step): equal rows, two
  values with thousands of ties at the cut, negatives, +-0, infinities, at candidate counts that reach every
  register variant of the one-workgroup kernel and the selection by parts - indices bit-equal to the oracle's rule.
* The two-stage rule at full request length for every variant: the 32K, ragged, 64K and 128K workloads.
* Structure-aware budgets -> cu_budgets -> ragged compress -> oracle, end to end.
"""
import numpy as np
import pytest

from oracle import codecomp_oracle as orc
from paper_2604_10235_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

W = 64


def crafted_rows(npre: int, need: int, seed: int) -> np.ndarray:
    """fp32 [rows][npre + W]: one crafted pattern per row (the window's own scores are junk that select ignores)."""
    g = np.random.default_rng(seed)
    n = npre + W
    rows = []
    rows.append(np.full(n, 0.5, np.float32))                                   # all equal: the first `need` win
    rows.append(np.zeros(n, np.float32))                                       # all zero
    r = np.zeros(n, np.float32); r[g.random(n) < 0.5] = -0.0                    # -0 and +0 are one value
    rows.append(r)
    r = np.full(n, 0.25, np.float32)                                           # two values, fewer high ones than slots:
    r[g.choice(npre, size=min(npre, max(1, need - need // 3)), replace=False)] = 0.75     # the cut falls among thousands of low ties
    rows.append(r)
    r = np.full(n, 0.25, np.float32)                                           # two values, more high ones than slots:
    r[g.choice(npre, size=min(npre, need + need // 2 + 1), replace=False)] = 0.75   # the cut falls among the high ties
    rows.append(r)
    rows.append(g.standard_normal(n).astype(np.float32))                       # both signs, (almost) no ties
    rows.append(np.round(g.standard_normal(n), 1).astype(np.float32))           # both signs, ~60 distinct values
    rows.append(-np.abs(g.standard_normal(n)).astype(np.float32))               # all negative
    r = np.where(g.random(n) < 0.5, -0.0, 0.0).astype(np.float32)               # a few positives and negatives around
    hot = g.choice(npre, size=min(npre, max(1, need // 4)), replace=False); r[hot] = g.random(len(hot)).astype(np.float32) + 0.1
    cold = g.choice(npre, size=npre // 5, replace=False); r[cold] = -1.0 - g.random(len(cold)).astype(np.float32)
    rows.append(r)                                                              # ... a sea of signed zeros: the cut is in it
    r = g.standard_normal(n).astype(np.float32)
    r[g.choice(npre, size=min(7, npre), replace=False)] = np.inf; r[g.choice(npre, size=min(7, npre), replace=False)] = -np.inf
    rows.append(r)
    r = (g.integers(0, 4, size=n) * np.float32(1e-42)).astype(np.float32)       # subnormals with ties
    rows.append(r)
    r = np.arange(n, dtype=np.float32)                                          # ascending: the last candidates win
    rows.append(r)
    rows.append(r[::-1].copy())                                                 # descending: the first win
    return np.stack(rows)


def select_on_device(rows, seqlens, budgets, layers=1):
    """rows [H][T] fp32 -> idx [L][H][TB] through codecomp_select (scores uploaded as they are)."""
    import torch
    from paper_2604_10235_amd import binding as b
    h, total = rows.shape
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    cb = np.concatenate([[0], np.cumsum(budgets)]).astype(np.int32)
    assert cu[-1] == total
    dev = torch.device("cuda:0")
    cu_d, cb_d = torch.from_numpy(cu).to(dev), torch.from_numpy(cb).to(dev)
    p = b.make_params(n_layers=layers, n_q_heads=h, n_kv_heads=h, head_dim=128, window=W, pool_kernel=1, prior_weight=0.0,
                      cu_seqlens_host=cu, cu_budgets_host=cb, cu_seqlens_dev=cu_d.data_ptr(), cu_budgets_dev=cb_d.data_ptr())
    sc = torch.from_numpy(np.broadcast_to(rows, (layers, h, total)).copy()).to(dev)
    idx = torch.full((layers, h, int(cb[-1])), -7, dtype=torch.int32, device=dev)
    ws = torch.empty(max(256, b.codecomp_workspace_bytes(p)), dtype=torch.uint8, device=dev)
    ws.fill_(0xFF)
    b.codecomp_select(sc, p, idx, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), cu, cb


# Which kernels run depends on the longest request and on the number of (layer, head, request) problems: with 26
# problems (2 layers x 13 rows) requests of 16384 candidates or more are cut into parts of 8192 (2, 3, 4, 5, 8, 9, 18
# parts here, including the budgets that keep nothing or everything); with 104 problems (8 layers) one workgroup per
# problem keeps 8 / 16 / 32 / 48 / 64 candidates per thread in registers up to 65536 candidates, parts beyond.
@pytest.mark.parametrize("npre,need,layers", [
    (3000, 200, 2), (9000, 1000, 2), (16383, 5000, 2), (16384, 5000, 2), (30000, 2000, 2), (40000, 3100, 2),
    (60000, 4096, 2), (70000, 5000, 2), (140000, 13043, 2), (9000, 8999, 2), (9000, 1, 2), (20000, 20000, 2),
    (20000, 0, 2), (20000, 19999, 2), (20000, 1, 2), (65536, 8192, 2),
    (9000, 1000, 8), (30000, 2000, 8), (40000, 3100, 8), (60000, 4096, 8), (65536, 8192, 8), (65537, 8192, 8)])
def test_select_on_crafted_scores(npre, need, layers):
    rows = crafted_rows(npre, need, seed=npre + need)
    idx, cu, cb = select_on_device(rows, [npre + W], [need + W], layers=layers)
    want = orc.select(rows.astype(np.float64), W, need + W)
    for l in range(layers):
        assert np.array_equal(idx[l].astype(np.int64), want), (npre, need, l)


def test_select_beyond_the_table_of_the_resolve_kernel():
    """More parts than the resolve kernel can keep running totals for (3 * parts > its 8200 words: 2734 parts of 8192
    candidates): the emitting parts then count the earlier parts' entries themselves."""
    npre, need = 2734 * 8192 + 5, 1_000_003
    g = np.random.default_rng(99)
    n = npre + W
    two = np.full(n, 0.25, np.float32)
    two[g.choice(npre, size=need - need // 3, replace=False)] = 0.75           # the cut falls among millions of low ties
    coarse = np.round(g.standard_normal(n), 1).astype(np.float32)               # ~60 distinct values
    rows = np.stack([two, coarse, np.full(n, 0.5, np.float32)])
    idx, cu, cb = select_on_device(rows, [n], [need + W])
    for r in range(rows.shape[0]):
        want = orc.select(rows[r:r + 1].astype(np.float64), W, need + W)[0]
        assert np.array_equal(idx[0, r].astype(np.int64), want), r


def test_select_on_crafted_scores_ragged():
    """Requests of very different lengths in one call (the longest one decides the kernel variant), budgets from the
    window alone to everything."""
    lens = [70000 + W, 300 + W, W, 9000 + W, 1 + W, 33000 + W]
    needs = [5000, 300, 0, 0, 1, 2000]
    parts = [crafted_rows(n - W, max(1, b), seed=17 + i) if n > W else np.zeros((13, W), np.float32)
             for i, (n, b) in enumerate(zip(lens, needs))]
    rows = np.concatenate(parts, axis=1)
    idx, cu, cb = select_on_device(rows, lens, [b + W for b in needs])
    want = orc.select_packed(rows.astype(np.float64)[None], cu, cb, W)
    assert np.array_equal(idx.astype(np.int64), want)


def test_select_by_parts_in_a_batch_of_many_requests():
    """One long request among 600 short ones: the whole batch is selected by parts (most requests are a single part,
    some have no candidate at all), and a workgroup finds its request among many."""
    g = np.random.default_rng(99)
    lens = [int(x) + W for x in g.integers(0, 700, size=600)]
    lens[0] = W; lens[599] = W + 1; lens[311] = 40000 + W; lens[312] = 17000 + W
    needs = [int(g.integers(0, n - W + 1)) for n in lens]
    rows = np.concatenate([crafted_rows(n - W, max(1, b), seed=1000 + i)[[(i + k_) % 13 for k_ in range(3)]] if n > W
                           else np.zeros((3, W), np.float32) for i, (n, b) in enumerate(zip(lens, needs))], axis=1)
    idx, cu, cb = select_on_device(rows, lens, [b + W for b in needs])
    want = orc.select_packed(rows.astype(np.float64)[None], cu, cb, W)
    assert np.array_equal(idx.astype(np.int64), want)


@pytest.mark.parametrize("longest", [1500, 2048, 3000, 4096, 4097])
def test_select_with_small_workgroups(longest):
    """Batches of requests of at most 4096 candidates with a thousand problems or more run 256-thread workgroups
    holding 8 or 16 candidates per thread (the longest request decides; one candidate more and the 1024-thread
    kernel runs): 120 requests x 3 rows x 3 layers, crafted rows."""
    g = np.random.default_rng(longest)
    lens = [int(x) + W for x in g.integers(0, min(longest, 2000), size=120)]
    lens[0] = W; lens[7] = W + 1; lens[60] = longest + W
    needs = [int(g.integers(0, n - W + 1)) for n in lens]
    needs[60] = longest // 3
    rows = np.concatenate([crafted_rows(n - W, max(1, b), seed=2000 + i)[[(i + k_) % 13 for k_ in range(3)]] if n > W
                           else np.zeros((3, W), np.float32) for i, (n, b) in enumerate(zip(lens, needs))], axis=1)
    idx, cu, cb = select_on_device(rows, lens, [b + W for b in needs], layers=3)
    want = orc.select_packed(rows.astype(np.float64)[None], cu, cb, W)[0]
    for l in range(3):
        assert np.array_equal(idx[l].astype(np.int64), want), l


def two_stage_on_device(rows, prior, seqlens, budgets, ratio, bmin, layers=1):
    """rows [H][T] fp32 (pooled attention), prior [T] -> idx [L][H][TB] through codecomp_select_two_stage."""
    import torch
    from paper_2604_10235_amd import binding as b
    h, total = rows.shape
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    cb = np.concatenate([[0], np.cumsum(budgets)]).astype(np.int32)
    dev = torch.device("cuda:0")
    cu_d, cb_d = torch.from_numpy(cu).to(dev), torch.from_numpy(cb).to(dev)
    p = b.make_params(n_layers=layers, n_q_heads=h, n_kv_heads=h, head_dim=128, window=W, pool_kernel=1, prior_weight=0.0,
                      cu_seqlens_host=cu, cu_budgets_host=cb, cu_seqlens_dev=cu_d.data_ptr(), cu_budgets_dev=cb_d.data_ptr(),
                      select_mode=1, span_budget_ratio=ratio, span_budget_min=bmin)
    sc = torch.from_numpy(np.broadcast_to(rows, (layers, h, total)).copy()).to(dev)
    pr = torch.from_numpy(prior.astype(np.float32)).to(dev)
    idx = torch.full((layers, h, int(cb[-1])), -7, dtype=torch.int32, device=dev)
    ws = torch.empty(max(256, b.codecomp_workspace_bytes(p)), dtype=torch.uint8, device=dev)
    ws.fill_(0xFF)
    b.codecomp_select_two_stage(sc, pr, p, idx, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), cu, cb


@pytest.mark.parametrize("seed", range(10))
def test_random_batches_with_long_requests(seed):
    """Seeded random batches that hold at least one long request (so that the selection runs by parts), budgets from
    the window alone to everything, scores with many ties; the additive rule and the two-stage rule (graded or binary
    prior, any span budget) against the oracle's rules on the same fp32 values."""
    g = np.random.default_rng(31000 + seed)
    n_seqs = int(g.integers(1, 7))
    lens = [W + int(g.integers(0, 3000)) for _ in range(n_seqs)]
    lens[int(g.integers(0, n_seqs))] = W + int(g.choice([16384, 20000, 33333, 65536, 65537, 90000]))
    if g.random() < 0.5:
        lens.append(W + int(g.integers(16384, 40000)))
    needs = [int(g.choice([0, 1, (n - W) // 10, (n - W) // 2, max(0, n - W - 1), n - W])) for n in lens]
    total = sum(lens)
    kind = int(g.integers(0, 3))
    if kind == 0:
        rows = g.random((3, total)).astype(np.float32)                                   # (almost) no ties
    elif kind == 1:
        rows = np.round(g.standard_normal((3, total)), 1).astype(np.float32)              # ~60 values, both signs
    else:
        rows = (g.integers(0, 3, size=(3, total)) * np.float32(0.25)).astype(np.float32)  # three values
    budgets = [b + W for b in needs]
    idx, cu, cb = select_on_device(rows, lens, budgets)
    assert np.array_equal(idx.astype(np.int64), orc.select_packed(rows.astype(np.float64)[None], cu, cb, W))
    # the two-stage rule on the same scores
    prior = np.where(g.random(total) < g.choice([0.05, 0.3, 0.9]), g.random(total) if g.random() < 0.5 else 1.0, 0.0).astype(np.float32)
    ratio, bmin = float(g.choice([0.0, 0.25, 0.5, 1.0])), int(g.choice([0, 7, 5000]))
    idx2, _, _ = two_stage_on_device(rows, prior, lens, budgets, ratio, bmin)
    for r in range(len(lens)):
        a, e = cu[r], cu[r + 1]
        want = orc.select_two_stage(rows[:, a:e].astype(np.float64), prior[a:e], W, budgets[r],
                                    span_ratio=float(np.float32(ratio)), span_min=bmin)
        assert np.array_equal(idx2[0, :, cb[r]:cb[r + 1]].astype(np.int64), want), (seed, r, lens[r], budgets[r], ratio, bmin)


def test_two_stage_with_small_workgroups_in_both_stages():
    """1100 requests of at most 3000 candidates: stage 1 (one problem per request) and stage 2 both run the 256-thread
    workgroups; priors with ties, span budgets that bind and that do not."""
    g = np.random.default_rng(31)
    lens = [int(x) + W for x in g.integers(0, 900, size=1100)]
    lens[5] = W; lens[500] = 3000 + W; lens[900] = 2049 + W
    needs = [int(g.integers(0, n - W + 1)) for n in lens]
    total = sum(lens)
    rows = np.round(g.standard_normal((2, total)), 1).astype(np.float32)
    prior = np.where(g.random(total) < 0.3, np.round(g.random(total), 1) + 0.1, 0.0).astype(np.float32)
    budgets = [b + W for b in needs]
    for ratio, bmin in ((0.5, 0), (0.2, 40)):
        idx, cu, cb = two_stage_on_device(rows, prior, lens, budgets, ratio, bmin)
        for r in range(len(lens)):
            a, e = cu[r], cu[r + 1]
            want = orc.select_two_stage(rows[:, a:e].astype(np.float64), prior[a:e], W, budgets[r],
                                        span_ratio=float(np.float32(ratio)), span_min=bmin)
            assert np.array_equal(idx[0, :, cb[r]:cb[r + 1]].astype(np.int64), want), (r, lens[r], budgets[r], ratio, bmin)


def two_stage_full(w, ratio=0.5, bmin=0, layers_checked=None):
    """Fused call in two-stage mode on a full-size workload; indices bit-equal to the oracle's two-stage rule on the
    GPU's own fp32 scores (every layer in `layers_checked`, every head, every request), gather bit-exact."""
    import torch
    from paper_2604_10235_amd import binding as b
    q, k, v, prior = wl.make_all(w, threads=16)
    prob = b.DeviceProblem(w, q, k, v, prior, select_mode=1, span_budget_ratio=ratio, span_budget_min=bmin)
    prob.compress(); torch.cuda.synchronize()
    sc = prob.scores.cpu().numpy(); idx = prob.idx.cpu().numpy()
    cu, cb = w.cu_seqlens(), w.cu_budgets()
    ratio32 = float(np.float32(ratio))
    protected_any = False
    for l in (range(w.n_layers) if layers_checked is None else layers_checked):
        for r in range(w.n_seqs):
            a, e = cu[r], cu[r + 1]
            want = orc.select_two_stage(sc[l, :, a:e].astype(np.float64), prior[a:e], w.window, w.budgets[r],
                                        span_ratio=ratio32, span_min=bmin)
            assert np.array_equal(idx[l, :, cb[r]:cb[r + 1]].astype(np.int64), want), (w.name, l, r)
            protected_any |= bool((prior[a:e][want[0]] > 0).any())
    assert protected_any
    assert np.array_equal(b.DeviceProblem.bits(prob.k_out), pu.host_gather(k, idx, cu, cb))
    assert np.array_equal(b.DeviceProblem.bits(prob.v_out), pu.host_gather(v, idx, cu, cb))
    # the scores of this mode carry no prior term: the mass of a head sums to W (pooling loses edge mass only)
    mass = sc.astype(np.float64).sum(axis=2) if w.n_seqs == 1 else None
    if mass is not None:
        assert np.all(mass <= w.window * (1 + 1e-4)) and np.all(mass >= w.window * 0.98)


def test_two_stage_qwen7b_32k_all_layers():           # 32 candidates per thread
    two_stage_full(wl.qwen7b_32k())


def test_two_stage_ragged_agentic():                  # 48 per thread (longest request 49088 tokens), 16 requests
    two_stage_full(wl.ragged_agentic())


def test_two_stage_llama8b_64k_two_layers():          # 64 per thread, binary prior: stage 1 is all ties
    two_stage_full(wl.scaled(wl.llama8b_64k(), n_layers=2))


def test_two_stage_paper_chunks():                    # 64 short chunks x 112 heads: 256-thread workgroups in stage 2
    two_stage_full(wl.paper_chunks(), layers_checked=[0, 13, 27])


def test_two_stage_long_128k_one_layer():             # selection by parts, binary prior, budget 13107
    two_stage_full(wl.scaled(wl.long_128k(), n_layers=1))


@pytest.mark.parametrize("ratio,bmin", [(1.0, 0), (0.1, 3000), (0.0, 0)])
def test_two_stage_span_budgets_at_32k(ratio, bmin):
    two_stage_full(wl.scaled(wl.qwen7b_32k(), n_layers=2), ratio=ratio, bmin=bmin)


def test_structure_aware_budgets_feed_the_ragged_call():
    """Sections "Structural Feature Extraction" / "Structure-Aware Budget Allocation" -> per-chunk budgets B_i ->
    cu_budgets of a ragged batch (one request per chunk) -> the whole path, against the oracle doing the same."""
    import torch
    from paper_2604_10235_amd import binding as b
    g = np.random.default_rng(4242)
    lens = [int(x) for x in g.integers(600, 4096, size=12)]                    # chunks of at most 4096 tokens
    feats = g.integers(0, 60, size=(len(lens), 6)).astype(np.float64)           # call / control / return / assign / cfg / pdg counts
    feats[3] = 0.0; feats[7] = 500.0                                            # one bare chunk, one saturated one
    tau = np.array([20., 15., 6., 30., 40., 40.]); wts = np.array([.25, .2, .15, .15, .15, .1])
    kw = dict(ratio=0.4, m_min=0.5, m_max=1.5, r_max=0.9, eps=1e-6)
    sigma = b.codecomp_chunk_structure_scores(feats, tau, wts)
    budgets = b.codecomp_chunk_budgets(sigma, np.array(lens), window=32, **kw)
    # the oracle's own arithmetic gives the same budgets (the library clamps into [W, |C_i|]; nothing is clamped here)
    want_b = orc.chunk_budgets(orc.chunk_structure_score(feats, tau, wts), lens, **kw)
    assert np.array_equal(budgets, want_b) and budgets.min() >= 32
    assert budgets[7] / lens[7] > 0.55 and budgets[3] / lens[3] < 0.25           # multipliers 1.5 and 0.5 of the ratio 0.4
    w = wl.scaled(wl.ragged_agentic(), n_layers=2, seqlens=lens, budgets=[int(x) for x in budgets], window=32)
    q, k, v, prior = wl.make_all(w)
    prob = b.DeviceProblem(w, q, k, v, prior)
    prob.compress(); torch.cuda.synchronize()
    cu, cb = w.cu_seqlens(), w.cu_budgets()
    assert np.array_equal(cb[1:] - cb[:-1], want_b)
    sc_ref, idx_ref, _, _ = orc.compress_packed(q, k, v, prior, cu, cb, window=w.window, pool_kernel=w.pool_kernel,
                                                prior_weight=w.prior_weight)
    sc = prob.scores.cpu().numpy(); idx = prob.idx.cpu().numpy()
    pu.assert_scores_close(sc, sc_ref)
    for l in range(w.n_layers):
        for h in range(w.n_kv_heads):
            for r in range(w.n_seqs):
                pu.assert_index_sets_match(idx[l, h, cb[r]:cb[r + 1]], idx_ref[l, h, cb[r]:cb[r + 1]],
                                           sc_ref[l, h, cu[r]:cu[r + 1]], w.window, what=f"idx[{l},{h},{r}]")
    assert np.array_equal(idx.astype(np.int64), orc.select_packed(sc.astype(np.float64), cu, cb, w.window))
    assert np.array_equal(b.DeviceProblem.bits(prob.k_out), pu.host_gather(k, idx, cu, cb))
    assert np.array_equal(b.DeviceProblem.bits(prob.v_out), pu.host_gather(v, idx, cu, cb))
    # the budgets took effect: the chunk with the richest structure keeps the largest share of its tokens
    kept = (cb[1:] - cb[:-1]) / np.array(lens)
    assert kept.argmax() == int(np.argmax(sigma)) and kept.argmin() == int(np.argmin(sigma))
