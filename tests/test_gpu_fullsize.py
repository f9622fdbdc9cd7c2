"""Full-size runs of the benchmark configurations through the fused entry point, in the launch
configuration bench.py times.  Everything that is integer or byte work is checked everywhere;
scores are compared with the fp64 oracle on sampled (layer, KV head, request) problems that it
finishes in seconds, and through size-independent properties on all of them."""
import numpy as np
import pytest

from oracle import codecomp_oracle as orc
from paper_2604_10235_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def run_full(w, samples, kv="bf16"):
    """samples: list of (layer, kv_head, request) whose scores are compared with the oracle."""
    import torch
    from paper_2604_10235_amd import binding as b
    q, k, v, prior = wl.make_all(w, threads=16)
    if kv == "fp8_e4m3":
        k, v = wl.bf16_bits_to_fp8_codes(k), wl.bf16_bits_to_fp8_codes(v)
    prob = b.DeviceProblem(w, q, k, v, prior)
    prob.compress(); torch.cuda.synchronize()
    sc = prob.scores.cpu().numpy()
    idx = prob.idx.cpu().numpy()
    cu, cb = w.cu_seqlens(), w.cu_budgets()
    G, W = w.group, w.window

    # byte work: gathered rows equal a host copy with the GPU's indices, everywhere
    assert np.array_equal(b.DeviceProblem.bits(prob.k_out), pu.host_gather(k, idx, cu, cb))
    assert np.array_equal(b.DeviceProblem.bits(prob.v_out), pu.host_gather(v, idx, cu, cb))
    # integer work: the selection rule applied by the oracle to the GPU's own fp32 scores, everywhere
    assert np.array_equal(idx.astype(np.int64), orc.select_packed(sc.astype(np.float64), cu, cb, W))
    # property at any size: the attention mass of a head sums to W; pooling loses only edge mass
    for r in range(w.n_seqs):
        a, e = cu[r], cu[r + 1]
        mass = (sc[:, :, a:e].astype(np.float64) - w.prior_weight * prior[a:e].astype(np.float64)).sum(axis=2)
        assert np.all(mass <= W * (1 + 1e-4)) and np.all(mass >= W * 0.98), (r, mass.min(), mass.max())
    assert np.isfinite(sc).all() and (sc >= 0).all()
    # sampled problems against the oracle
    worst = 0.0
    for (l, h, r) in samples:
        a, e = int(cu[r]), int(cu[r + 1])
        ref = orc.score(orc.bf16_bits_to_f64(q[l, r, h * G:(h + 1) * G]), orc.keys_to_f64(k[l, h:h + 1, a:e], kv),
                        prior[a:e], pool_kernel=w.pool_kernel, prior_weight=w.prior_weight)
        worst = max(worst, pu.assert_scores_close(sc[l, h, a:e], ref[0], what=f"scores[{l},{h},{r}]"))
        idx_ref = orc.select(ref, W, w.budgets[r])[0]
        pu.assert_index_sets_match(idx[l, h, cb[r]:cb[r + 1]], idx_ref, ref[0], W, what=f"idx[{l},{h},{r}]")
    return worst


def test_qwen7b_32k_all_layers():
    w = wl.qwen7b_32k()
    samples = [(0, 0, 0), (0, 3, 0), (13, 1, 0), (27, 2, 0), (27, 3, 0)]
    run_full(w, samples)


def test_ragged_agentic_full():
    w = wl.ragged_agentic()
    shortest = int(np.argmin(w.seqlens)); longest = int(np.argmax(w.seqlens))
    run_full(w, [(0, 0, shortest), (0, 2, longest), (0, 3, 5)])


def test_paper_chunks_full():
    # the paper's own setting: 64 chunks of 142 .. 2313 tokens, window 128 (896 rows in two row splits), pooling 5,
    # half of every chunk kept; the oracle scores the shortest, the longest and a middle chunk
    w = wl.paper_chunks()
    order = np.argsort(w.seqlens)
    run_full(w, [(0, 0, int(order[0])), (13, 2, int(order[-1])), (27, 3, int(order[len(order) // 2])), (5, 1, 7)])


@pytest.mark.timeout(600)
def test_llama8b_64k_all_layers():
    # all 32 layers; the oracle scores sampled heads of the first, a middle and the last layer
    run_full(wl.llama8b_64k(), [(0, 0, 0), (15, 4, 0), (31, 7, 0)])


@pytest.mark.timeout(600)
def test_long_128k_all_layers():
    # all 28 layers; W = 128, G = 7: 896 rows in two row splits, budget partly forced by the prior, selection
    # by parts (16 parts per problem); the oracle scores one head of the first, a middle and the last layer
    run_full(wl.long_128k(), [(0, 1, 0), (14, 3, 0), (27, 0, 0)])


def test_qwen7b_32k_all_layers_fp8_cache():
    run_full(wl.qwen7b_32k(), [(0, 1, 0), (14, 0, 0), (27, 3, 0)], kv="fp8_e4m3")


def test_one_million_tokens_in_one_request():
    # far beyond the configurations: 2**20 keys under one head (16384 tiles of one problem spread over the whole
    # chip, selection by 128 parts, 50000 kept rows)
    w = wl.scaled(wl.qwen7b_32k(), n_layers=1, n_q_heads=2, n_kv_heads=1, window=32, seqlens=[1 << 20], budgets=[50000])
    run_full(w, [(0, 0, 0)])
