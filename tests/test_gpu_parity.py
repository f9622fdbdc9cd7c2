"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

from oracle import codecomp_oracle as orc
from paper_2604_10235_amd import workloads as wl
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _binding():
    from paper_2604_10235_amd import binding
    return binding


def oracle_variant(flags: int) -> dict:
    """Oracle keyword arguments for a set of CODECOMP_VARIANT_* flags."""
    return dict(group_reduce="sum" if flags & 1 else "max" if flags & 2 else "mean",
                pool_mode="max" if flags & 4 else "avg",
                softmax_domain="prefix" if flags & 8 else "all",
                pool_domain="prefix" if flags & 16 else "row")


def run_case(w, *, fused=True, check_oracle=True, variant=0, kv="bf16", score_workgroups=0):
    """Runs the three steps (or the fused call) and compares every stage with the oracle.  kv = "fp8_e4m3":
    the cache (k and v) is the FP8 copy of the workload's bf16 cache."""
    import torch
    b = _binding()
    q, k, v, prior = wl.make_all(w)
    if kv == "fp8_e4m3":
        k, v = wl.bf16_bits_to_fp8_codes(k), wl.bf16_bits_to_fp8_codes(v)
    prob = b.DeviceProblem(w, q, k, v, prior, score_variant=variant, score_workgroups=score_workgroups)
    if fused:
        prob.compress()
    else:
        prob.score(); prob.select(); prob.gather()
    torch.cuda.synchronize()
    sc_gpu = prob.scores.cpu().numpy()
    idx_gpu = prob.idx.cpu().numpy()
    ko, vo = b.DeviceProblem.bits(prob.k_out), b.DeviceProblem.bits(prob.v_out)
    cu, cb = w.cu_seqlens(), w.cu_budgets()

    # gather: bit-exact against a host row copy with the GPU's own indices
    assert np.array_equal(ko, pu.host_gather(k, idx_gpu, cu, cb))
    assert np.array_equal(vo, pu.host_gather(v, idx_gpu, cu, cb))
    # select: integer work, must equal the oracle's rule applied to the very same fp32 scores
    idx_same = orc.select_packed(sc_gpu.astype(np.float64), cu, cb, w.window)
    assert np.array_equal(idx_gpu.astype(np.int64), idx_same)
    if not check_oracle:
        return prob, sc_gpu, idx_gpu
    # scores and index sets against the fp64 oracle
    sc_ref = orc.score_packed(q, k, prior, cu, pool_kernel=w.pool_kernel, prior_weight=w.prior_weight,
                              k_format=kv, **oracle_variant(variant))
    pu.assert_scores_close(sc_gpu, sc_ref)
    idx_ref = orc.select_packed(sc_ref, cu, cb, w.window)
    for l in range(w.n_layers):
        for h in range(w.n_kv_heads):
            for r in range(w.n_seqs):
                pu.assert_index_sets_match(idx_gpu[l, h, cb[r]:cb[r + 1]], idx_ref[l, h, cb[r]:cb[r + 1]],
                                           sc_ref[l, h, cu[r]:cu[r + 1]], w.window, what=f"idx[{l},{h},{r}]")
    return prob, sc_gpu, idx_gpu


def test_tiny_config_full():
    run_case(wl.tiny(), fused=False)
    run_case(wl.tiny(), fused=True)


def test_qwen_shape_ragged_tail():
    # 5000 keys = 4 chunks of 1024 + 904 = 14 tiles of 64 + 8: several chunks, several tiles, ragged tail
    run_case(wl.scaled(wl.qwen7b_32k(), n_layers=2, seqlens=[5000]))


def test_llama_shape_with_drift():
    w = wl.scaled(wl.llama8b_64k(), n_layers=2, seqlens=[3001], n_q_heads=8, n_kv_heads=2)
    run_case(w)


def test_long_shape_two_row_splits():
    # W = 128, G = 7: 896 softmax rows -> two workgroups along the row axis
    run_case(wl.scaled(wl.long_128k(), n_layers=1, seqlens=[4100], n_kv_heads=2, n_q_heads=14))


def test_ragged_batch():
    w = wl.scaled(wl.ragged_agentic(), seqlens=[700, 1300, 64, 2049, 1024, 65], budgets=[70, 130, 64, 204, 1024, 65])
    run_case(w, fused=True)
    run_case(w, fused=False)


@pytest.mark.parametrize("wgs,lead", [(1, 4), (3, -1), (7, 4), (13, 9), (64, 1), (2048, 4), (2048, 40)])
def test_any_split_of_the_tile_sequence_gives_the_same_scores(wgs, lead):
    """The score passes cut the tile sequence of all (layer, head, request) problems into one range per
    workgroup; a range may cover several problems, start inside one, or hold no tile at all.  Forced grid
    sizes and segment-start weights: the result must not depend on them (fp32 sums regroup: 1e-5)."""
    import torch
    b = _binding()
    w = wl.scaled(wl.ragged_agentic(), n_layers=2, seqlens=[700, 1300, 64, 2049, 130], budgets=[70, 130, 64, 204, 70])
    q, k, v, prior = wl.make_all(w)
    ref = b.DeviceProblem(w, q, k, v, prior)
    ref.score()
    torch.cuda.synchronize()
    sc_ref = ref.scores.cpu().numpy()
    cu = w.cu_seqlens()
    pu.assert_scores_close(sc_ref, orc.score_packed(q, k, prior, cu, pool_kernel=w.pool_kernel, prior_weight=w.prior_weight))
    prob = b.DeviceProblem(w, q, k, v, prior, score_workgroups=wgs, score_lead_tiles=lead)    # lead < 0: none
    prob.score()
    torch.cuda.synchronize()
    np.testing.assert_allclose(prob.scores.cpu().numpy(), sc_ref, rtol=1e-5, atol=1e-30)


@pytest.mark.parametrize("group,window", [(5, 64), (6, 64), (7, 64), (3, 100), (9, 32), (13, 40), (15, 32), (16, 32)])
def test_row_blocks_shared_between_waves(group, window):
    """More than 8 blocks of 32 softmax rows: eight waves, some blocks owned by two waves (one per half of
    every tile); their statistics are merged per row."""
    run_case(wl.scaled(wl.qwen7b_32k(), n_layers=1, seqlens=[1500, 230], budgets=[window + 50, window + 3], window=window,
                       n_q_heads=2 * group, n_kv_heads=2))


@pytest.mark.parametrize("variant", [1, 4, 8, 16, 1 | 4, 8 | 16, 1 | 4 | 8 | 16, 2, 2 | 4 | 8 | 16])
def test_score_tail_variants(variant):
    """Group sum / max, max pooling, prefix-only softmax and pooling, alone and combined: 448 rows (shared row
    blocks, 14 blocks = 7 heads of 2), several requests, one of them nothing but its window."""
    w = wl.scaled(wl.qwen7b_32k(), n_layers=2, seqlens=[1500, 64, 700, 65], budgets=[150, 64, 90, 64], n_kv_heads=2,
                  n_q_heads=14)
    run_case(w, variant=variant)
    run_case(wl.scaled(wl.tiny(), seqlens=[1000], budgets=[100], prior_weight=0.0), variant=variant, fused=False)


def test_prefix_softmax_without_any_prefix():
    """Every request is only its window: no key to attend to, all masses zero, scores = lambda * prior."""
    import torch
    b = _binding()
    w = wl.scaled(wl.tiny(), seqlens=[32, 32], budgets=[32, 32])
    q, k, v, prior = wl.make_all(w)
    prob = b.DeviceProblem(w, q, k, v, prior, score_variant=b.VARIANT_SOFTMAX_PREFIX)
    prob.workspace.fill_(0xFF)
    prob.compress()
    torch.cuda.synchronize()
    sc = prob.scores.cpu().numpy()
    np.testing.assert_array_equal(sc, np.broadcast_to((np.float32(w.prior_weight) * prior)[None, None, :], sc.shape))
    assert np.array_equal(prob.idx.cpu().numpy()[0, 0], np.concatenate([np.arange(32), np.arange(32)]))


@pytest.mark.parametrize("kw", [
    dict(seqlens=[32], budgets=[32], window=32),                       # N == W == B: window only, no prefix
    dict(seqlens=[1], budgets=[1], window=1),                          # a single token
    dict(seqlens=[300], budgets=[300], window=16),                     # B == N: identity
    dict(seqlens=[300], budgets=[16], window=16),                      # B == W: window only
    dict(seqlens=[37], budgets=[20], window=5),                        # shorter than one tile, odd window
    dict(seqlens=[1000], budgets=[100], window=40, n_q_heads=12),      # R = 3 * 40 = 120 rows, not a multiple of 32
    dict(seqlens=[777], budgets=[99], window=32, pool_kernel=1),       # no pooling
    dict(seqlens=[777], budgets=[99], window=32, prior_weight=0.0),    # attention only
    dict(seqlens=[777], budgets=[99], window=32, pool_kernel=31),      # wide pooling
    dict(seqlens=[1500], budgets=[200], window=32, head_dim=64, n_q_heads=8),   # d = 64 with a group of 2
    dict(seqlens=[3000], budgets=[400], window=32, pool_kernel=1025),  # the widest pooling the path takes
    dict(seqlens=[12000], budgets=[900], window=32),                   # selection with 16 candidates per thread in registers
    dict(seqlens=[40000, 9000], budgets=[3000, 700], window=32),       # ... and with 48 (chosen from the longest request)
    dict(seqlens=[1500], budgets=[200], window=64, head_dim=64, n_q_heads=28),  # d = 64 with eight waves (448 rows)
    dict(seqlens=[2000, 600], budgets=[700, 512], window=512, n_q_heads=8, n_kv_heads=2),   # 2048 rows: four row splits
    dict(seqlens=[1100], budgets=[1050], window=1024, n_q_heads=64, n_kv_heads=1),  # 65536 rows: the most the path takes
])
def test_edge_cases(kw):
    base = dict(n_layers=1, n_q_heads=4, n_kv_heads=4, head_dim=128)
    base.update(kw)
    run_case(wl.scaled(wl.qwen7b_32k(), **base))


def test_zero_keys_closed_form():
    # all keys equal (zero): every token gets mass W/N, pooled with zero padding (closed form, no oracle)
    import torch
    b = _binding()
    w = wl.scaled(wl.qwen7b_32k(), n_layers=1, seqlens=[20000], prior_weight=0.0)
    q, k, v, prior = wl.make_all(w)
    k[:] = 0
    prob = b.DeviceProblem(w, q, k, v, prior)
    prob.score(); torch.cuda.synchronize()
    sc = prob.scores.cpu().numpy().astype(np.float64)
    n, W, kk = 20000, w.window, w.pool_kernel
    expect = np.full(n, W / n)
    for e in range(3):
        expect[e] = expect[n - 1 - e] = (W / n) * (kk - 3 + e) / kk
    np.testing.assert_allclose(sc, np.tile(expect, (1, w.n_kv_heads, 1)), rtol=1e-5)


def test_deterministic_and_workspace_poison():
    import torch
    w = wl.scaled(wl.qwen7b_32k(), n_layers=2, seqlens=[3000, 1111], budgets=[300, 111])
    prob, sc1, idx1 = run_case(w, check_oracle=False)
    k1, v1 = prob.k_out.clone(), prob.v_out.clone()
    prob.workspace.fill_(0xFF)            # NaN patterns: nothing may be read before it is written
    prob.scores.fill_(float("nan")); prob.idx.fill_(-1); prob.k_out.fill_(0); prob.v_out.fill_(0)
    prob.compress(); torch.cuda.synchronize()
    assert np.array_equal(prob.scores.cpu().numpy(), sc1)
    assert np.array_equal(prob.idx.cpu().numpy(), idx1)
    assert torch.equal(prob.k_out, k1) and torch.equal(prob.v_out, v1)


def test_strided_kv_and_output():
    # K/V stored token-major ([T][H_kv][d], as a paged cache would) through the stride arguments
    import torch
    b = _binding()
    w = wl.scaled(wl.qwen7b_32k(), n_layers=2, seqlens=[2100])
    q, k, v, prior = wl.make_all(w)
    ref = b.DeviceProblem(w, q, k, v, prior)
    ref.compress(); torch.cuda.synchronize()
    prob = b.DeviceProblem(w, q, k, v, prior)
    L, H, T, d = k.shape
    prob.k = ref.k.permute(0, 2, 1, 3).contiguous()      # [L][T][H][d]
    prob.v = ref.v.permute(0, 2, 1, 3).contiguous()
    prob.params.kv_stride_layer, prob.params.kv_stride_head, prob.params.kv_stride_tok = T * H * d, d, H * d
    TB = w.total_budget
    prob.k_out = torch.zeros((L, TB, H, d), dtype=torch.bfloat16, device="cuda:0")
    prob.v_out = torch.zeros_like(prob.k_out)
    prob.params.out_stride_layer, prob.params.out_stride_head, prob.params.out_stride_tok = TB * H * d, d, H * d
    prob.compress(); torch.cuda.synchronize()
    assert torch.equal(prob.scores, ref.scores) and torch.equal(prob.idx, ref.idx)
    assert torch.equal(prob.k_out.permute(0, 2, 1, 3), ref.k_out)
    assert torch.equal(prob.v_out.permute(0, 2, 1, 3), ref.v_out)


# ------------------------------------------------------------------ two-stage selection, structure score

def run_two_stage(w, ratio, bmin, fused=True):
    import torch
    b = _binding()
    q, k, v, prior = wl.make_all(w)
    prob = b.DeviceProblem(w, q, k, v, prior, select_mode=1, span_budget_ratio=ratio, span_budget_min=bmin)
    if fused:
        prob.compress()
    else:
        prob.score(); prob.select(); prob.gather()
    torch.cuda.synchronize()
    sc = prob.scores.cpu().numpy(); idx = prob.idx.cpu().numpy()
    cu, cb = w.cu_seqlens(), w.cu_budgets()
    ratio32 = float(np.float32(ratio))
    # scores are the pooled attention alone (no prior term) ...
    ref = orc.score_packed(q, k, prior, cu, pool_kernel=w.pool_kernel, prior_weight=0.0)
    pu.assert_scores_close(sc, ref)
    # ... the selection is integer work: the oracle's rule on the GPU's own fp32 scores, bit for bit
    for l in range(w.n_layers):
        for r in range(w.n_seqs):
            a, e = cu[r], cu[r + 1]
            want = orc.select_two_stage(sc[l, :, a:e].astype(np.float64), prior[a:e], w.window, w.budgets[r],
                                        span_ratio=ratio32, span_min=bmin)
            assert np.array_equal(idx[l, :, cb[r]:cb[r + 1]].astype(np.int64), want), (l, r)
    assert np.array_equal(b.DeviceProblem.bits(prob.k_out), pu.host_gather(k, idx, cu, cb))
    assert np.array_equal(b.DeviceProblem.bits(prob.v_out), pu.host_gather(v, idx, cu, cb))
    return prob, idx, prior


@pytest.mark.parametrize("ratio,bmin", [(0.5, 0), (1.0, 0), (0.0, 0), (0.25, 40), (0.5, 100000)])
def test_two_stage_selection(ratio, bmin):
    run_two_stage(wl.scaled(wl.qwen7b_32k(), n_layers=2, seqlens=[5000]), ratio, bmin)                 # graded prior
    run_two_stage(wl.scaled(wl.long_128k(), n_layers=1, seqlens=[4100], n_kv_heads=2, n_q_heads=14), ratio, bmin,
                  fused=False)                                                                          # binary prior, many ties
    run_two_stage(wl.scaled(wl.ragged_agentic(), seqlens=[700, 1300, 64, 2049, 65], budgets=[70, 130, 64, 204, 65]),
                  ratio, bmin)


def test_two_stage_keeps_more_structure_than_attention_alone():
    import torch
    b = _binding()
    w = wl.scaled(wl.qwen7b_32k(), n_layers=2, seqlens=[6000, 3000], budgets=[480, 240])
    prob, idx, prior = run_two_stage(w, 0.5, 0)
    out = torch.empty((w.n_layers, w.n_kv_heads, w.n_seqs), dtype=torch.float32, device="cuda:0")
    b.codecomp_structure_score(prob.idx, prob.prior, prob.params, out); torch.cuda.synchronize()
    got = out.cpu().numpy()
    cu, cb = w.cu_seqlens(), w.cu_budgets()
    for l in range(w.n_layers):
        for r in range(w.n_seqs):
            ref = orc.structure_score(idx[l, :, cb[r]:cb[r + 1]], prior[cu[r]:cu[r + 1]], w.seqlens[r])
            np.testing.assert_allclose(got[l, :, r], ref, rtol=1e-6)
    # attention-only selection on the same inputs retains fewer marked tokens
    w0 = wl.scaled(w, prior_weight=0.0)
    prob0, _, _ = run_case(w0, check_oracle=False)
    out0 = torch.empty_like(out)
    b.codecomp_structure_score(prob0.idx, prob0.prior, prob0.params, out0); torch.cuda.synchronize()
    assert (out0.cpu().numpy() < got).all()


def test_structure_score_without_marked_tokens_is_nan():
    import torch
    b = _binding()
    w = wl.scaled(wl.tiny(), flag_rate=0.0)
    prob, _, _ = run_case(w, check_oracle=False)
    out = torch.zeros((1, 4, 1), dtype=torch.float32, device="cuda:0")
    b.codecomp_structure_score(prob.idx, prob.prior, prob.params, out); torch.cuda.synchronize()
    assert torch.isnan(out).all()


def test_large_logits_stay_finite_and_accurate():
    # keys scaled by 16 (exact in bf16): logits of several hundred, one key dominates most rows
    import torch
    b = _binding()
    w = wl.scaled(wl.qwen7b_32k(), n_layers=1, seqlens=[3000], n_q_heads=8, n_kv_heads=2)
    q, k, v, prior = wl.make_all(w)
    kf = orc.bf16_bits_to_f64(k) * 16.0
    k16 = wl.f32_to_bf16_bits(kf.astype(np.float32))
    assert np.array_equal(orc.bf16_bits_to_f64(k16), kf)
    prob = b.DeviceProblem(w, q, k16, v, prior)
    prob.score(); torch.cuda.synchronize()
    sc = prob.scores.cpu().numpy()
    assert np.isfinite(sc).all()
    ref = orc.score_packed(q, k16, prior, w.cu_seqlens(), pool_kernel=w.pool_kernel, prior_weight=w.prior_weight)
    # masses below 1e-30 are below fp32 resolution of the sums they come from; compare the rest relatively
    big = ref > 1e-30
    assert (np.abs(sc[big] - ref[big]) / ref[big]).max() < 1e-3


def test_logits_that_outrun_the_first_tile_reference():
    # the first keys of every chunk are ordinary, later keys are 64 times larger (exact in bf16): their logits
    # exceed anything seen in the first tile by hundreds of nats, which the row statistics must survive
    import torch
    b = _binding()
    w = wl.scaled(wl.qwen7b_32k(), n_layers=1, seqlens=[4500], n_q_heads=8, n_kv_heads=2)
    q, k, v, prior = wl.make_all(w)
    kf = orc.bf16_bits_to_f64(k)
    kf[:, :, 700:] *= 64.0
    kbig = wl.f32_to_bf16_bits(kf.astype(np.float32))
    assert np.array_equal(orc.bf16_bits_to_f64(kbig), kf)
    prob = b.DeviceProblem(w, q, kbig, v, prior)
    prob.score(); torch.cuda.synchronize()
    sc = prob.scores.cpu().numpy()
    assert np.isfinite(sc).all()
    ref = orc.score_packed(q, kbig, prior, w.cu_seqlens(), pool_kernel=w.pool_kernel, prior_weight=w.prior_weight)
    big = ref > 1e-30
    assert (np.abs(sc[big] - ref[big]) / ref[big]).max() < 1e-3
    mass = (sc.astype(np.float64) - w.prior_weight * prior).sum(axis=2)
    assert np.all(np.abs(mass - w.window) < 0.02 * w.window)


@pytest.mark.parametrize("wgs", [0, 5, 61, 2048])
@pytest.mark.parametrize("variant", [0, 8])
def test_workgroups_enter_the_tile_sequence_anywhere(wgs, variant):
    """More than 16 requests: a workgroup finds the request its range starts in with a cooperative search and then
    walks from request to request.  Forced grid sizes put the range starts anywhere (inside leads, on the last
    request, in the second problem); with the prefix-only softmax some requests have no tile at all."""
    rng = np.random.default_rng(77)
    lens = [int(x) for x in rng.choice([32, 33, 64, 100, 257, 900, 2100], size=45)]
    lens[7] = 32; lens[44] = 32                                       # nothing but the window (also as the last request)
    w = wl.scaled(wl.ragged_agentic(), n_layers=2, seqlens=lens, budgets=[max(32, n // 4) for n in lens], window=32,
                  n_kv_heads=2, n_q_heads=6)
    run_case(w, variant=variant, score_workgroups=wgs)


def test_many_short_requests():
    """300 packed requests of 40..167 tokens: every per-request lookup (tile sequence, merge, pooling, select) at scale."""
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(40, 168, size=300)]
    w = wl.scaled(wl.ragged_agentic(), seqlens=lens, budgets=[max(32, n // 3) for n in lens], window=32,
                  n_kv_heads=2, n_q_heads=4)
    run_case(w)


def test_very_many_very_short_requests():
    """400 packed requests of 8..24 tokens with a window of 4: a 2048-token tile of the pooling kernel meets over a
    hundred requests (beyond the 64 whose bounds a wave keeps in one register, so every token looks its request up),
    and most requests are shorter than two pooling widths."""
    rng = np.random.default_rng(8)
    lens = [int(x) for x in rng.integers(8, 25, size=400)]
    w = wl.scaled(wl.ragged_agentic(), seqlens=lens, budgets=[max(4, n // 2) for n in lens], window=4,
                  n_kv_heads=2, n_q_heads=4)
    run_case(w)


def test_compress_replays_from_a_hip_graph():
    """The fused call captured into a graph: no allocation, no synchronisation, no memset inside.  Replays are
    interleaved with eager work on other inputs and must reproduce the eager result bit for bit every time."""
    import torch
    b = _binding()
    w = wl.scaled(wl.qwen7b_32k(), n_layers=2, seqlens=[3000, 700], budgets=[300, 100])
    q, k, v, prior = wl.make_all(w)
    prob = b.DeviceProblem(w, q, k, v, prior)
    prob.compress()                                   # eager reference (and first-call set-up outside the capture)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (prob.scores, prob.idx, prob.k_out, prob.v_out)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        prob.compress()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        prob.compress()
    other = b.DeviceProblem(wl.tiny(), *wl.make_all(wl.tiny()))
    for _ in range(3):
        for t in (prob.scores, prob.k_out, prob.v_out):
            t.zero_()
        prob.idx.fill_(-1)
        prob.workspace.fill_(0xFF)
        other.compress()                              # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((prob.scores, prob.idx, prob.k_out, prob.v_out), ref):
            assert torch.equal(got.view(torch.uint8) if got.dtype == torch.bfloat16 else got,
                               want.view(torch.uint8) if want.dtype == torch.bfloat16 else want)


# ------------------------------------------------------------------ FP8 (E4M3) cache

def test_fp8_cache_tiny_and_ragged():
    run_case(wl.tiny(), fused=False, kv="fp8_e4m3")
    run_case(wl.tiny(), fused=True, kv="fp8_e4m3")
    w = wl.scaled(wl.ragged_agentic(), seqlens=[700, 1300, 64, 2049, 1024, 65], budgets=[70, 130, 64, 204, 1024, 65])
    run_case(w, kv="fp8_e4m3")


def test_fp8_cache_model_shapes():
    """Eight waves with shared row blocks (448 rows), a ragged last tile, head_dim 128; four waves; two row splits."""
    run_case(wl.scaled(wl.qwen7b_32k(), n_layers=2, seqlens=[5000]), kv="fp8_e4m3")
    run_case(wl.scaled(wl.llama8b_64k(), n_layers=2, seqlens=[3001], n_q_heads=8, n_kv_heads=2), kv="fp8_e4m3")
    run_case(wl.scaled(wl.long_128k(), n_layers=1, seqlens=[4100], n_kv_heads=2, n_q_heads=14), kv="fp8_e4m3")


@pytest.mark.parametrize("variant", [2, 1 | 4 | 8 | 16])
def test_fp8_cache_with_score_variants(variant):
    w = wl.scaled(wl.qwen7b_32k(), n_layers=1, seqlens=[1500, 64, 700], budgets=[150, 64, 90], n_kv_heads=2, n_q_heads=14)
    run_case(w, variant=variant, kv="fp8_e4m3")


@pytest.mark.parametrize("band", range(8))
def test_fp8_every_code_is_read_as_its_value(band):
    """Keys drawn from 16 neighbouring magnitude codes (both signs) at a time, from the subnormals up to 448, with
    the queries scaled so that the logits are of order one: a code widened to the wrong number moves the scores."""
    import torch
    b = _binding()
    g = np.random.default_rng(500 + band)
    w = wl.scaled(wl.tiny(), n_layers=1, seqlens=[333], budgets=[80], prior_weight=0.0)
    d, n = w.head_dim, 333
    mags = np.arange(16 * band, min(16 * band + 16, 0x7F), dtype=np.uint8)              # 0x7f is NaN
    k = (g.choice(mags, size=(1, w.n_kv_heads, n, d)) | (g.integers(0, 2, size=(1, w.n_kv_heads, n, d)) << 7)).astype(np.uint8)
    rms = float(np.sqrt(np.mean(orc.fp8_e4m3_to_f64(mags).astype(np.float64) ** 2)))
    q = wl.f32_to_bf16_bits((g.standard_normal((1, 1, w.n_q_heads, w.window, d)) * (2.0 / rms)).astype(np.float32))
    prior = np.zeros(n, dtype=np.float32)
    prob = b.DeviceProblem(w, q, k, k[:, ::-1].copy(), prior)
    prob.compress()
    torch.cuda.synchronize()
    ref = orc.score_packed(q, k, prior, w.cu_seqlens(), pool_kernel=w.pool_kernel, prior_weight=0.0, k_format="fp8_e4m3")
    assert ref.std() > 0.2 * ref.mean()                        # the softmax is far from flat: the key values matter
    pu.assert_scores_close(prob.scores.cpu().numpy(), ref)
    idx = prob.idx.cpu().numpy()
    assert np.array_equal(b.DeviceProblem.bits(prob.k_out), pu.host_gather(k, idx, w.cu_seqlens(), w.cu_budgets()))
    assert np.array_equal(b.DeviceProblem.bits(prob.v_out), pu.host_gather(k[:, ::-1], idx, w.cu_seqlens(), w.cu_budgets()))


def test_fp8_scores_equal_the_scores_of_the_same_numbers_in_bf16():
    """Every E4M3 number is a bf16 number: the two caches holding the same values must give the same bits."""
    import torch
    b = _binding()
    w = wl.scaled(wl.qwen7b_32k(), n_layers=1, seqlens=[2100, 300], budgets=[300, 100])
    q, k, v, prior = wl.make_all(w)
    k8 = wl.bf16_bits_to_fp8_codes(k)
    same = torch.from_numpy(k8).view(torch.float8_e4m3fn).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    p8 = b.DeviceProblem(w, q, k8, k8, prior)
    p16 = b.DeviceProblem(w, q, same, same, prior)
    p8.compress(); p16.compress()
    torch.cuda.synchronize()
    assert torch.equal(p8.scores, p16.scores) and torch.equal(p8.idx, p16.idx)


@pytest.mark.parametrize("seed", range(24))
def test_random_valid_shapes(seed):
    """Seeded random draws over everything the parameters allow at small sizes: head counts and group sizes (one to
    sixteen row blocks: every wave count and row-block layout), window, head_dim, request mix, pool width, prior
    weight, score-tail variants, cache type; additive selection against the oracle as in every other case."""
    g = np.random.default_rng(9000 + seed)
    d = int(g.choice([64, 128]))
    h_kv = int(g.integers(1, 4))
    group = int(g.integers(1, 9))
    window = int(g.choice([1, 7, 16, 32, 33, 48, 64, 96]))
    n_seqs = int(g.integers(1, 5))
    lens = [int(window + g.integers(0, 1800)) for _ in range(n_seqs)]
    budgets = [int(g.integers(window, n + 1)) for n in lens]
    variant = int(g.choice([0, 0, 1, 4, 8, 16, 8 | 16, 1 | 4]))
    if window % 32 == 0 and group * window <= 512 and g.random() < 0.3:
        variant = (variant & ~1) | 2                                   # largest head mass
    kv = "fp8_e4m3" if g.random() < 0.35 else "bf16"
    w = wl.scaled(wl.qwen7b_32k(), name=f"rand{seed}", n_layers=int(g.integers(1, 3)), seqlens=lens, budgets=budgets,
                  window=window, head_dim=d, n_kv_heads=h_kv, n_q_heads=h_kv * group,
                  pool_kernel=int(g.choice([1, 3, 5, 7, 9, 21])), prior_weight=float(g.choice([0.0, 0.5, 1.0, 3.0])))
    run_case(w, fused=bool(g.integers(0, 2)), variant=variant, kv=kv)


@pytest.mark.parametrize("seed", range(6))
def test_random_batches_with_long_requests_end_to_end(seed):
    """Like test_random_valid_shapes, but every batch holds a request long enough for the selection to run by parts
    (few heads and a small window keep the oracle quick): score, select and gather against the oracle."""
    g = np.random.default_rng(7700 + seed)
    window = int(g.choice([16, 32, 64]))
    n_seqs = int(g.integers(1, 4))
    lens = [int(window + g.integers(0, 3000)) for _ in range(n_seqs)]
    lens[int(g.integers(0, n_seqs))] = window + int(g.choice([16384, 20011, 40000, 70001]))
    budgets = [int(g.choice([window, window + (n - window) // 16, window + (n - window) // 2, n])) for n in lens]
    h_kv = int(g.integers(1, 3))
    group = int(g.choice([1, 2, 4]))
    kv = "fp8_e4m3" if g.random() < 0.3 else "bf16"
    w = wl.scaled(wl.qwen7b_32k(), name=f"randlong{seed}", n_layers=1, seqlens=lens, budgets=budgets, window=window,
                  head_dim=int(g.choice([64, 128])), n_kv_heads=h_kv, n_q_heads=h_kv * group,
                  pool_kernel=int(g.choice([1, 5, 7])), prior_weight=float(g.choice([0.0, 1.0, 2.0])))
    run_case(w, fused=bool(g.integers(0, 2)), kv=kv)
    if seed % 2 == 0:
        run_two_stage(w, float(g.choice([0.25, 0.5, 1.0])), int(g.choice([0, 100])), fused=True)


def test_readme_example_runs_as_written():
    """The usage example of the README, taken from the file and executed: its marked tokens and its window are kept,
    and the compact cache holds the rows the indices name."""
    import os
    import torch
    text = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "README.md")).read()
    lines = text[text.index("    import numpy as np, torch"):].splitlines()
    stop = next(i for i, line in enumerate(lines) if line.strip() and not line.startswith("    "))   # end of the indented block
    code = "\n".join(line[4:] for line in lines[:stop])
    ns = {}
    exec(compile(code, "README.md", "exec"), ns)
    torch.cuda.synchronize()
    idx, k, k_out, N, W, B = ns["idx"].cpu().numpy(), ns["k"], ns["k_out"], ns["N"], ns["W"], ns["B"]
    assert (np.diff(idx, axis=-1) > 0).all() and idx.min() >= 0 and idx.max() == N - 1
    assert (idx[..., -W:] == np.arange(N - W, N)).all()
    marked = np.arange(100, 140)
    assert all(np.isin(marked, idx[l, h]).all() for l in range(idx.shape[0]) for h in range(idx.shape[1]))
    want = torch.gather(k, 2, ns["idx"].long().unsqueeze(-1).expand(-1, -1, -1, k.shape[-1]))
    assert torch.equal(k_out, want)


def test_a_plain_c_program_compresses_through_the_c_abi():
    """csrc/abi_demo.c (built with the library): HIP runtime + codecomp.h only, no Python in the call path; it checks
    its own outputs and says so."""
    import os
    import subprocess
    from paper_2604_10235_amd import build
    assert os.path.exists(build.ABI_DEMO), "abi_demo.exe is missing: build first (python -m paper_2604_10235_amd.build)"
    r = subprocess.run([build.ABI_DEMO], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.startswith("abi_demo: ok"), (r.returncode, r.stdout, r.stderr)
