"""codecomp_compress_static (the fused call whose scratch memory is a device array inside the library, for
callers that cannot allocate) against codecomp_compress on the same inputs: every output bit for bit, on two
calls in a row, the second with a smaller input, and the size limit as an error."""
import numpy as np
import pytest

from paper_2604_10235_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _outputs(prob):
    import torch
    torch.cuda.synchronize()
    return [prob.scores.cpu().numpy().copy(), prob.idx.cpu().numpy().copy(),
            prob.k_out.view(torch.int16).cpu().numpy().copy(), prob.v_out.view(torch.int16).cpu().numpy().copy()]


def _poison(prob):
    prob.scores.fill_(float("nan")); prob.idx.fill_(-1); prob.k_out.zero_(); prob.v_out.zero_()


def test_static_scratch_call_equals_the_workspace_call_twice_in_a_row():
    from paper_2604_10235_amd import binding as b
    # first call: 448 softmax rows (eight waves, shared row blocks), two requests, ragged tails, two-stage off
    big = wl.scaled(wl.qwen7b_32k(), n_layers=3, seqlens=[9000, 2500], budgets=[700, 250])
    # second call: a smaller input of another shape (four waves, one request), so that it reuses the front of the
    # array that the first call filled
    small = wl.scaled(wl.llama8b_64k(), n_layers=1, seqlens=[1777], budgets=[300], n_q_heads=8, n_kv_heads=2)
    probs = []
    for w in (big, small):
        q, k, v, prior = wl.make_all(w)
        p = b.DeviceProblem(w, q, k, v, prior)
        assert b.codecomp_workspace_bytes(p.params) <= b.STATIC_SCRATCH_BYTES
        p.compress()
        want = _outputs(p)
        probs.append((p, want))
    for p, want in probs:                       # the two static calls back to back, big then small
        _poison(p)
        p.compress_static()
    for p, want in probs:
        got = _outputs(p)
        for g, x in zip(got, want):
            assert np.array_equal(g, x, equal_nan=True)
    # and once more in the other order, with the two-stage rule on the small one
    q, k, v, prior = wl.make_all(small)
    two = b.DeviceProblem(small, q, k, v, prior, select_mode=1, span_budget_ratio=0.5)
    two.compress()
    want_two = _outputs(two)
    _poison(two)
    two.compress_static()
    p, want = probs[0]
    _poison(p)
    p.compress_static()
    for g, x in zip(_outputs(two), want_two):
        assert np.array_equal(g, x, equal_nan=True)
    for g, x in zip(_outputs(p), want):
        assert np.array_equal(g, x, equal_nan=True)
