"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
public header declares, and rejects bad arguments with the documented codes before any launch."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2604_10235_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built():
    if not os.path.exists(b.LIB_PATH):
        from paper_2604_10235_amd import build
        build.build_library(verbose=False)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "codecomp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(codecomp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"codecomp_score", "codecomp_select", "codecomp_gather", "codecomp_compress",
            "codecomp_workspace_bytes", "codecomp_validate", "codecomp_status_string", "codecomp_version",
            "codecomp_score_stages", "codecomp_select_two_stage", "codecomp_structure_score",
            "codecomp_chunk_budgets", "codecomp_chunk_structure_scores", "codecomp_score_layout"} <= set(names)
    lib = b.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_peaks_library_exports_its_declared_symbol():
    from paper_2604_10235_amd import peaks
    text = open(os.path.join(ROOT, "include", "codecomp_peaks.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(codecomp_[a-z_]+)\s*\(", text)))
    assert names == ["codecomp_measure_pass_model", "codecomp_measure_peaks"]
    lib = C.CDLL(peaks.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    # 8 doubles and 3 int32 (+ padding to 8): the binding's mirror of the struct
    assert C.sizeof(peaks.codecomp_peaks) == 8 * 8 + 16 and peaks.codecomp_peaks.mix_waves_per_simd.offset == 64
    # bad arguments are refused on the host
    lib.codecomp_measure_peaks.restype = C.c_int
    lib.codecomp_measure_peaks.argtypes = [C.c_void_p] * 3 + [C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
    out = peaks.codecomp_peaks()
    assert lib.codecomp_measure_peaks(None, 0x1000, 0x1000, 1 << 20, 0x1000, C.byref(out), None) == -1
    assert lib.codecomp_measure_peaks(0x1000, 0x1000, 0x1000, 1000, 0x1000, C.byref(out), None) == -1
    # the pass model: 12 rows of 2 int32 + 4 doubles, 4 int32 after them
    assert C.sizeof(peaks.codecomp_pass_model_row) == 40 and C.sizeof(peaks.codecomp_pass_model) == 12 * 40 + 16
    assert peaks.codecomp_pass_model.n_rows.offset == 480 and peaks.codecomp_pass_model.status.offset == 488
    header = open(os.path.join(ROOT, "include", "codecomp_peaks.h")).read()
    assert int(re.search(r"#define CODECOMP_PASS_MODEL_MAX_ROWS (\d+)", header).group(1)) == peaks.PASS_MODEL_MAX_ROWS
    for bit, _ in peaks.PASS_MODEL_FEATURES.items():
        assert re.search(r"#define CODECOMP_PASS_MODEL_[A-Z]+ %d\b" % bit, header), bit
    lib.codecomp_measure_pass_model.restype = C.c_int
    lib.codecomp_measure_pass_model.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
    pm = peaks.codecomp_pass_model()
    assert lib.codecomp_measure_pass_model(None, 0x1000, 1 << 30, 0x1000, C.byref(pm), None) == -1
    assert lib.codecomp_measure_pass_model(0x1000, 0x1000, (1 << 30) + 8, 0x1000, C.byref(pm), None) == -1


def test_headers_compile_as_plain_c_and_a_c_program_links(tmp_path):
    """The boundary is a C ABI: both headers go through a C99 compiler with warnings as errors, and a C program that
    calls the host-only entry points links against the library and gets the binding's answers."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "abi.c"
    src.write_text(r"""
#include <stdio.h>
#include <string.h>
#include "codecomp.h"
#include "codecomp_peaks.h"
int main(void) {
  codecomp_params p;
  int32_t cu[2] = {0, 4096}, cb[2] = {0, 512};
  memset(&p, 0, sizeof p);
  p.n_layers = 2; p.n_q_heads = 8; p.n_kv_heads = 2; p.head_dim = 128; p.window = 64; p.pool_kernel = 7;
  p.prior_weight = 1.0f; p.n_seqs = 1;
  p.cu_seqlens_host = cu; p.cu_budgets_host = cb;
  p.cu_seqlens_dev = (const int32_t*)(size_t)4096; p.cu_budgets_dev = (const int32_t*)(size_t)4096;   /* never read here */
  printf("%d %zu %zu %d %s\n", codecomp_validate(&p), codecomp_workspace_bytes(&p), sizeof p, codecomp_version(),
         codecomp_status_string(CODECOMP_EINVAL_POOL));
  p.pool_kernel = 4;
  printf("%d\n", codecomp_validate(&p));
  return 0;
}
""")
    exe = tmp_path / "abi"
    libdir = os.path.dirname(b.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-l:libcodecomp.so", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    rc, ws, size, version, text = out[0].split(" ", 4)
    p = good(n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128, window=64, pool_kernel=7,
             cu_seqlens_host=np.array([0, 4096]), cu_budgets_host=np.array([0, 512]))
    assert int(rc) == 0 and int(ws) == b.codecomp_workspace_bytes(p) and int(size) == C.sizeof(b.codecomp_params)
    assert int(version) == b.version() and text == b.status_string(-5)
    assert int(out[1]) == -5


def test_selection_by_parts_shows_in_the_workspace_size():
    # a request beyond 65536 candidates (or a long one among few problems) is selected by parts of 8192 candidates:
    # 2048 16-bit counts per (layer * head, part)
    def ws(n, layers):
        return b.codecomp_workspace_bytes(good(n_layers=layers, cu_seqlens_host=np.array([0, n]), cu_budgets_host=np.array([0, 100])))
    few, many = 2, 60                                    # 2 KV heads: 4 and 120 (layer, head, request) problems
    assert ws(16 + 16384, few) - ws(16 + 16383, few) >= few * 2 * 2 * 2048 * 2           # two parts from 16384 candidates on
    assert ws(16 + 16384, many) - ws(16 + 16383, many) < 4096 * many                      # many problems: one workgroup each
    assert ws(16 + 65537, many) - ws(16 + 65536, many) >= many * 2 * 9 * 2048 * 2         # nine parts beyond 65536


def test_struct_layout_matches_header():
    # 10 x 4-byte fields, 4 pointers, 10 x int64 strides, span budget (float + int32), variant flags + kv_dtype,
    # the two launch-shape fields
    assert C.sizeof(b.codecomp_params) == 40 + 32 + 80 + 8 + 8 + 8
    assert b.codecomp_params.score_workgroups.offset == 168
    assert b.codecomp_params.score_variant.offset == 160
    assert b.codecomp_params.span_budget_ratio.offset == 152
    assert b.codecomp_params.cu_seqlens_host.offset == 40
    assert b.codecomp_params.q_stride_layer.offset == 72


def good(**over):
    kw = dict(n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128, window=16, pool_kernel=7, prior_weight=1.0,
              cu_seqlens_host=np.array([0, 100, 300]), cu_budgets_host=np.array([0, 20, 60]),
              cu_seqlens_dev=0x1000, cu_budgets_dev=0x2000)
    kw.update(over)
    return b.make_params(**kw)


def test_valid_params_and_workspace_size():
    p = good()
    assert b.codecomp_validate(p) == 0
    for variant in (1, 4, 8, 16, 1 | 4 | 8 | 16):
        assert b.codecomp_validate(good(score_variant=variant)) == 0
    assert b.codecomp_validate(good(score_variant=2 | 4, window=32, cu_budgets_host=np.array([0, 40, 80]))) == 0
    ws = b.codecomp_workspace_bytes(p)
    assert ws > 0 and ws % 256 == 0
    # the raw attention mass alone needs L * H_kv * T floats
    assert ws >= 2 * 2 * 300 * 4


@pytest.mark.parametrize("over,code", [
    (dict(n_layers=0), -2),
    (dict(score_workgroups=-1), -2),
    (dict(score_lead_tiles=65), -2),
    (dict(n_q_heads=7), -6),
    (dict(n_kv_heads=0), -6),
    (dict(head_dim=96), -7),
    (dict(pool_kernel=4), -5),
    (dict(pool_kernel=0), -5),
    (dict(prior_weight=-1.0), -10),
    (dict(prior_weight=float("nan")), -10),
    (dict(softmax_scale=-0.5), -10),
    (dict(window=0), -3),
    (dict(window=101), -3),                                         # W > N_0 = 100
    (dict(cu_budgets_host=np.array([0, 10, 60])), -4),              # B_0 = 10 < W
    (dict(cu_budgets_host=np.array([0, 101, 141])), -4),            # B_0 > N_0
    (dict(cu_seqlens_host=np.array([1, 100, 300])), -8),
    (dict(cu_seqlens_host=np.array([0, 100, 100])), -8),            # empty request
    (dict(cu_seqlens_dev=0), -1),
    (dict(kv_stride_tok=100), -2),                                  # not a multiple of 8 elements
    (dict(kv_stride_tok=64), -2),                                   # rows would overlap
    (dict(select_mode=2), -11),
    (dict(score_variant=32), -11),                                     # unknown flag
    (dict(score_variant=1 | 2), -11),                                  # group sum and max together
    (dict(score_variant=2), -11),                                      # group max needs window % 32 == 0 (16 here)
    (dict(score_variant=2, window=64, n_q_heads=18, cu_seqlens_host=np.array([0, 100, 300]),
          cu_budgets_host=np.array([0, 70, 140])), -11),                # group max needs all rows in one workgroup (9 * 64 > 512)
    (dict(kv_dtype=2), -11),
    (dict(kv_dtype=-1), -11),
    (dict(kv_dtype=1, kv_stride_tok=136), -2),      # FP8 rows move as 16-byte pieces of 16 elements
    (dict(select_mode=1, span_budget_ratio=1.5), -11),
    (dict(select_mode=1, span_budget_ratio=0.5, span_budget_min=-1), -11),
    (dict(pool_kernel=1027), -5),
])
def test_rejected_parameters(over, code):
    p = good(**over)
    assert b.codecomp_validate(p) == code
    assert b.codecomp_workspace_bytes(p) == 0
    assert b.status_string(code)


def test_launching_calls_validate_before_touching_a_gpu():
    # fake, well-aligned, non-null "device" pointers: every call must fail in validation, nothing is launched
    lib = b.lib()
    fake = 0x10000
    p = good(head_dim=96)
    assert lib.codecomp_score(fake, fake, fake, C.byref(p), fake, fake, 1 << 30, None) == -7
    assert lib.codecomp_select(fake, C.byref(p), fake, fake, 1 << 30, None) == -7
    assert lib.codecomp_gather(fake, fake, fake, C.byref(p), fake, fake, None) == -7
    assert lib.codecomp_compress(fake, fake, fake, fake, C.byref(p), fake, fake, fake, fake, fake, 1 << 30, None) == -7
    p = good()
    assert lib.codecomp_score(None, fake, fake, C.byref(p), fake, fake, 1 << 30, None) == -1
    assert lib.codecomp_score(fake, fake, fake, C.byref(p), fake, fake, 16, None) == -9       # workspace too small
    assert lib.codecomp_score(fake, fake, fake, C.byref(p), fake, fake + 8, 1 << 30, None) == -9  # misaligned
    assert lib.codecomp_score(fake + 2, fake, fake, C.byref(p), fake, fake, 1 << 30, None) == -2  # q not 16-byte aligned
    assert lib.codecomp_score_stages(fake, fake, fake, C.byref(p), fake, fake, 1 << 30, 0, None) == -2
    assert lib.codecomp_score_stages(fake, fake, fake, C.byref(p), fake, fake, 1 << 30, 16, None) == -2
    assert lib.codecomp_compress(fake, fake, None, fake, C.byref(p), fake, fake, fake, fake, fake, 1 << 30, None) == -1
    # the two selection entry points refuse the other mode
    assert lib.codecomp_select_two_stage(fake, fake, C.byref(p), fake, fake, 1 << 30, None) == -11
    p2 = good(select_mode=1, span_budget_ratio=0.5)
    assert lib.codecomp_select(fake, C.byref(p2), fake, fake, 1 << 30, None) == -11
    assert lib.codecomp_structure_score(None, fake, C.byref(p), fake, None) == -1


def test_static_scratch_call_validates_on_the_host():
    # the call without workspace arguments: same checks, and parameters that need more scratch than the library's
    # device array holds are rejected before anything touches a GPU
    from paper_2604_10235_amd import workloads as wl
    lib = b.lib()
    fake = 0x10000
    assert lib.codecomp_compress_static(fake, fake, fake, fake, C.byref(good(head_dim=96)), fake, fake, fake, fake, None) == -7
    assert lib.codecomp_compress_static(fake, fake, None, fake, C.byref(good()), fake, fake, fake, fake, None) == -1
    assert lib.codecomp_compress_static(fake, fake + 4, fake, fake, C.byref(good()), fake, fake, fake, fake, None) == -2
    w = wl.long_128k()
    p = b.make_params(n_layers=w.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                      window=w.window, pool_kernel=w.pool_kernel, prior_weight=w.prior_weight,
                      cu_seqlens_host=w.cu_seqlens(), cu_budgets_host=w.cu_budgets(), cu_seqlens_dev=256, cu_budgets_dev=256)
    assert b.codecomp_workspace_bytes(p) > b.STATIC_SCRATCH_BYTES
    assert lib.codecomp_compress_static(fake, fake, fake, fake, C.byref(p), fake, fake, fake, fake, None) == -9
    text = open(os.path.join(ROOT, "include", "codecomp.h")).read()
    assert re.search(r"#define CODECOMP_STATIC_SCRATCH_BYTES \(32 \* 1024 \* 1024\)", text) and b.STATIC_SCRATCH_BYTES == 32 << 20


def test_binding_raises_with_status_text():
    with pytest.raises(b.CodecompError) as e:
        b._check(-4, "codecomp_select")
    assert "BUDGET" in str(e.value)


def test_workload_recipes():
    from paper_2604_10235_amd import workloads as wl
    for name, mk in wl.CONFIGS.items():
        w = mk()
        assert all(w.window <= bb <= n for bb, n in zip(w.budgets, w.seqlens)), name
    w = wl.ragged_agentic()
    assert w.n_seqs == 16 and all(8192 <= n <= 49152 for n in w.seqlens)
    assert all(bb == int(0.08 * n) for bb, n in zip(w.budgets, w.seqlens))
    t = wl.tiny()
    q, k, v, prior = wl.make_all(t)
    assert q.shape == (1, 1, 4, 32, 64) and k.shape == (1, 4, 2048, 64) and prior.shape == (2048,)
    assert set(np.unique(prior)) == {0.0, 1.0}
    q2, k2, _, prior2 = wl.make_all(t)
    assert np.array_equal(k, k2) and np.array_equal(q, q2) and np.array_equal(prior, prior2)   # seeded
    # bf16 rounding is round-to-nearest-even
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.140625], dtype=np.float32)
    import torch
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.f32_to_bf16_bits(x), ref)


def test_host_budget_functions_match_oracle():
    from oracle import codecomp_oracle as orc
    g = np.random.default_rng(5)
    feats = g.integers(0, 60, size=(9, 6)).astype(np.float64)
    tau = np.array([20.0, 12.0, 6.0, 30.0, 80.0, 50.0]); wts = np.array([0.2, 0.18, 0.14, 0.14, 0.17, 0.17])
    sigma = b.codecomp_chunk_structure_scores(feats, tau, wts)
    np.testing.assert_allclose(sigma, orc.chunk_structure_score(feats, tau, wts), rtol=1e-14)
    lens = g.integers(128, 4097, size=9)
    kw = dict(ratio=0.4, m_min=0.5, m_max=1.5, r_max=0.9, eps=1e-6)
    got = b.codecomp_chunk_budgets(sigma, lens, window=0, **kw)
    assert np.array_equal(got, orc.chunk_budgets(sigma, lens, **kw))
    # equal scores -> multiplier midway; the window clamp only ever raises a budget, the chunk length caps it
    got = b.codecomp_chunk_budgets(np.ones(3), [1000, 100, 70], window=64, **kw)
    assert list(got) == [400, 64, 64]
    got = b.codecomp_chunk_budgets([0.0, 1.0], [100, 100], ratio=2.0, m_min=0.5, m_max=1.5, r_max=5.0, eps=1e-6, window=8)
    assert list(got) == [100, 100]
    with pytest.raises(b.CodecompError):
        b.codecomp_chunk_budgets(np.ones(2), [10, 10], window=11, **kw)
    with pytest.raises(b.CodecompError):
        b.codecomp_chunk_structure_scores(feats, np.zeros(6), wts)


@pytest.mark.parametrize("group,window", [(1, 1), (1, 32), (1, 64), (4, 32), (7, 32), (4, 64), (5, 64), (6, 64), (7, 64),
                                          (8, 64), (7, 128), (3, 100), (9, 64), (13, 40), (16, 64)])
def test_score_layout_covers_every_row_block_once_and_evens_out_the_simds(group, window):
    """Every (row block, half tile) unit has exactly one owner, and with more than four waves (one workgroup
    per compute unit, waves w and w+4 on one SIMD) the four SIMDs carry the same number of units +-1."""
    n = max(256, 2 * window)
    p = good(n_q_heads=2 * group, n_kv_heads=2, window=window, cu_seqlens_host=np.array([0, n]),
             cu_budgets_host=np.array([0, window + 8]))
    rc, splits, blocks, waves, desc = b.codecomp_score_layout(p)
    assert rc == 0
    rows = group * window
    assert splits == -(-rows // 512) and splits * blocks * 32 >= rows and 1 <= waves <= 8 and blocks <= 16
    assert (blocks - 1) * 32 * splits < rows + 32 * splits          # no block beyond what the rows need
    owners = np.zeros((blocks, 2), dtype=int)                       # owners[block][half]
    load = np.zeros(8, dtype=int)
    for w in range(waves):
        rb0, rb1, halves = desc[w] & 255, (desc[w] >> 8) & 255, (desc[w] >> 16) & 3
        assert rb0 < blocks
        owners[rb0] += 1
        load[w] += 2
        for h in range(2):
            if halves >> h & 1:
                assert rb1 < blocks and rb1 != rb0
                owners[rb1][h] += 1
                load[w] += 1
    assert (owners == 1).all()
    assert all(d == 0 for d in desc[waves:])
    if waves > 4:
        simd = load[:4] + load[4:]
        assert simd.max() - simd.min() <= 1, (desc, simd)
        assert simd.max() == -(-2 * blocks // 4)
