"""ctypes binding of libcodecomp.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; nothing here computes.  Tensors are
torch CUDA(ROCm) tensors used as device memory, the stream is torch's current stream.  The
library must have been built in-tree (paper_2604_10235_amd/build.py); loading fails loudly
otherwise - there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# CODECOMP_LIB selects another build of the same library (experiments); the default is the in-tree one
LIB_PATH = os.environ.get("CODECOMP_LIB") or os.path.join(_HERE, "libcodecomp.so")

STATUS = {
    0: "CODECOMP_OK", -1: "CODECOMP_EINVAL_NULL", -2: "CODECOMP_EINVAL_SHAPE", -3: "CODECOMP_EINVAL_WINDOW",
    -4: "CODECOMP_EINVAL_BUDGET", -5: "CODECOMP_EINVAL_POOL", -6: "CODECOMP_EINVAL_HEADS",
    -7: "CODECOMP_EINVAL_HEADDIM", -8: "CODECOMP_EINVAL_SEQLENS", -9: "CODECOMP_EINVAL_WORKSPACE",
    -10: "CODECOMP_EINVAL_PRIOR", -11: "CODECOMP_EINVAL_MODE",
}


class codecomp_params(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("window", C.c_int32), ("pool_kernel", C.c_int32), ("prior_weight", C.c_float), ("softmax_scale", C.c_float),
        ("n_seqs", C.c_int32), ("select_mode", C.c_int32),
        ("cu_seqlens_host", C.c_void_p), ("cu_seqlens_dev", C.c_void_p),
        ("cu_budgets_host", C.c_void_p), ("cu_budgets_dev", C.c_void_p),
        ("q_stride_layer", C.c_int64), ("q_stride_seq", C.c_int64), ("q_stride_head", C.c_int64),
        ("q_stride_tok", C.c_int64),
        ("kv_stride_layer", C.c_int64), ("kv_stride_head", C.c_int64), ("kv_stride_tok", C.c_int64),
        ("out_stride_layer", C.c_int64), ("out_stride_head", C.c_int64), ("out_stride_tok", C.c_int64),
        ("span_budget_ratio", C.c_float), ("span_budget_min", C.c_int32),
        ("score_variant", C.c_int32), ("kv_dtype", C.c_int32),
        ("score_workgroups", C.c_int32), ("score_lead_tiles", C.c_int32),
    ]


class CodecompError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({STATUS.get(status, 'hipError_t' if status > 0 else '?')}): "
                         f"{status_string(status)}")


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built: the HIP path has no substitute."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2604_10235_amd.build)")
        # The device memory and the streams that this binding hands to the library come from torch, which ships
        # its own HIP runtime.  Loaded first, that runtime is the one the library binds to; the other way round
        # the process ends up with two runtimes and every launch fails with hipErrorNoDevice.
        import torch  # noqa: F401
        l = C.CDLL(LIB_PATH)
        P = C.POINTER(codecomp_params)
        l.codecomp_workspace_bytes.restype = C.c_size_t
        l.codecomp_workspace_bytes.argtypes = [P]
        l.codecomp_validate.restype = C.c_int
        l.codecomp_validate.argtypes = [P]
        l.codecomp_score_layout.restype = C.c_int
        l.codecomp_score_layout.argtypes = [P, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                            C.POINTER(C.c_uint32)]
        l.codecomp_score.restype = C.c_int
        l.codecomp_score.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_size_t,
                                     C.c_void_p]
        l.codecomp_score_stages.restype = C.c_int
        l.codecomp_score_stages.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_size_t,
                                            C.c_uint, C.c_void_p]
        l.codecomp_select.restype = C.c_int
        l.codecomp_select.argtypes = [C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.codecomp_select_two_stage.restype = C.c_int
        l.codecomp_select_two_stage.argtypes = [C.c_void_p, C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.codecomp_gather.restype = C.c_int
        l.codecomp_gather.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, P, C.c_void_p, C.c_void_p, C.c_void_p]
        l.codecomp_compress.restype = C.c_int
        l.codecomp_compress.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, P, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        l.codecomp_compress_static.restype = C.c_int
        l.codecomp_compress_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, P, C.c_void_p, C.c_void_p,
                                               C.c_void_p, C.c_void_p, C.c_void_p]
        l.codecomp_structure_score.restype = C.c_int
        l.codecomp_structure_score.argtypes = [C.c_void_p, C.c_void_p, P, C.c_void_p, C.c_void_p]
        DP, IP = C.POINTER(C.c_double), C.POINTER(C.c_int32)
        l.codecomp_chunk_structure_scores.restype = C.c_int
        l.codecomp_chunk_structure_scores.argtypes = [DP, DP, DP, C.c_int32, C.c_int32, DP]
        l.codecomp_chunk_budgets.restype = C.c_int
        l.codecomp_chunk_budgets.argtypes = [DP, IP, C.c_int32, C.c_double, C.c_double, C.c_double, C.c_double,
                                             C.c_double, C.c_int32, IP]
        l.codecomp_status_string.restype = C.c_char_p
        l.codecomp_status_string.argtypes = [C.c_int]
        l.codecomp_version.restype = C.c_int
        l.codecomp_version.argtypes = []
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().codecomp_status_string(int(status)).decode()


def version() -> int:
    return lib().codecomp_version()


def make_params(*, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int, window: int, pool_kernel: int,
                prior_weight: float, cu_seqlens_host: np.ndarray, cu_budgets_host: np.ndarray,
                cu_seqlens_dev: int = 0, cu_budgets_dev: int = 0, softmax_scale: float = 0.0, **strides):
    """Fills a codecomp_params.  The host arrays are kept alive on the returned object; the device
    pointers are plain integers (tensor.data_ptr())."""
    csl = np.ascontiguousarray(cu_seqlens_host, dtype=np.int32)
    cbl = np.ascontiguousarray(cu_budgets_host, dtype=np.int32)
    p = codecomp_params()
    p.n_layers, p.n_q_heads, p.n_kv_heads, p.head_dim = n_layers, n_q_heads, n_kv_heads, head_dim
    p.window, p.pool_kernel, p.prior_weight, p.softmax_scale = window, pool_kernel, prior_weight, softmax_scale
    p.n_seqs = len(csl) - 1
    p.cu_seqlens_host = csl.ctypes.data
    p.cu_budgets_host = cbl.ctypes.data
    p.cu_seqlens_dev = cu_seqlens_dev
    p.cu_budgets_dev = cu_budgets_dev
    for name, val in strides.items():      # strides, select_mode, span_budget_*, score_variant, kv_dtype, score_workgroups ...
        setattr(p, name, val)
    p._keep = (csl, cbl)
    return p


def codecomp_validate(params: codecomp_params) -> int:
    return lib().codecomp_validate(C.byref(params))


def codecomp_score_layout(params: codecomp_params):
    """(status, row_splits, row_blocks, waves, wave_desc[8]) of the score passes for these parameters."""
    rs, rb, nw = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    desc = (C.c_uint32 * 8)()
    rc = lib().codecomp_score_layout(C.byref(params), C.byref(rs), C.byref(rb), C.byref(nw), desc)
    return rc, rs.value, rb.value, nw.value, list(desc)


def codecomp_workspace_bytes(params: codecomp_params) -> int:
    return lib().codecomp_workspace_bytes(C.byref(params))


def _ptr(t) -> int:
    return 0 if t is None else int(t.data_ptr())


def _stream() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != 0:
        raise CodecompError(rc, where)


def codecomp_score(q_obs, k, prior, params, scores, workspace) -> None:
    _check(lib().codecomp_score(_ptr(q_obs), _ptr(k), _ptr(prior), C.byref(params), _ptr(scores), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream()), "codecomp_score")


STAGE_ROW_STATS, STAGE_ROW_MERGE, STAGE_MASS, STAGE_FINISH, STAGE_ALL = 1, 2, 4, 8, 15
VARIANT_GROUP_SUM, VARIANT_GROUP_MAX, VARIANT_POOL_MAX, VARIANT_SOFTMAX_PREFIX, VARIANT_POOL_PREFIX = 1, 2, 4, 8, 16
KV_BF16, KV_FP8_E4M3 = 0, 1


def codecomp_score_stages(q_obs, k, prior, params, scores, workspace, stages: int) -> None:
    _check(lib().codecomp_score_stages(_ptr(q_obs), _ptr(k), _ptr(prior), C.byref(params), _ptr(scores),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(), int(stages),
                                       _stream()), "codecomp_score_stages")


def codecomp_select(scores, params, idx, workspace) -> None:
    _check(lib().codecomp_select(_ptr(scores), C.byref(params), _ptr(idx), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream()), "codecomp_select")


def codecomp_select_two_stage(scores, prior, params, idx, workspace) -> None:
    _check(lib().codecomp_select_two_stage(_ptr(scores), _ptr(prior), C.byref(params), _ptr(idx), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream()),
           "codecomp_select_two_stage")


def codecomp_gather(k, v, idx, params, k_out, v_out) -> None:
    _check(lib().codecomp_gather(_ptr(k), _ptr(v), _ptr(idx), C.byref(params), _ptr(k_out), _ptr(v_out), _stream()),
           "codecomp_gather")


def codecomp_compress(q_obs, k, v, prior, params, scores, idx, k_out, v_out, workspace) -> None:
    _check(lib().codecomp_compress(_ptr(q_obs), _ptr(k), _ptr(v), _ptr(prior), C.byref(params), _ptr(scores),
                                   _ptr(idx), _ptr(k_out), _ptr(v_out), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()), "codecomp_compress")


STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


def codecomp_compress_static(q_obs, k, v, prior, params, scores, idx, k_out, v_out) -> None:
    _check(lib().codecomp_compress_static(_ptr(q_obs), _ptr(k), _ptr(v), _ptr(prior), C.byref(params), _ptr(scores),
                                          _ptr(idx), _ptr(k_out), _ptr(v_out), _stream()), "codecomp_compress_static")


def codecomp_structure_score(idx, prior, params, retained) -> None:
    _check(lib().codecomp_structure_score(_ptr(idx), _ptr(prior), C.byref(params), _ptr(retained), _stream()),
           "codecomp_structure_score")


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def codecomp_chunk_structure_scores(features, tau, weights) -> np.ndarray:
    f = np.ascontiguousarray(features, dtype=np.float64)
    t = np.ascontiguousarray(tau, dtype=np.float64)
    w = np.ascontiguousarray(weights, dtype=np.float64)
    out = np.empty(f.shape[0], dtype=np.float64)
    _check(lib().codecomp_chunk_structure_scores(_dp(f), _dp(t), _dp(w), f.shape[0], f.shape[1], _dp(out)),
           "codecomp_chunk_structure_scores")
    return out


def codecomp_chunk_budgets(sigma, chunk_len, *, ratio, m_min, m_max, r_max, eps, window) -> np.ndarray:
    s = np.ascontiguousarray(sigma, dtype=np.float64)
    ln = np.ascontiguousarray(chunk_len, dtype=np.int32)
    out = np.empty(len(s), dtype=np.int32)
    ip = C.POINTER(C.c_int32)
    _check(lib().codecomp_chunk_budgets(_dp(s), ln.ctypes.data_as(ip), len(s), ratio, m_min, m_max, r_max, eps, window,
                                        out.ctypes.data_as(ip)), "codecomp_chunk_budgets")
    return out


class DeviceProblem:
    """Device buffers of one workload: inputs uploaded from the host arrays of the workload
    generator, outputs and workspace allocated with torch.  Plumbing only.  k_bits / v_bits of dtype
    uint8 are an FP8 E4M3 cache (kv_dtype = KV_FP8_E4M3), uint16 a bf16 one."""

    def __init__(self, w, q_bits: np.ndarray, k_bits: np.ndarray, v_bits: Optional[np.ndarray], prior: np.ndarray,
                 device: str = "cuda:0", select_mode: int = 0, span_budget_ratio: float = 0.5,
                 span_budget_min: int = 0, score_variant: int = 0, score_workgroups: int = 0, score_lead_tiles: int = 0):
        import torch
        self.w = w
        dev = torch.device(device)

        def up_bits(x):
            return torch.from_numpy(x.view(np.int16)).to(dev).view(torch.bfloat16)

        fp8 = k_bits.dtype == np.uint8
        if v_bits is not None and v_bits.dtype != k_bits.dtype:
            raise ValueError("k and v must have the same storage type")

        def up_kv(x):
            return torch.from_numpy(x).to(dev) if fp8 else up_bits(x)

        self.q = up_bits(q_bits)
        self.k = up_kv(k_bits)
        self.v = up_kv(v_bits) if v_bits is not None else None
        self.prior = torch.from_numpy(prior).to(dev)
        self.n_layers = int(k_bits.shape[0])
        self.cu_seqlens = torch.from_numpy(w.cu_seqlens()).to(dev)
        self.cu_budgets = torch.from_numpy(w.cu_budgets()).to(dev)
        self.params = make_params(n_layers=self.n_layers, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                                  head_dim=w.head_dim, window=w.window, pool_kernel=w.pool_kernel,
                                  prior_weight=w.prior_weight, cu_seqlens_host=w.cu_seqlens(),
                                  cu_budgets_host=w.cu_budgets(), cu_seqlens_dev=_ptr(self.cu_seqlens),
                                  cu_budgets_dev=_ptr(self.cu_budgets), select_mode=select_mode,
                                  span_budget_ratio=span_budget_ratio, span_budget_min=span_budget_min,
                                  score_variant=score_variant, kv_dtype=KV_FP8_E4M3 if fp8 else KV_BF16,
                                  score_workgroups=score_workgroups, score_lead_tiles=score_lead_tiles)
        rc = codecomp_validate(self.params)
        _check(rc, "codecomp_validate")
        T, TB = w.total_tokens, w.total_budget
        self.scores = torch.empty((self.n_layers, w.n_kv_heads, T), dtype=torch.float32, device=dev)
        self.idx = torch.empty((self.n_layers, w.n_kv_heads, TB), dtype=torch.int32, device=dev)
        self.k_out = torch.empty((self.n_layers, w.n_kv_heads, TB, w.head_dim),
                                 dtype=torch.uint8 if fp8 else torch.bfloat16, device=dev)
        self.v_out = torch.empty_like(self.k_out)
        self.workspace = torch.empty(max(256, codecomp_workspace_bytes(self.params)), dtype=torch.uint8, device=dev)

    def score(self):
        codecomp_score(self.q, self.k, self.prior, self.params, self.scores, self.workspace)

    def score_stages(self, stages: int):
        codecomp_score_stages(self.q, self.k, self.prior, self.params, self.scores, self.workspace, stages)

    def select(self):
        if self.params.select_mode == 1:
            codecomp_select_two_stage(self.scores, self.prior, self.params, self.idx, self.workspace)
        else:
            codecomp_select(self.scores, self.params, self.idx, self.workspace)

    def gather(self):
        codecomp_gather(self.k, self.v, self.idx, self.params, self.k_out, self.v_out)

    def compress(self):
        codecomp_compress(self.q, self.k, self.v, self.prior, self.params, self.scores, self.idx, self.k_out,
                          self.v_out, self.workspace)

    def compress_static(self):
        codecomp_compress_static(self.q, self.k, self.v, self.prior, self.params, self.scores, self.idx, self.k_out,
                                 self.v_out)

    @staticmethod
    def bits(t) -> np.ndarray:
        """bf16 tensor -> host uint16 bit patterns (a uint8 tensor of FP8 codes comes back as it is)."""
        import torch
        if t.dtype == torch.uint8:
            return t.cpu().numpy()
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
