"""Seeded synthetic inputs for the prefill KV-eviction path (score -> select -> gather).

This module only draws random inputs and packs them as bf16 bit patterns; it holds none of
the method's arithmetic.  Both the CPU oracle tests and the HIP path are fed the *same
arrays* produced here (bits are shared through memory, never regenerated per side).

Tensors (numpy, host):
  q_obs  uint16 (bf16 bits)  [L][n_seqs][H_q][W][d]   observation-window queries
  k, v   uint16 (bf16 bits)  [L][H_kv][sum N_r][d]    cached keys / values, sequences packed
  prior  float32             [sum N_r]                per-token structural prior, shared by
                                                      layers and heads (a property of the text)

The first five workload recipes follow the benchmark configurations of this repository, the sixth
(`paper_chunks`) the compression setting of the paper's appendix; they stand
in for repository-code contexts (head shapes of the named model families, capacity ratios in
the paper's range, span lengths in the range of its structural spans, heavy-hitter key rows
to mimic attention sinks).  No item of any public benchmark is used.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence, Tuple

import numpy as np

MASTER_SEED = 260410235

# tensor ids used in the RNG key
_T_Q, _T_K, _T_V, _T_HEAVY, _T_PRIOR, _T_LENS = 1, 2, 3, 4, 5, 6


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seqlens: Tuple[int, ...]          # N_r per request (one entry = dense)
    window: int                       # W
    budgets: Tuple[int, ...]          # B_r per request (window included)
    pool_kernel: int                  # k (odd)
    prior_weight: float               # lambda
    heavy_rate: float                 # fraction of K rows scaled by heavy_scale
    heavy_scale: float
    drift_amp: float                  # K_t += drift_amp * sin(t / drift_period) on every dim
    drift_period: float
    span_min: int
    span_max: int
    flag_rate: float                  # fraction of spans flagged structural
    prior_lo: float                   # flagged tokens get p ~ U(prior_lo, prior_hi); lo == hi -> constant
    prior_hi: float

    @property
    def n_seqs(self) -> int:
        return len(self.seqlens)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seqlens))

    @property
    def total_budget(self) -> int:
        return int(sum(self.budgets))

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seqlens)]).astype(np.int32)

    def cu_budgets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.budgets)]).astype(np.int32)


def _rng(cfg_id: int, tensor: int, layer: int = 0, extra: int = 0) -> np.random.Generator:
    key = [MASTER_SEED, (cfg_id << 48) | (tensor << 40) | (layer << 20) | extra]
    return np.random.Generator(np.random.Philox(key=key))


def ragged_lengths(cfg_id: int, n_seqs: int, lo: int, hi: int) -> Tuple[int, ...]:
    g = _rng(cfg_id, _T_LENS)
    return tuple(int(x) for x in g.integers(lo, hi + 1, size=n_seqs))


def _make(name, cfg_id, L, hq, hkv, d, seqlens, W, budgets, k, lam, heavy_rate, drift, spans, flag, plo, phi):
    return Workload(name, cfg_id, L, hq, hkv, d, tuple(seqlens), W, tuple(budgets), k, lam,
                    heavy_rate, 4.0, drift, 512.0, spans[0], spans[1], flag, plo, phi)


def tiny() -> Workload:
    """Config 1: single layer, no GQA, d=64, N=2048, W=32, B=256; binary prior, 20 % of spans flagged."""
    return _make("tiny", 1, 1, 4, 4, 64, [2048], 32, [256], 7, 1.0, 0.02, 0.0, (4, 12), 0.20, 1.0, 1.0)


def qwen7b_32k() -> Workload:
    """Config 2: 28 layers, 28 q / 4 kv heads, d=128, N=32768, W=64, B=2048; p~U(0.5,1) on 15 % of spans."""
    return _make("qwen7b_32k", 2, 28, 28, 4, 128, [32768], 64, [2048], 7, 1.0, 0.02, 0.0, (4, 12), 0.15, 0.5, 1.0)


def llama8b_64k() -> Workload:
    """Config 3: 32 layers, 32 q / 8 kv heads, N=65536, W=64, B=4096, lambda=0.5; drifting keys, binary prior."""
    return _make("llama8b_64k", 3, 32, 32, 8, 128, [65536], 64, [4096], 7, 0.5, 0.01, 0.3, (4, 12), 0.25, 1.0, 1.0)


def long_128k() -> Workload:
    """Config 4: 28 layers, 28 q / 4 kv heads, N=131072, W=128, B=13107, lambda=2; binary prior, spans 2-24."""
    return _make("long_128k", 4, 28, 28, 4, 128, [131072], 128, [13107], 7, 2.0, 0.0, 0.0, (2, 24), 0.10, 1.0, 1.0)


def ragged_agentic(n_seqs: int = 16, lo: int = 8192, hi: int = 49152) -> Workload:
    """Config 5: 16 requests of independent lengths in one ragged launch, one layer, B_r = floor(0.08 N_r)."""
    lens = ragged_lengths(5, n_seqs, lo, hi)
    budgets = [int(np.floor(0.08 * n)) for n in lens]
    return _make("ragged_agentic", 5, 1, 28, 4, 128, lens, 64, budgets, 7, 1.0, 0.0, 0.0, (4, 12), 0.20, 0.0, 1.0)


def paper_chunks(n_chunks: int = 64, capacity: float = 0.5) -> Workload:
    """The compression setting of the paper's own experiments (appendix "Compression settings") on a 7B-shaped model:
    the context comes as chunks of 128 to 4096 tokens (file-level chunks aimed at 512 tokens: lengths
    512 * exp(0.7 z), z ~ N(0,1), clipped), every chunk is compressed on its own with a window of 128 tokens, average
    pooling of width 5 and a capacity of 0.4 to 0.6 (here B_r = max(W, floor(capacity * N_r))); structural spans of
    16 to 48 tokens (the paper's minimum span is 16), a quarter of them marked, binary prior."""
    g = _rng(6, _T_LENS)
    lens = np.clip(np.rint(512.0 * np.exp(0.7 * g.standard_normal(n_chunks))), 128, 4096).astype(np.int64)
    budgets = [max(128, int(np.floor(capacity * n))) for n in lens]
    return _make("paper_chunks", 6, 28, 28, 4, 128, [int(n) for n in lens], 128, budgets, 5, 1.0, 0.0, 0.0, (16, 48),
                 0.25, 1.0, 1.0)


CONFIGS = {
    "tiny": tiny,
    "qwen7b_32k": qwen7b_32k,
    "llama8b_64k": llama8b_64k,
    "long_128k": long_128k,
    "ragged_agentic": ragged_agentic,
    "paper_chunks": paper_chunks,
}


def scaled(w: Workload, *, name: Optional[str] = None, n_layers: Optional[int] = None,
           seqlens: Optional[Sequence[int]] = None, budgets: Optional[Sequence[int]] = None,
           **overrides) -> Workload:
    """A smaller (or otherwise altered) copy of a workload with the same recipe: used for parity cases."""
    kw = dict(overrides)
    if name is not None:
        kw["name"] = name
    if n_layers is not None:
        kw["n_layers"] = n_layers
    if seqlens is not None:
        kw["seqlens"] = tuple(int(x) for x in seqlens)
        if budgets is None:
            ratio = w.total_budget / w.total_tokens
            budgets = [max(w.window if "window" not in kw else kw["window"], int(np.floor(ratio * n))) for n in seqlens]
    if budgets is not None:
        kw["budgets"] = tuple(int(x) for x in budgets)
    return dataclasses.replace(w, **kw)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_fp8_codes(bits: np.ndarray) -> np.ndarray:
    """An FP8 (OCP E4M3) copy of a bf16 cache, as a serving stack that keeps its KV cache in 8 bits would hold
    it: every element rounded to the nearest E4M3 number by the library cast (magnitudes clamped to the
    format's largest finite value, 448, first).  Returns uint8 codes of the same shape."""
    import torch
    x = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(torch.float32)
    return x.clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def make_prior(w: Workload) -> np.ndarray:
    """Per-token prior: each request is cut into spans of uniform length in [span_min, span_max];
    a span is flagged with probability flag_rate; tokens of a flagged span get p (one draw per
    token when prior_lo < prior_hi, the constant prior_hi otherwise), all other tokens 0."""
    out = np.zeros(w.total_tokens, dtype=np.float32)
    cu = w.cu_seqlens()
    for r, n in enumerate(w.seqlens):
        g = _rng(w.cfg_id, _T_PRIOR, 0, r)
        max_spans = n // w.span_min + 1
        lens = g.integers(w.span_min, w.span_max + 1, size=max_spans)
        flags = g.random(max_spans) < w.flag_rate
        ends = np.cumsum(lens)
        n_sp = int(np.searchsorted(ends, n, side="left")) + 1      # last span truncated at n
        span_of_tok = np.repeat(np.arange(n_sp), lens[:n_sp])[:n]
        tok_flag = flags[span_of_tok]
        if w.prior_lo < w.prior_hi:
            vals = g.uniform(w.prior_lo, w.prior_hi, size=n).astype(np.float32)
        else:
            vals = np.full(n, w.prior_hi, dtype=np.float32)
        out[cu[r]:cu[r + 1]] = np.where(tok_flag, vals, np.float32(0))
    return out


def _normal_bits(g: np.random.Generator, shape, *, row_scale: Optional[np.ndarray] = None,
                 row_add: Optional[np.ndarray] = None, block_rows: int = 1 << 16) -> np.ndarray:
    """N(0,1) float32 -> optional per-row add/scale -> bf16 bits, generated in row blocks to bound memory.
    `shape` = (rows, d)."""
    rows, d = shape
    out = np.empty((rows, d), dtype=np.uint16)
    for r0 in range(0, rows, block_rows):
        r1 = min(rows, r0 + block_rows)
        x = g.standard_normal((r1 - r0, d), dtype=np.float32)
        if row_add is not None:
            x += row_add[r0:r1, None]
        if row_scale is not None:
            x *= row_scale[r0:r1, None]
        out[r0:r1] = f32_to_bf16_bits(x)
    return out


def make_layer(w: Workload, layer: int, *, with_v: bool = True):
    """Inputs of one layer: q_obs [n_seqs][H_q][W][d], k and v [H_kv][sum N][d], all bf16 bits."""
    d, T = w.head_dim, w.total_tokens
    q = _normal_bits(_rng(w.cfg_id, _T_Q, layer), (w.n_seqs * w.n_q_heads * w.window, d))
    q = q.reshape(w.n_seqs, w.n_q_heads, w.window, d)
    # per-row modifiers: positional drift (position is sequence-local), then heavy-hitter scaling
    pos = np.concatenate([np.arange(n, dtype=np.float32) for n in w.seqlens])
    add = None
    if w.drift_amp != 0.0:
        add = np.tile((w.drift_amp * np.sin(pos / np.float32(w.drift_period))).astype(np.float32), w.n_kv_heads)
    scale = None
    if w.heavy_rate > 0.0:
        heavy = _rng(w.cfg_id, _T_HEAVY, layer).random(w.n_kv_heads * T) < w.heavy_rate
        scale = np.where(heavy, np.float32(w.heavy_scale), np.float32(1)).astype(np.float32)
    k = _normal_bits(_rng(w.cfg_id, _T_K, layer), (w.n_kv_heads * T, d), row_scale=scale, row_add=add)
    k = k.reshape(w.n_kv_heads, T, d)
    v = None
    if with_v:
        v = _normal_bits(_rng(w.cfg_id, _T_V, layer), (w.n_kv_heads * T, d)).reshape(w.n_kv_heads, T, d)
    return q, k, v


def make_all(w: Workload, *, with_v: bool = True, threads: int = 8, layers: Optional[Sequence[int]] = None):
    """All layers stacked: q [L][n_seqs][H_q][W][d], k/v [L][H_kv][sum N][d], prior [sum N]."""
    layers = list(range(w.n_layers)) if layers is None else list(layers)
    nl, d, T = len(layers), w.head_dim, w.total_tokens
    q = np.empty((nl, w.n_seqs, w.n_q_heads, w.window, d), dtype=np.uint16)
    k = np.empty((nl, w.n_kv_heads, T, d), dtype=np.uint16)
    v = np.empty((nl, w.n_kv_heads, T, d), dtype=np.uint16) if with_v else None

    def fill(i):
        ql, kl, vl = make_layer(w, layers[i], with_v=with_v)
        q[i], k[i] = ql, kl
        if with_v:
            v[i] = vl

    with ThreadPoolExecutor(max_workers=max(1, min(threads, nl))) as ex:
        list(ex.map(fill, range(nl)))
    return q, k, v, make_prior(w)
