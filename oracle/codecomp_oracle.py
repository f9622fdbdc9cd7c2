"""CPU oracle for the prefill KV-eviction path of CodeComp: score -> select -> gather.

TEST INFRASTRUCTURE ONLY.  This is the plain fp64 definition of what the HIP path must
compute, written straight from the paper's equations, with no blocking, fusion or
reordering.  It shares no code with the HIP path and must never be imported by it; only
tests, the smoke check and the benchmark's CPU-baseline leg may call it.

What it follows (paper sections / equations):

  * Section "Attention-based KV Cache Compression", its only equation
        A = softmax(Q K^T / sqrt(d)),   u(j) = sum_{t=1..W} A(t, j)
    with Q the W observation-window queries and K the cached keys; the softmax of one
    query row runs over every cached key (the equation carries no mask).
  * Appendix "Compression settings": the attention scores are average-pooled over a
    sliding window (size 5 in the paper; the width is a parameter here).
  * Sections "Span-Level Structural Protection" / "Attention-based KV Cache Compression":
    structure decides what must be kept and attention fills the remaining capacity.  The
    paper states this as a two-stage rule and gives no formula that mixes a dense per-token
    prior with the attention mass.  The reading used throughout this repository is
        c(j) = pooled_u(j) + lambda * p(j)
    followed by ONE top-(B - W) over the prefix [0, N - W); its lambda -> infinity limit
    with a binary prior is the paper's "protected tokens first, attention fills the rest".
    PARITY UNPINNED BY THE PAPER for this combination rule: no worked example or printed
    number distinguishes the additive reading from the two-stage rule.  It is pinned only
    by closed forms (lambda = 0, lambda large) and brute force.
  * The same section keeps the best-scored context tokens until the chunk's remaining budget is
    used up, and compresses every transformer layer on its own: selection is per
    layer (and here per KV head), and the compact cache holds the retained K/V rows in
    their original order.

Readings where the paper is silent (all listed again in the design notes of this repo):
  - grouped-query attention: the G query heads sharing one KV head are averaged (mean);
  - pooling: stride 1, same length, zero padding, divisor always k, over the whole row;
  - the last W tokens (the observation window itself) are always kept and count towards B;
  - ties between equal scores go to the lower token index;
  - kept indices are emitted in ascending order.

Variants of the score tail (other readings of what the paper leaves open, switchable; the
defaults are the readings above):
  - group_reduce "sum" / "max": the G query heads of a KV head are summed / the largest head
    mass wins, instead of averaged;
  - pool_mode "max": max pooling instead of the appendix's average pooling;
  - softmax_domain "prefix": the softmax of section "Attention-based KV Cache Compression"
    runs over the context keys only (the section gives K one row per context token), i.e. the N - W keys before the
    observation window; window columns get no mass;
  - pool_domain "prefix": pooling never looks across the boundary between context and window.

Storage variant (not from the paper, which scores a bf16 cache): k_format "fp8_e4m3" takes the cached
keys (and values) as 8-bit floating point codes, OCP E4M3 (1 sign, 4 exponent bits with bias 7, 3
mantissa bits, no infinities, S.1111.111 = NaN).  A code stands for exactly the real number it encodes;
the equations above are applied to those numbers.  A per-tensor dequantisation factor belongs in `scale`.

All arrays are numpy.  bf16 inputs arrive as uint16 bit patterns and are widened exactly.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def fp8_e4m3_to_f64(codes: np.ndarray) -> np.ndarray:
    """Exact value of OCP FP8 E4M3 codes (uint8): (-1)^s * 2^(e-7) * (1 + m/8) for exponent field
    e in 1..15, (-1)^s * 2^-6 * (m/8) for e = 0 (subnormals and zero); e = 15 with m = 7 is NaN."""
    c = np.ascontiguousarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 0x7).astype(np.float64)
    normal = np.ldexp(1.0 + m / 8.0, e - 7)
    subnormal = np.ldexp(m / 8.0, -6)
    mag = np.where(e == 0, subnormal, normal)
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return sign * mag


def keys_to_f64(k, k_format: str = "bf16") -> np.ndarray:
    """Cached keys as stored ("bf16": uint16 patterns, "fp8_e4m3": uint8 codes) -> the numbers they hold."""
    assert k_format in ("bf16", "fp8_e4m3")
    return bf16_bits_to_f64(k) if k_format == "bf16" else fp8_e4m3_to_f64(k)


# ----------------------------------------------------------------------------------------
# score
# ----------------------------------------------------------------------------------------

def attention_rows(q: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """A = softmax(q k^T * scale) for one query head: q [W, d], k [N, d] -> A [W, N].
    (The equation of section "Attention-based KV Cache Compression"; rows sum to 1.)"""
    s = (q @ k.T) * scale
    s = s - s.max(axis=1, keepdims=True)          # stabiliser: leaves the softmax unchanged
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def window_attention_mass(q_obs: np.ndarray, k: np.ndarray, scale: float | None = None, *,
                          group_reduce: str = "mean", softmax_keys: int | None = None) -> np.ndarray:
    """u[h, j] = reduce_{g<G} sum_{t<W} A[h*G+g][t, j], reduce = mean (default), sum or max.

    q_obs float64 [H_q, W, d]; k float64 [H_kv, N, d]; returns float64 [H_kv, N].
    Query head h_q reads KV head h_q // G (contiguous grouping).  softmax_keys = m restricts
    every softmax to the first m keys; the other columns get zero mass."""
    h_q, w, d = q_obs.shape
    h_kv, n, d2 = k.shape
    assert d == d2 and h_q % h_kv == 0 and group_reduce in ("mean", "sum", "max")
    g = h_q // h_kv
    m = n if softmax_keys is None else int(softmax_keys)
    assert 0 <= m <= n
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    per_head = np.zeros((h_q, n), dtype=np.float64)
    if m > 0:
        for hq in range(h_q):
            a = attention_rows(q_obs[hq], k[hq // g, :m], scale)
            per_head[hq, :m] = a.sum(axis=0)      # u(j) = sum_t A(t, j)
    grouped = per_head.reshape(h_kv, g, n)
    if group_reduce == "max":
        return grouped.max(axis=1)
    u = grouped.sum(axis=1)
    return u / g if group_reduce == "mean" else u


def average_pool(u: np.ndarray, kernel: int, extent: int | None = None) -> np.ndarray:
    """pooled[j] = (1/k) sum_{|delta| <= (k-1)/2} u[j + delta], terms outside [0, E) are zero.
    Works on the last axis.  E = extent (default: the whole axis); positions >= E get 0."""
    assert kernel >= 1 and kernel % 2 == 1
    half = (kernel - 1) // 2
    n = u.shape[-1] if extent is None else int(extent)
    out = np.zeros_like(u, dtype=np.float64)
    for delta in range(-half, half + 1):
        lo, hi = max(0, -delta), min(n, n - delta)        # j with 0 <= j + delta < n
        if hi > lo:
            out[..., lo:hi] += u[..., lo + delta:hi + delta]
    return out / kernel


def max_pool(u: np.ndarray, kernel: int, extent: int | None = None) -> np.ndarray:
    """pooled[j] = max_{|delta| <= (k-1)/2, 0 <= j + delta < E} u[j + delta]; positions >= E get 0."""
    assert kernel >= 1 and kernel % 2 == 1
    half = (kernel - 1) // 2
    n = u.shape[-1] if extent is None else int(extent)
    out = np.zeros_like(u, dtype=np.float64)
    for j in range(n):
        out[..., j] = u[..., max(0, j - half):min(n, j + half + 1)].max(axis=-1)
    return out


def fuse_prior(pooled: np.ndarray, prior: np.ndarray, prior_weight: float) -> np.ndarray:
    """c[h, j] = pooled[h, j] + lambda * p[j]; the prior is shared by all heads."""
    return pooled + float(prior_weight) * np.asarray(prior, dtype=np.float64)[None, :]


def score(q_obs: np.ndarray, k: np.ndarray, prior: np.ndarray, *, pool_kernel: int,
          prior_weight: float, scale: float | None = None, group_reduce: str = "mean",
          pool_mode: str = "avg", softmax_domain: str = "all", pool_domain: str = "row") -> np.ndarray:
    """Scores of one request in one layer: float64 [H_kv, N].  The observation window is the
    last W = q_obs.shape[1] tokens; "prefix" domains are the N - W tokens before it."""
    assert pool_mode in ("avg", "max") and softmax_domain in ("all", "prefix") and pool_domain in ("row", "prefix")
    n, w = k.shape[1], q_obs.shape[1]
    u = window_attention_mass(q_obs, k, scale, group_reduce=group_reduce,
                              softmax_keys=n - w if softmax_domain == "prefix" else None)
    extent = n - w if pool_domain == "prefix" else None
    pooled = average_pool(u, pool_kernel, extent) if pool_mode == "avg" else max_pool(u, pool_kernel, extent)
    return fuse_prior(pooled, prior, prior_weight)


# ----------------------------------------------------------------------------------------
# select
# ----------------------------------------------------------------------------------------

def select(scores: np.ndarray, window: int, budget: int) -> np.ndarray:
    """Kept token indices per head: int64 [H, budget], ascending.

    The last `window` tokens are always kept.  The other budget - window come from the
    prefix [0, N - window): rank it by (score descending, index ascending) and take the
    head of that ranking."""
    h, n = scores.shape
    assert 1 <= window <= n and window <= budget <= n
    take = budget - window
    out = np.empty((h, budget), dtype=np.int64)
    tail = np.arange(n - window, n, dtype=np.int64)
    for i in range(h):
        prefix = scores[i, : n - window]
        order = np.argsort(-prefix, kind="stable")        # stable: equal scores keep index order
        out[i] = np.concatenate([np.sort(order[:take]), tail])
    return out


# ----------------------------------------------------------------------------------------
# gather
# ----------------------------------------------------------------------------------------

def gather(k: np.ndarray, v: np.ndarray, idx: np.ndarray):
    """k_out[h, i, :] = k[h, idx[h, i], :], same for v (a copy of rows; any dtype)."""
    h = k.shape[0]
    k_out = np.stack([k[i][idx[i]] for i in range(h)])
    v_out = np.stack([v[i][idx[i]] for i in range(h)])
    return k_out, v_out


# ----------------------------------------------------------------------------------------
# whole path: layers x requests (packed / ragged)
# ----------------------------------------------------------------------------------------

def score_packed(q_bits, k_bits, prior, cu_seqlens, *, pool_kernel, prior_weight, scale=None,
                 layers=None, k_format="bf16", **variant) -> np.ndarray:
    """q_bits uint16 [L][n_seqs][H_q][W][d], k_bits [L][H_kv][T][d] (uint16 bf16 patterns, or uint8
    codes with k_format "fp8_e4m3"), prior [T], cu_seqlens [n_seqs+1] -> scores float64 [L][H_kv][T].
    Every (layer, request) is scored on its own; layers not listed in `layers` are left as NaN."""
    n_layers, h_kv, total, _ = k_bits.shape
    out = np.full((n_layers, h_kv, total), np.nan, dtype=np.float64)
    for l in (range(n_layers) if layers is None else layers):
        for r in range(len(cu_seqlens) - 1):
            a, b = int(cu_seqlens[r]), int(cu_seqlens[r + 1])
            out[l, :, a:b] = score(bf16_bits_to_f64(q_bits[l, r]), keys_to_f64(k_bits[l, :, a:b], k_format),
                                   prior[a:b], pool_kernel=pool_kernel, prior_weight=prior_weight, scale=scale,
                                   **variant)
    return out


def select_packed(scores, cu_seqlens, cu_budgets, window) -> np.ndarray:
    """scores [L][H][T] -> idx int64 [L][H][sum B_r]; indices are local to their request."""
    n_layers, h, _ = scores.shape
    out = np.empty((n_layers, h, int(cu_budgets[-1])), dtype=np.int64)
    for l in range(n_layers):
        for r in range(len(cu_seqlens) - 1):
            a, b = int(cu_seqlens[r]), int(cu_seqlens[r + 1])
            oa, ob = int(cu_budgets[r]), int(cu_budgets[r + 1])
            out[l, :, oa:ob] = select(scores[l, :, a:b], window, ob - oa)
    return out


def gather_packed(k, v, idx, cu_seqlens, cu_budgets):
    """k, v [L][H][T][d] (any dtype), idx [L][H][sum B_r] request-local -> compact [L][H][sum B_r][d]."""
    n_layers, h, _, d = k.shape
    k_out = np.empty((n_layers, h, int(cu_budgets[-1]), d), dtype=k.dtype)
    v_out = np.empty_like(k_out, dtype=v.dtype)
    for l in range(n_layers):
        for r in range(len(cu_seqlens) - 1):
            a, b = int(cu_seqlens[r]), int(cu_seqlens[r + 1])
            oa, ob = int(cu_budgets[r]), int(cu_budgets[r + 1])
            k_out[l, :, oa:ob], v_out[l, :, oa:ob] = gather(k[l, :, a:b], v[l, :, a:b], idx[l, :, oa:ob])
    return k_out, v_out


def compress_packed(q_bits, k_bits, v_bits, prior, cu_seqlens, cu_budgets, *, window, pool_kernel,
                    prior_weight, scale=None, k_format="bf16"):
    """The whole path.  Returns (scores, idx, k_out, v_out)."""
    sc = score_packed(q_bits, k_bits, prior, cu_seqlens, pool_kernel=pool_kernel,
                      prior_weight=prior_weight, scale=scale, k_format=k_format)
    idx = select_packed(sc, cu_seqlens, cu_budgets, window)
    k_out, v_out = gather_packed(k_bits, v_bits, idx, cu_seqlens, cu_budgets)
    return sc, idx, k_out, v_out


# ----------------------------------------------------------------------------------------
# structure-aware budgets (host-side arithmetic of section "Structure-Aware Budget Allocation")
# ----------------------------------------------------------------------------------------

def log_norm(x, tau):
    """Norm(x; tau) = min(1, log(1 + x) / log(1 + tau))  (section "Structural Feature Extraction")."""
    return np.minimum(1.0, np.log1p(np.asarray(x, dtype=np.float64)) / np.log1p(np.asarray(tau, dtype=np.float64)))


def chunk_structure_score(features, tau, weights):
    """sigma_i = sum_k w_k * Norm(f_ik; tau_k); features [n_chunks, K]."""
    return (log_norm(features, tau) * np.asarray(weights, dtype=np.float64)).sum(axis=1)


def chunk_budgets(sigma, chunk_len, *, ratio, m_min, m_max, r_max, eps):
    """B_i = floor(|C_i| * min(r_max, r * m_i)) with
    s_i = 0.5 if all sigma are equal else (sigma_i - sigma_min) / max(eps, sigma_max - sigma_min),
    m_i = m_min + (m_max - m_min) * clip(s_i, 0, 1)."""
    sigma = np.asarray(sigma, dtype=np.float64)
    lo, hi = sigma.min(), sigma.max()
    if hi == lo:
        s = np.full_like(sigma, 0.5)
    else:
        s = (sigma - lo) / max(eps, hi - lo)
    m = m_min + (m_max - m_min) * np.clip(s, 0.0, 1.0)
    return np.floor(np.asarray(chunk_len, dtype=np.float64) * np.minimum(r_max, ratio * m)).astype(np.int64)


# ----------------------------------------------------------------------------------------
# structure score: fraction of structurally critical tokens that survive compression
# ----------------------------------------------------------------------------------------

def structure_score(idx, prior, n):
    """Per head: |{kept j : p[j] > 0}| / |{j < n : p[j] > 0}| (section "Experiment", Str. Score; the
    structurally critical tokens are those the prior marks).  idx [H, B]; NaN when nothing is marked."""
    flagged = np.asarray(prior[:n]) > 0
    total = int(flagged.sum())
    out = np.full(idx.shape[0], np.nan)
    if total:
        for h in range(idx.shape[0]):
            out[h] = flagged[idx[h]].sum() / total
    return out


# ----------------------------------------------------------------------------------------
# the paper's literal order: structure first, attention fills the rest
# ----------------------------------------------------------------------------------------

def span_budget(prefix_budget: int, ratio: float, minimum: int) -> int:
    """B_span = min(B, max(B_min, floor(rho_span * B)))  (section "Span-Level Structural Protection")."""
    return int(min(prefix_budget, max(minimum, np.floor(ratio * prefix_budget))))


def select_two_stage(pooled: np.ndarray, prior: np.ndarray, window: int, budget: int, *, span_ratio: float,
                     span_min: int) -> np.ndarray:
    """Kept indices per head, int64 [H, budget], ascending.

    Token-level form of the two-stage rule on a dense prior: the last `window` tokens are always
    kept; of the Bp = budget - window prefix slots, stage 1 gives up to B_span to tokens the prior
    marks (p > 0), largest p first, equal p first in sequence; stage 2 gives the remaining slots to
    the other prefix tokens by pooled attention mass (descending, equal mass first in sequence)."""
    h, n = pooled.shape
    assert 1 <= window <= n and window <= budget <= n
    npre, bp = n - window, budget - window
    p = np.asarray(prior[:npre], dtype=np.float64)
    marked = np.flatnonzero(p > 0)
    by_prior = marked[np.argsort(-p[marked], kind="stable")]
    protected = by_prior[: min(span_budget(bp, span_ratio, span_min), len(marked))]
    is_protected = np.zeros(npre, dtype=bool)
    is_protected[protected] = True
    others = np.flatnonzero(~is_protected)
    tail = np.arange(npre, n, dtype=np.int64)
    out = np.empty((h, budget), dtype=np.int64)
    for i in range(h):
        fill = others[np.argsort(-pooled[i, others], kind="stable")][: bp - len(protected)]
        out[i] = np.concatenate([np.sort(np.concatenate([protected, fill])), tail])
    return out
