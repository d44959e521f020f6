"""CPU oracle for attention over a paged (block-sparse-row) KV cache.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 NumPy; written from the paper's
definitions; shares no code with the GPU library and must never be imported
by it.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
use it.

What it computes, for request i, query head h (kv head h // g), query token j:

  * gather (Sec. 3.1.1, BSR KV-cache): row t of the request's keys is
    k_pool[kv_indices[kv_indptr[i] + t // page_size], h // g, t % page_size, :]
    for t < l_kv(i) = (n_pages - 1) * page_size + last_page_len(i);
  * attention state (Sec. 2.2, the LSE and O equations):
        lse = log sum_{t in I} exp(sm_scale * <q, k_t>)
        o   = sum_{t in I} exp(sm_scale * <q, k_t> - lse) * v_t
    with I = all tokens, or with causal masking (Sec. 4.2) the tokens
    t <= l_kv - l_qo + j (the appended tokens are already in the cache, so
    query j sits at absolute position l_kv - l_qo + j);
  * merge (Sec. 2.2, the (+) operator on attention states).

Readings where the paper is silent: the softmax scale is an explicit argument
and lse is the natural log of the scaled logits; an empty index set gives
o = 0, lse = -inf, which is the identity of (+).

Pins (tests/test_oracle_*.py): brute-force triple loops on tiny inputs, the
single-key / identical-keys / zero-query closed forms, split-merge equality,
page-permutation invariance, causal == lower-triangular mask, GQA == MHA with
repeated heads, composable == concatenated.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def request_kv_len(kv_indptr, last_page_len, page_size: int, i: int) -> int:
    n_pg = int(kv_indptr[i + 1]) - int(kv_indptr[i])
    return 0 if n_pg == 0 else (n_pg - 1) * page_size + int(last_page_len[i])


def gather_rows(pool_f64_of, kv_indices, kv_indptr, last_page_len, page_size: int,
                i: int, kv_head: int) -> np.ndarray:
    """Dense [l_kv, D] float64 rows of request i for one kv head.

    pool_f64_of(page_ids, kv_head) -> float64 [len(page_ids), page_size, D]
    (a callable so that huge pools are widened only where they are read)."""
    l_kv = request_kv_len(kv_indptr, last_page_len, page_size, i)
    pages = np.asarray(kv_indices[int(kv_indptr[i]):int(kv_indptr[i + 1])], dtype=np.int64)
    if l_kv == 0:
        d = pool_f64_of(np.zeros(0, dtype=np.int64), kv_head).shape[-1]
        return np.zeros((0, d), dtype=np.float64)
    blk = pool_f64_of(pages, kv_head)                  # [n_pg, page_size, D]
    return blk.reshape(-1, blk.shape[-1])[:l_kv]


def attention_state(q: np.ndarray, K: np.ndarray, V: np.ndarray, sm_scale: float,
                    visible: np.ndarray | None = None, logits_soft_cap: float = 0.0,
                    bias: np.ndarray | None = None) -> Tuple[np.ndarray, np.ndarray]:
    """Attention states of m queries against n keys.

    q [m, D], K [n, D], V [n, D] float64; visible: optional bool [m, n].
    Returns o [m, D], lse [m].  Rows with no visible key: o = 0, lse = -inf.
    Variants of Sec. 3.2.3 (logits transform / mask): with logits_soft_cap = c > 0 the scaled logits
    become c * tanh(s / c); `bias` [m, n] is added after that (ALiBi); a window is part of `visible`."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    m, n = q.shape[0], K.shape[0]
    s = sm_scale * (q @ K.T)                            # [m, n]
    if logits_soft_cap > 0.0:
        s = logits_soft_cap * np.tanh(s / logits_soft_cap)
    if bias is not None:
        s = s + bias
    if visible is not None:
        s = np.where(visible, s, -np.inf)
    o = np.zeros((m, V.shape[1] if V.ndim == 2 else q.shape[1]), dtype=np.float64)
    lse = np.full(m, -np.inf, dtype=np.float64)
    if n == 0:
        return o, lse
    mx = s.max(axis=1)
    live = np.isfinite(mx)
    if live.any():
        e = np.exp(s[live] - mx[live, None])            # masked entries -> exp(-inf) = 0
        z = e.sum(axis=1)
        lse[live] = mx[live] + np.log(z)
        o[live] = (e / z[:, None]) @ V
    return o, lse


def causal_visible(l_qo: int, l_kv: int) -> np.ndarray:
    """visible[j, t] = t <= l_kv - l_qo + j."""
    j = np.arange(l_qo)[:, None]
    t = np.arange(l_kv)[None, :]
    return t <= (l_kv - l_qo + j)


def variant_mask_and_bias(l_qo: int, l_kv: int, causal: bool, window_left: int = -1,
                          alibi_slope: float | None = None):
    """Visibility and additive bias of one (request, head) under the variants: query j sits at absolute
    position pos = l_kv - l_qo + j (the appended tokens are already in the cache); a window of
    `window_left` >= 0 hides tokens t < pos - window_left; ALiBi adds slope * (t - pos)."""
    j = np.arange(l_qo)[:, None]
    t = np.arange(l_kv)[None, :]
    pos = l_kv - l_qo + j
    vis = (t <= pos) if causal else np.ones((l_qo, l_kv), dtype=bool)
    if window_left >= 0:
        vis = vis & (t >= pos - window_left)
    bias = None if alibi_slope is None else alibi_slope * (t - pos).astype(np.float64)
    return vis, bias


def rope(x: np.ndarray, pos: np.ndarray, theta: float, scale: float = 1.0) -> np.ndarray:
    """Rotary position embedding as a query / key transform (Sec. 3.2.3; the fused-RoPE kernels of Sec. 4.3):
    x [n, D] at positions pos [n].  Component pair (d, d + D/2), d < D/2, is rotated by the angle
    (pos / scale) * theta ** (-2 d / D) (the "rotate half" pairing; the paper does not fix the pairing)."""
    n, D = x.shape
    half = D // 2
    assert 2 * half == D
    freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / D)
    ang = (np.asarray(pos, dtype=np.float64)[:, None] / scale) * freq[None, :]
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[:, :half], x[:, half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=1)


def batch_attention(q_f64: np.ndarray, k_pool_of, v_pool_of, qo_indptr, kv_indptr, kv_indices,
                    last_page_len, page_size: int, num_kv_heads: int, sm_scale: float,
                    causal: bool, requests: Sequence[int] | None = None,
                    heads: Sequence[int] | None = None, logits_soft_cap: float = 0.0,
                    window_left: int = -1, alibi_slopes=None, rope_theta: float = 0.0,
                    rope_scale: float = 1.0) -> Tuple[np.ndarray, np.ndarray]:
    """o [nnz_qo, H_qo, D], lse [nnz_qo, H_qo] (float64).

    Entries for requests / heads outside the optional selections are NaN.  The last arguments are the
    attention variants (soft cap of the logits, sliding window, per-head ALiBi slopes; rope_theta > 0: queries
    and keys are rotated by their positions first: key t of a request at position t, query j at
    l_kv - l_qo + j)."""
    nnz, H, D = q_f64.shape
    g = H // num_kv_heads
    assert g * num_kv_heads == H
    B = len(last_page_len)
    o = np.full((nnz, H, D), np.nan, dtype=np.float64)
    lse = np.full((nnz, H), np.nan, dtype=np.float64)
    req_list = range(B) if requests is None else requests
    head_list = range(H) if heads is None else heads
    for i in req_list:
        r0, r1 = int(qo_indptr[i]), int(qo_indptr[i + 1])
        l_qo = r1 - r0
        if l_qo == 0:
            continue
        l_kv = request_kv_len(kv_indptr, last_page_len, page_size, i)
        vis = causal_visible(l_qo, l_kv) if causal else None
        cache = {}
        for h in head_list:
            kvh = h // g
            if kvh not in cache:
                cache = {kvh: (gather_rows(k_pool_of, kv_indices, kv_indptr, last_page_len, page_size, i, kvh),
                               gather_rows(v_pool_of, kv_indices, kv_indptr, last_page_len, page_size, i, kvh))}
            K, V = cache[kvh]
            qh = q_f64[r0:r1, h, :]
            if rope_theta > 0.0:
                K = rope(K, np.arange(l_kv), rope_theta, rope_scale)
                qh = rope(qh, l_kv - l_qo + np.arange(l_qo), rope_theta, rope_scale)
            bias = None
            vis_h = vis
            if window_left >= 0 or alibi_slopes is not None:
                vis_h, bias = variant_mask_and_bias(l_qo, l_kv, causal, window_left,
                                                    None if alibi_slopes is None else float(alibi_slopes[h]))
            oo, ll = attention_state(qh, K, V, sm_scale, vis_h, logits_soft_cap, bias)
            o[r0:r1, h, :] = oo
            lse[r0:r1, h] = ll
    return o, lse


def merge_pair(o_a: np.ndarray, lse_a: np.ndarray, o_b: np.ndarray, lse_b: np.ndarray
               ) -> Tuple[np.ndarray, np.ndarray]:
    """(o, lse)_a (+) (o, lse)_b elementwise over leading dims; o [..., D], lse [...]."""
    o_a = np.asarray(o_a, dtype=np.float64)
    o_b = np.asarray(o_b, dtype=np.float64)
    lse_a = np.asarray(lse_a, dtype=np.float64)
    lse_b = np.asarray(lse_b, dtype=np.float64)
    m = np.maximum(lse_a, lse_b)
    both_empty = np.isneginf(m)
    m_safe = np.where(both_empty, 0.0, m)
    w_a = np.exp(lse_a - m_safe)
    w_b = np.exp(lse_b - m_safe)
    den = w_a + w_b
    den_safe = np.where(both_empty, 1.0, den)
    o = (w_a[..., None] * o_a + w_b[..., None] * o_b) / den_safe[..., None]
    o = np.where(both_empty[..., None], 0.0, o)
    lse = np.where(both_empty, -np.inf, m_safe + np.log(den_safe))
    return o, lse


def merge_states(o_parts: np.ndarray, lse_parts: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Left fold of (+) over axis 1: o_parts [n_rows, n_states, D], lse_parts [n_rows, n_states]."""
    o_parts = np.asarray(o_parts, dtype=np.float64)
    lse_parts = np.asarray(lse_parts, dtype=np.float64)
    n_rows, n_states, D = o_parts.shape
    o = np.zeros((n_rows, D), dtype=np.float64)
    lse = np.full(n_rows, -np.inf, dtype=np.float64)
    for s in range(n_states):
        o, lse = merge_pair(o, lse, o_parts[:, s, :], lse_parts[:, s])
    return o, lse
