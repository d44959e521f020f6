"""CPU oracle package: TEST INFRASTRUCTURE ONLY.

`attention` holds the fp64 definition of paged attention states and their
merge; `fp8` the decoding of the 8-bit KV cache format; `plan_replica` the step-by-step replica of the paper's scheduling
algorithm.  Nothing in the GPU library imports this package; only tests, the
smoke check and the benchmark's CPU-baseline leg do.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np

from . import attention, fp8, plan_replica  # noqa: F401


def run_batch(batch, requests: Sequence[int] | None = None,
              heads: Sequence[int] | None = None, logits_soft_cap: float = 0.0, window_left: int = -1,
              alibi_slopes=None, rope_theta: float = 0.0, rope_scale: float = 1.0) -> Tuple[np.ndarray, np.ndarray]:
    """Oracle (o, lse) of a `workloads.PagedBatch` (exact widening of the stored
    16-bit inputs to float64, then `attention.batch_attention`)."""
    from workloads import widen

    dt = batch.dtype
    q = widen(batch.q_bits, dt)

    if getattr(batch, "kv_dtype", "") == "fp8_e4m3":   # 8-bit KV cache (App. F): value = decoded code * scale
        def k_of(pages, h):
            return fp8.e4m3_to_f64(batch.k_bits[pages, h]) * batch.k_scale

        def v_of(pages, h):
            return fp8.e4m3_to_f64(batch.v_bits[pages, h]) * batch.v_scale
    else:
        def k_of(pages, h):
            return widen(batch.k_bits[pages, h], dt)

        def v_of(pages, h):
            return widen(batch.v_bits[pages, h], dt)

    return attention.batch_attention(
        q, k_of, v_of, batch.qo_indptr, batch.kv_indptr, batch.kv_indices, batch.last_page_len,
        batch.page_size, batch.num_kv_heads, batch.sm_scale, batch.causal,
        requests=requests, heads=heads, logits_soft_cap=logits_soft_cap, window_left=window_left,
        alibi_slopes=alibi_slopes, rope_theta=rope_theta, rope_scale=rope_scale)
