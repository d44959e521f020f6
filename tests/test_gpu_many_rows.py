"""GPU parity with more than 2^32 bytes of output: `o[nnz_qo, H_qo, D]` in fp32 passes 4 GiB at 262 144 query
positions (H_qo = 32, D = 128), so row offsets in bytes need 64 bits in every kernel, and the append kernel's
scheduled loop, which addresses its outputs with 32-bit byte offsets, has to hand the rows beyond that to the
general path (Sec. 3.2.2: the output of a tile is written at the tile's rows of the ragged tensor).

The batch is a small batch repeated R times: repetition r has the small batch's lengths and page table and, as its
queries, a copy of the small batch's queries, so its rows must equal the oracle's rows of the small batch.  Every
output row is compared."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import DeviceBatch, LSE_TOL, O_TOL, make_wrapper

pytestmark = pytest.mark.gpu

ROWS_4GIB = 2 ** 32 // (32 * 128 * 4)  # query positions whose fp32 rows fill 4 GiB


def run_repeated(small, mode, reps, **kw):
    nq, npg = int(small.qo_indptr[-1]), int(small.kv_indptr[-1])
    assert nq * reps > ROWS_4GIB
    print(f"[case] {small.name} x {reps} mode={mode}: {small.batch * reps} requests, {nq * reps} query positions, "
          f"qo={small.qo_lens()[:6].tolist()} kv={small.kv_lens()[:6].tolist()}", flush=True)
    o_ref, lse_ref = oracle.run_batch(small)
    big = dataclasses.replace(
        small,
        qo_indptr=np.concatenate([[0]] + [small.qo_indptr[1:].astype(np.int64) + r * nq for r in range(reps)]).astype(np.int32),
        kv_indptr=np.concatenate([[0]] + [small.kv_indptr[1:].astype(np.int64) + r * npg for r in range(reps)]).astype(np.int32),
        kv_indices=np.tile(small.kv_indices, reps), last_page_len=np.tile(small.last_page_len, reps))
    dev = DeviceBatch(small)
    q = dev.q.repeat(reps, 1, 1)
    kv_indices = dev.kv_indices[:npg].repeat(reps)
    w = make_wrapper(big, mode, **kw)
    w.plan(big.qo_indptr, big.kv_indptr, big.last_page_len, causal=big.causal)
    H, D = small.num_qo_heads, small.head_dim
    o = torch.full((nq * reps, H, D), float("nan"), dtype=torch.float32, device=dev.device)
    lse = torch.full((nq * reps, H), float("nan"), dtype=torch.float32, device=dev.device)
    assert o.numel() * 4 > 2 ** 32
    w.run(q, dev.k_pool, dev.v_pool, kv_indices, small.sm_scale, o=o, lse=lse)
    torch.cuda.synchronize()
    w.close()
    ref_o = torch.from_numpy(o_ref).to(dev.device)      # float64
    ref_l = torch.from_numpy(lse_ref).to(dev.device)
    err_o = err_l = 0.0
    o, lse = o.view(reps, nq, H, D), lse.view(reps, nq, H)
    for r0 in range(0, reps, 64):
        err_o = max(err_o, float((o[r0:r0 + 64].double() - ref_o).abs().nan_to_num(nan=float("inf")).max()))
        err_l = max(err_l, float((lse[r0:r0 + 64].double() - ref_l).abs().nan_to_num(nan=float("inf")).max()))
    print(f"[ok] {small.name} x {reps} mode={mode}: err_o={err_o:.2e} err_lse={err_l:.2e}", flush=True)
    assert err_o <= O_TOL and err_l <= LSE_TOL, (err_o, err_l)


def test_decode():
    g = np.random.Generator(np.random.PCG64(801))
    small = workloads.make_batch("dec64", 801, workloads.BF16, 32, 8, 128, 16, [1] * 64, g.integers(1, 300, size=64), False,
                                 poison=False)
    run_repeated(small, "decode", ROWS_4GIB // 64 + 100)


def test_append():
    """chunks of at least 128 tokens run the scheduled loop while their rows' byte offsets fit 32 bits and the
    general path after that; shorter ones the general path"""
    g = np.random.Generator(np.random.PCG64(802))
    qo = np.full(42, 64)
    small = workloads.make_batch("app42", 802, workloads.BF16, 32, 8, 128, 16, qo, qo + g.integers(0, 260, size=42), True,
                                 poison=False)
    run_repeated(small, "append", ROWS_4GIB // (42 * 64) + 4)


@pytest.mark.parametrize("mode", ["tile16", "tile64"])
def test_tiles(mode):
    g = np.random.Generator(np.random.PCG64(803))
    qo = np.full(64, 4)
    small = workloads.make_batch("ver64", 803, workloads.BF16, 32, 8, 128, 16, qo, qo + g.integers(0, 300, size=64), True,
                                 poison=False)
    run_repeated(small, mode, ROWS_4GIB // 256 + 30, max_formats=1)  # (partial states per CTA, not per work item: 18 GB less)
