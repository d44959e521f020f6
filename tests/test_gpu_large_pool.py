"""GPU parity with K/V pools larger than 4 GiB each: a cache sized for this part's memory has pages whose byte
offset from the pool's start does not fit 32 bits, and every kernel forms page addresses as base + id * page
bytes (Sec. 3.1.1: the page table is the index array of a block-sparse matrix).  The cases are small batches
whose pages are scattered over such a pool, half of them at its very end; the oracle sees the same batch with its
pages packed."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import DeviceBatch, assert_close, run_gpu

pytestmark = pytest.mark.gpu

POOL_BYTES = 5 * 1024 ** 3  # per pool (K and V each)


class ScatteredPools:
    """The device tensors of `batch` with its pages moved into pools of POOL_BYTES: page j stays at j if j is even and
    goes to (pages of the large pool) - (pages of the batch) + j otherwise; the page table follows."""

    def __init__(self, batch):
        dev = DeviceBatch(batch)
        self.batch, self.device, self.q, self.scales = batch, dev.device, dev.q, dev.scales
        n_small = dev.k_pool.shape[0]
        page_bytes = dev.k_pool[0].numel() * dev.k_pool.element_size()
        n_big = -(-POOL_BYTES // page_bytes)
        ids = torch.arange(n_small, device=dev.device)
        new_id = torch.where(ids % 2 == 0, ids, n_big - n_small + ids)
        self.last_offset = int(new_id.max()) * page_bytes
        assert self.last_offset >= 2 ** 32
        pools = []
        for small in (dev.k_pool, dev.v_pool):
            big = torch.empty((n_big,) + tuple(small.shape[1:]), dtype=small.dtype, device=dev.device)
            big[new_id] = small
            pools.append(big)
        self.k_pool, self.v_pool = pools
        self.kv_indices = new_id[dev.kv_indices.long()].to(torch.int32)
        # (an empty batch has one placeholder id)
        if len(batch.kv_indices) == 0:
            self.kv_indices = dev.kv_indices


def check(batch, mode, what, **kw):
    print(f"[case] {what}: {batch.name} mode={mode} page_size={batch.page_size} dtype={batch.dtype} kv={batch.kv_dtype} "
          f"qo={batch.qo_lens()[:8].tolist()} kv_len={batch.kv_lens()[:8].tolist()} kw={kw}", flush=True)
    o_ref, lse_ref = oracle.run_batch(batch)
    dev = ScatteredPools(batch)
    o, lse = run_gpu(batch, mode, dev=dev, **kw)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: last page at byte {dev.last_offset}, err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    del dev
    torch.cuda.empty_cache()


@pytest.mark.parametrize("ps", [16, 1])
def test_decode(ps):
    for seed, dtype, kv_dtype in ((701, workloads.BF16, ""), (702, workloads.F16, ""), (703, workloads.BF16, workloads.FP8)):
        b = workloads.random_case(seed + ps, dtype=dtype, page_size=ps, batch=6, max_kv=700, kv_dtype=kv_dtype,
                                  k_scale=0.5 if kv_dtype else 1.0, v_scale=2.0 if kv_dtype else 1.0)
        check(b, "decode", f"decode ps={ps}")
    b = workloads.make_batch("long", 710 + ps, workloads.BF16, 32, 8, 128, ps, [1, 1, 1], [2500, 77, 600], False)
    check(b, "decode", f"decode split ps={ps}", num_ctas=8 * 16, min_chunk=64)


@pytest.mark.parametrize("ps", [16, 8, 1])
def test_append(ps):
    """page size 16: the scheduled loop and (short chunks) the general path; 8 and 1: the loop's variants for other
    page sizes"""
    for seed, dtype in ((721, workloads.BF16), (722, workloads.F16)):
        b = workloads.make_batch("appchain", seed + ps, dtype, 8, 2, 128, ps, [200, 64, 130, 9], [1500, 700, 131, 9], True)
        check(b, "append", f"append ps={ps}", num_ctas=2 * 3, min_chunk=128)
    b = workloads.make_batch("appsplit", 730 + ps, workloads.BF16, 8, 2, 128, ps, [64, 30], [1000, 777], True)
    check(b, "append", f"append split ps={ps}", num_ctas=2 * 16, min_chunk=128)


@pytest.mark.parametrize("mode", ["tile16", "tile64"])
def test_tiles(mode):
    b = workloads.make_batch("verify", 741, workloads.BF16, 32, 8, 128, 16, [4, 1, 16, 3, 7], [900, 300, 2000, 3, 64], True)
    check(b, mode, f"{mode}")


def test_variants():
    """the logits hooks run other instantiations of both kernels"""
    from test_gpu_variants import run_variant
    for mode, qo, kv in (("decode", [1, 1, 1], [900, 77, 2000]), ("append", [200, 64, 9], [1500, 700, 9])):
        b = workloads.make_batch("var", 751, workloads.BF16, 8, 2, 128, 16, qo, kv, True)
        var = dict(logits_soft_cap=30.0, window_left=300)
        print(f"[case] variants: {b.name} mode={mode} qo={qo} kv={kv} {var}", flush=True)
        o_ref, lse_ref = oracle.run_batch(b, **var)
        dev = ScatteredPools(b)
        o, lse = run_variant(b, mode=mode, dev=dev, **var)
        e = assert_close(o, lse, o_ref, lse_ref, f"variants {mode}")
        print(f"[ok] variants {mode}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
        del dev
        torch.cuda.empty_cache()
