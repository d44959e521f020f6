"""GPU parity of decode over an 8-bit KV cache (App. F: fp8 K/V, 16-bit queries, fp32 accumulation)
against the oracle, which decodes the same E4M3 codes: every code value, both query types, the
GQA group sizes, ragged tails, empty requests, split chunks with merge, the strided pool layout,
and the small variants of the two decode workloads."""
import dataclasses

import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, O_TOL, assert_close, run_gpu
from oracle.fp8 import e4m3_to_f64

pytestmark = pytest.mark.gpu
FP8 = workloads.FP8


def check(batch, what, dev=None, **kw):
    print(f"[case] {what}: {batch.name} dtype={batch.dtype} kv={batch.kv_dtype} heads={batch.num_qo_heads}/"
          f"{batch.num_kv_heads} kv_len={batch.kv_lens()[:10].tolist()} scales=({batch.k_scale}, {batch.v_scale}) kw={kw}",
          flush=True)
    o_ref, lse_ref = oracle.run_batch(batch)
    o, lse = run_gpu(batch, "decode", dev=dev, **kw)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    return o, lse


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
def test_every_code_is_widened_exactly(dtype):
    # one key per request: o = V[0] * v_scale exactly (p = 1, l = 1), so every finite code shows its value
    b = workloads.make_batch("codes", 70, dtype, 2, 2, 128, 16, [1, 1], [1, 1], False, permute_pages=False,
                             kv_dtype=FP8, k_scale=1.0, v_scale=0.25)
    v = b.v_bits.copy()
    codes = np.arange(256, dtype=np.uint8)
    codes[[0x7F, 0xFF]] = 0          # the two NaN codes are left out
    v[0, 0, 0, :] = codes[:128]      # request 0 = page 0, kv head 0 / 1: codes 0..127 / 128..255
    v[0, 1, 0, :] = codes[128:]
    v[1, 0, 0, :] = codes[128:][::-1]
    v[1, 1, 0, :] = codes[:128][::-1]
    b = dataclasses.replace(b, v_bits=v)
    o, lse = check(b, f"all codes {dtype}")
    want = e4m3_to_f64(b.v_bits[:, :, 0, :]) * b.v_scale           # [request = page, head, D]
    assert np.array_equal(o, want), "one key: the output is that key's V, bit for bit"


@pytest.mark.parametrize("g", [1, 2, 4])
@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
def test_random_batches(g, dtype):
    for seed in (201, 202):
        b = workloads.random_case(seed + g, dtype=dtype, num_qo_heads=2 * g, num_kv_heads=2, batch=6, max_kv=400,
                                  kv_dtype=FP8, k_scale=0.5, v_scale=2.0)
        check(b, f"rand g={g} {dtype}")


def test_ragged_tails_and_every_tile_count():
    # 1..9 tiles of 32 tokens with every kind of tail: the four-deep load pipeline starts and drains cleanly
    kv = [1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 160, 191, 192, 193, 255, 256, 257, 288]
    b = workloads.make_batch("tails", 71, workloads.BF16, 8, 2, 128, 16, [1] * len(kv), kv, False, kv_dtype=FP8,
                             k_scale=2.0, v_scale=0.5)
    check(b, "tails", num_ctas=2 * 8, min_chunk=4096)


def test_split_chunks_and_merge():
    b = workloads.make_batch("split8", 72, workloads.BF16, 8, 2, 128, 16, [1, 1, 1], [3000, 40, 700], False,
                             kv_dtype=FP8, k_scale=0.5, v_scale=2.0)
    check(b, "split", num_ctas=2 * 16, min_chunk=64)


def test_strided_pool_layout():
    b = workloads.make_batch("nhd8", 73, workloads.F16, 8, 2, 128, 16, [1, 1, 1], [333, 64, 200], False, kv_dtype=FP8,
                             k_scale=1.0, v_scale=1.0)
    check(b, "NHD", dev=DeviceBatch(b, kv_layout="NHD"))


def test_small_decode_workloads():
    check(workloads.config2(small=True, kv_dtype=FP8), "c2 small")
    check(workloads.config4(small=True, kv_dtype=FP8), "c4 small")


def test_append_handle_refuses_the_8_bit_cache():
    import torch
    import paper_2501_01005_amd as fi
    b = workloads.make_batch("refuse", 74, workloads.BF16, 4, 1, 128, 16, [3], [40], True, kv_dtype=FP8)
    dev = DeviceBatch(b)
    w = fi.PagedAttention(dtype=b.dtype, num_qo_heads=4, num_kv_heads=1, mode="append", max_batch=1, max_qo_tiles=1)
    w.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=True)
    with pytest.raises(fi.Fi355Error) as ei:
        w.run(dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, b.sm_scale, k_scale=1.0, v_scale=1.0)
    assert ei.value.code == fi.FI_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    w.close()
