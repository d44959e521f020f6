"""GPU parity for the hand-scheduled main loop of the append kernel: the chunk lengths at which a
work item switches between the generic path and the loop, tiles cut by the causal diagonal or
by the end of the chunk, reference raises, split chunks (partial slots), both input types,
every GQA group size, the strided pool layout and the rounded copy of the output."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, O_TOL, assert_close, run_gpu

pytestmark = pytest.mark.gpu


def check(batch, what, dev=None, **kw):
    print(f"[case] {what}: {batch.name} dtype={batch.dtype} heads={batch.num_qo_heads}/{batch.num_kv_heads} "
          f"qo={batch.qo_lens()[:8].tolist()} kv={batch.kv_lens()[:8].tolist()} causal={batch.causal} kw={kw}", flush=True)
    o_ref, lse_ref = oracle.run_batch(batch)
    o, lse = run_gpu(batch, "append", dev=dev, **kw)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)


@pytest.mark.parametrize("causal", [False, True])
def test_chunk_lengths_around_the_loop_thresholds(causal):
    # the loop takes chunks of >= 128 tokens whose first 64 every row sees; 64-token tiles
    kvs = [127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 321]
    for qo in (1, 17, 64, 65):
        lens = [kv for kv in kvs if kv >= qo]
        b = workloads.make_batch("thr", 31 + qo, workloads.BF16, 4, 1, 128, 16, [qo] * len(lens), lens, causal)
        check(b, f"thresholds qo={qo}", num_ctas=4, min_chunk=1024)


@pytest.mark.parametrize("g", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
def test_group_sizes_and_input_types(g, dtype):
    b = workloads.make_batch("gq", 50 + g, dtype, 2 * g, 2, 128, 16, [256 // g + 3, 40, 9], [500, 333, 200], True)
    check(b, f"g={g} {dtype}", num_ctas=2 * 4, min_chunk=1024)


def test_split_chunks_go_through_partial_slots():
    # small chunks force every long tile to be split: the loop writes partial states, merge folds them
    b = workloads.make_batch("split", 61, workloads.BF16, 8, 2, 128, 16, [70, 130], [900, 1500], True)
    check(b, "split 256", num_ctas=2 * 32, min_chunk=256)
    check(b, "split 192", num_ctas=2 * 64, min_chunk=192)
    nc = workloads.make_batch("splitnc", 62, workloads.F16, 8, 2, 128, 16, [64, 30], [1000, 777], False)
    check(nc, "split non-causal", num_ctas=2 * 16, min_chunk=128)


def test_reference_is_raised_inside_the_loop():
    # logits that grow along the sequence: every later tile holds a new row maximum, far beyond the
    # headroom the lazy softmax leaves, also inside the tiles the diagonal cuts
    import dataclasses
    b = workloads.make_batch("grow", 63, workloads.BF16, 4, 1, 128, 16, [64, 20], [512, 300], True, permute_pages=False,
                             poison=False)
    k = workloads.widen(b.k_bits, b.dtype).copy()       # [P, Hkv, 16, D]
    q = workloads.widen(b.q_bits, b.dtype)
    n_pages = k.shape[0]
    ramp = (np.arange(n_pages * 16, dtype=np.float64).reshape(n_pages, 1, 16, 1) / 16.0) ** 1.0
    direction = np.sign(q[0, 0]).reshape(1, 1, 1, -1)   # every query has positive overlap with it on average
    k = 0.25 * k + 0.1 * ramp * direction
    b2 = dataclasses.replace(b, k_bits=workloads.f32_to_bits(k.astype(np.float32), b.dtype))
    check(b2, "growing logits", num_ctas=4, min_chunk=1024)


def test_strided_pool_layout_and_rounded_output():
    import torch
    b = workloads.make_batch("nhd", 64, workloads.BF16, 8, 2, 128, 16, [64, 33], [400, 260], True)
    dev = DeviceBatch(b, kv_layout="NHD")
    check(b, "NHD layout", dev=dev, num_ctas=2 * 4, min_chunk=1024)
    for dtype in (workloads.BF16, workloads.F16):
        b = workloads.make_batch("cast", 65, dtype, 8, 2, 128, 16, [64, 33], [400, 260], True)
        o, lse, oc = run_gpu(b, "append", with_cast=True, num_ctas=2 * 4, min_chunk=1024)
        ulp = 2.0 ** -8 if dtype == workloads.BF16 else 2.0 ** -11
        bound = np.maximum(np.abs(o), 2.0 ** -14) * ulp
        assert np.all(np.abs(oc - o) <= bound), f"rounded output of {dtype} is off by more than half an ulp"
        o_ref, lse_ref = oracle.run_batch(b)
        assert_close(o, lse, o_ref, lse_ref, f"cast {dtype}")
        assert np.abs(oc - o_ref).max() <= O_TOL + np.abs(o_ref).max() * ulp


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
def test_seams_between_work_items_of_one_cta(dtype):
    """A single CTA per kv head walks the whole work list, so every kind of neighbour meets: an item of the
    scheduled loop after another one (its first tiles are requested into LDS while the one before writes its
    outputs), after a generic-path item, before one (the requested tiles are dropped), idle wavefronts (query tiles
    of less than 256 rows) on either side, chunks that end inside their second tile, and the last item."""
    qo = [64, 3, 64, 130, 1, 64, 40, 64, 64, 7, 200]
    kv = [300, 50, 128, 700, 100, 129, 140, 64, 191, 400, 260]
    for causal in (True, False):
        b = workloads.make_batch("seams", 70 + int(causal), dtype, 8, 2, 128, 16, qo, kv, causal)
        check(b, f"seams causal={causal}", num_ctas=2 * 1, min_chunk=1024)
        check(b, f"seams causal={causal}, split chunks", num_ctas=2 * 2, min_chunk=128)
