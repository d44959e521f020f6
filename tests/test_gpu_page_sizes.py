"""GPU parity for page sizes other than the tuned 16 (Sec. 3.1.1: the block size of the BSR cache is a free
parameter; App. B compares page sizes): decode goes through its general code path, where every lane looks up the
page of the token row it loads; append runs the scheduled loop's variant for page sizes 4, 8 and 32 (a wavefront's
four consecutive rows per load share a page), its per-row variant for page sizes 1 and 2 (a page id per token row,
64-bit addresses per lane) and the general path for page size 64."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, assert_close, run_gpu

pytestmark = pytest.mark.gpu


def check(batch, mode, what, dev=None, **kw):
    print(f"[case] {what}: {batch.name} mode={mode} page_size={batch.page_size} dtype={batch.dtype} kv={batch.kv_dtype} "
          f"qo={batch.qo_lens()[:8].tolist()} kv_len={batch.kv_lens()[:8].tolist()} kw={kw}", flush=True)
    o_ref, lse_ref = oracle.run_batch(batch)
    o, lse = run_gpu(batch, mode, dev=dev, **kw)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)


@pytest.mark.parametrize("ps", [1, 2, 8, 32, 64])
def test_decode(ps):
    for seed, dtype, kv_dtype in ((301, workloads.BF16, ""), (302, workloads.F16, ""), (303, workloads.BF16, workloads.FP8)):
        b = workloads.random_case(seed + ps, dtype=dtype, num_qo_heads=8, num_kv_heads=2, page_size=ps, batch=6,
                                  max_kv=400, kv_dtype=kv_dtype, k_scale=0.5 if kv_dtype else 1.0,
                                  v_scale=2.0 if kv_dtype else 1.0)
        check(b, "decode", f"decode ps={ps}")
    # long requests split over many CTAs (partial slots + merge), chunk boundaries on page boundaries
    b = workloads.make_batch("long", 310 + ps, workloads.BF16, 8, 2, 128, ps, [1, 1, 1], [2500, 77, 600], False)
    check(b, "decode", f"decode split ps={ps}", num_ctas=2 * 16, min_chunk=64)


@pytest.mark.parametrize("ps", [1, 2, 4, 8, 32, 64])
def test_append(ps):
    for seed, dtype, causal in ((321, workloads.BF16, True), (322, workloads.F16, False)):
        b = workloads.make_batch("app", seed + ps, dtype, 8, 2, 128, ps, [70, 9, 130, 1], [400, 9, 333, 64], causal)
        check(b, "append", f"append ps={ps} causal={causal}", num_ctas=2 * 4, min_chunk=128)
    b = workloads.make_batch("appsplit", 330 + ps, workloads.BF16, 8, 2, 128, ps, [64, 30], [1000, 777], True)
    check(b, "append", f"append split ps={ps}", num_ctas=2 * 16, min_chunk=128)


@pytest.mark.parametrize("ps", [1, 2, 4, 8, 32])
def test_append_work_items_that_follow_each_other_in_the_scheduled_loop(ps):
    """Default grid on the small causal-append configuration and long chunks on few CTAs: several work items per CTA
    run the loop back to back (the next item's first tiles are requested by the item before it), with ragged last
    pages, chunk ends inside a page-size-32 page pair, and both storage types."""
    check(workloads.config3(small=True, page_size=ps), "append", f"c3 small ps={ps}")
    for seed, dtype in ((351, workloads.BF16), (352, workloads.F16)):
        b = workloads.make_batch("appchain", seed + ps, dtype, 8, 2, 128, ps, [200, 64, 130, 300], [1500, 700, 131, 900], True)
        check(b, "append", f"append chain ps={ps}", num_ctas=2 * 3, min_chunk=128)
        check(b, "append", f"append chain ps={ps}, default grid")
    b = workloads.make_batch("appfull", 360 + ps, workloads.BF16, 8, 2, 128, ps, [64, 64], [2048, 1000], False)
    check(b, "append", f"append not causal ps={ps}", num_ctas=2 * 8, min_chunk=256)


def test_strided_layout_with_small_pages():
    b = workloads.make_batch("nhd_ps8", 340, workloads.BF16, 8, 2, 128, 8, [1, 1, 1], [333, 64, 200], False)
    check(b, "decode", "decode NHD ps=8", dev=DeviceBatch(b, kv_layout="NHD"))
    b = workloads.make_batch("nhd_ps8a", 341, workloads.BF16, 8, 2, 128, 8, [40, 3], [300, 64], True)
    check(b, "append", "append NHD ps=8", dev=DeviceBatch(b, kv_layout="NHD"), num_ctas=2 * 4, min_chunk=128)
