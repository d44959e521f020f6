"""GPU parity of contiguous KV (fi_run with kv_indices = NULL: the identity page table, rows addressed affinely,
no page id loaded; the dense baseline of App. B) against the fp64 oracle and against the paged run with an
explicit identity table (same arithmetic: the same bits)."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, assert_close, run_gpu

pytestmark = pytest.mark.gpu


def check(batch, mode, what, layout="HND", same_path=True, **kw):
    print(f"[case] {what}: {batch.name} page_size={batch.page_size} layout={layout} qo={batch.qo_lens()[:6].tolist()} "
          f"kv={batch.kv_lens()[:6].tolist()} kw={kw}", flush=True)
    o_ref, lse_ref = oracle.run_batch(batch)
    dev = DeviceBatch(batch, kv_layout=layout)
    o, lse = run_gpu(batch, mode, dev=dev, contiguous=True, **kw)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    o_p, lse_p = run_gpu(batch, mode, dev=dev, **kw)                      # the identity table given explicitly
    if same_path:
        assert np.array_equal(o, o_p) and np.array_equal(lse, lse_p), f"{what}: differs from the paged run"
    else:
        assert_close(o_p, lse_p, o_ref, lse_ref, what + " (paged run)")
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}" + ("; bit-identical to the paged run" if same_path else ""),
          flush=True)


@pytest.mark.parametrize("layout", ["HND", "NHD"])
@pytest.mark.parametrize("page_size", [16, 1, 8])
def test_decode_over_contiguous_kv(page_size, layout):
    b = workloads.config2(small=True, permute_pages=False, page_size=page_size)
    check(b, "decode", f"decode contiguous ps{page_size}", layout, num_ctas=8 * 32, min_chunk=64)


@pytest.mark.parametrize("layout", ["HND", "NHD"])
@pytest.mark.parametrize("page_size", [16, 1, 2, 4, 8, 32, 64])
def test_append_over_contiguous_kv(page_size, layout):
    """At every page size the run without a page table takes the same variant of the scheduled loop as the paged run,
    with computed instead of loaded page ids (page size 64: both on the general path): the same bits."""
    b = workloads.config3(small=True, permute_pages=False, page_size=page_size)
    check(b, "append", f"append contiguous ps{page_size}", layout)              # default grid
    check(b, "append", f"append contiguous ps{page_size}, split", layout, num_ctas=8 * 16, min_chunk=32)
    # long chunks on few CTAs: several items per CTA run the loop back to back (the next item's first tiles are
    # requested with computed ids too)
    b = workloads.make_batch("contig_chain", 77 + page_size, workloads.F16, 8, 2, 128, page_size, [200, 64, 130, 300],
                             [1500, 700, 131, 900], True, permute_pages=False)
    check(b, "append", f"append contiguous chain ps{page_size}", layout, num_ctas=2 * 3, min_chunk=128)


def test_ragged_tensor_is_page_size_one_nhd():
    """[tokens, H_kv, D] with a request's tokens in consecutive rows = page size 1, layout NHD, no page table."""
    import torch
    b = workloads.config2(small=True, permute_pages=False, page_size=1)
    dev = DeviceBatch(b, kv_layout="NHD")
    st = dev.k_pool.stride()   # (page = token, head, slot: a dimension of size 1, d)
    assert (st[0], st[1], st[3]) == (b.num_kv_heads * 128, 128, 1) and dev.k_pool.shape[2] == 1
    check(b, "decode", "ragged tensor", "NHD")


def test_full_sizes_equal_the_paged_run_with_an_identity_table():
    for b, mode in ((workloads.config2(permute_pages=False), "decode"), (workloads.config3(permute_pages=False), "append")):
        print(f"[case] contiguous at full size: {b.name}", flush=True)
        dev = DeviceBatch(b)
        o, lse = run_gpu(b, mode, dev=dev, contiguous=True)
        o_p, lse_p = run_gpu(b, mode, dev=dev)
        assert not np.isnan(o).any() and np.array_equal(o, o_p) and np.array_equal(lse, lse_p)
        sample = [0, b.batch // 2, b.batch - 1]
        o_ref, lse_ref = oracle.run_batch(b, requests=sample)
        e = assert_close(o, lse, o_ref, lse_ref, b.name)
        print(f"[ok] {b.name}: bit-identical to the paged run; requests {sample} vs oracle err_o={e[0]:.2e}", flush=True)


def test_refused_where_not_built():
    import torch
    import paper_2501_01005_amd as fi
    b = workloads.config2(small=True, permute_pages=False, kv_dtype=workloads.FP8)
    with pytest.raises(fi.Fi355Error) as e:
        run_gpu(b, "decode", contiguous=True)
    assert e.value.code == fi.FI_ERR_UNSUPPORTED
