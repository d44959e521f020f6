"""GPU parity for the output written in the input type only (fi_run with o = NULL, o_cast given): every kernel
that writes final rows (decode, the contraction kernel, the contraction inside the decode launch, both paths of
the append kernel) must write the same 16-bit rows as when it writes both outputs, the same lse, and stay
within the comparison bound of the oracle plus half a unit in the last place of the 16-bit type."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, LSE_TOL, O_TOL, make_wrapper

pytestmark = pytest.mark.gpu

CASES = [
    # decode: split and unsplit requests, a one-token and an empty one
    ("decode", dict(min_chunk=32), 8, 2, [1] * 5, [3000, 700, 40, 1, 0], False),
    ("decode", dict(min_chunk=32, merge=2), 8, 2, [1] * 5, [3000, 700, 40, 1, 0], False),
    # append: scheduled-loop items, general-path items, idle wavefronts, split chunks
    ("append", dict(num_ctas=8, min_chunk=1024), 8, 2, [64, 3, 64, 130, 1, 40, 200], [300, 50, 128, 700, 100, 140, 260], True),
    ("append", dict(num_ctas=16, min_chunk=256), 8, 2, [70, 130], [900, 1500], True),
    ("append", dict(num_ctas=8, min_chunk=1024), 4, 1, [64, 30], [1000, 777], False),
]


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_output_in_the_input_type_only(case, dtype):
    import torch
    mode, kw, hq, hkv, qo, kv, causal = CASES[case]
    b = workloads.make_batch("out16", 300 + case, dtype, hq, hkv, 128, 16, qo, kv, causal)
    print(f"[case] 16-bit output only: {mode} {kw} dtype={dtype} heads={hq}/{hkv} qo={qo} kv={kv} causal={causal}", flush=True)
    o_ref, lse_ref = oracle.run_batch(b)
    dev = DeviceBatch(b)
    w = make_wrapper(b, mode, **kw)
    w.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=causal)
    nnz = dev.q.shape[0]
    bits = torch.int16

    def run(with_wide):
        o = torch.full((nnz, hq, 128), float("nan"), dtype=torch.float32, device=dev.device) if with_wide else False
        lse = torch.full((nnz, hq), float("nan"), dtype=torch.float32, device=dev.device)
        oc = torch.full((nnz, hq, 128), -7.0, dtype=dev.q.dtype, device=dev.device)
        w.run(dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, b.sm_scale, o=o, lse=lse, o_cast=oc)
        torch.cuda.synchronize()
        return oc, lse

    oc_both, lse_both = run(True)
    oc_only, lse_only = run(False)
    assert torch.equal(oc_only.view(bits), oc_both.view(bits)), "the 16-bit rows differ from those written beside the fp32 rows"
    assert torch.equal(lse_only.view(torch.int32), lse_both.view(torch.int32))
    sel = ~np.isnan(lse_ref)
    oc = oc_only.double().cpu().numpy()
    lse = lse_only.double().cpu().numpy()
    ulp = 2.0 ** -8 if dtype == workloads.BF16 else 2.0 ** -11
    err = np.abs(oc[sel] - o_ref[sel])
    assert np.all(err <= O_TOL + np.abs(o_ref[sel]) * ulp), f"max |o16 - o_ref| = {err.max():.3e}"
    fin = sel & ~np.isneginf(lse_ref)
    assert np.array_equal(np.isneginf(lse) & sel, np.isneginf(lse_ref) & sel)
    assert np.abs(lse[fin] - lse_ref[fin]).max() <= LSE_TOL
    print(f"[ok] 16-bit output only: err_o={err.max():.2e}", flush=True)
    w.close()


def test_no_output_at_all_is_an_error():
    import torch
    import paper_2501_01005_amd as fi
    b = workloads.make_batch("noout", 320, workloads.BF16, 8, 2, 128, 16, [1, 1], [40, 20], False)
    dev = DeviceBatch(b)
    w = make_wrapper(b, "decode")
    w.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=False)
    lse = torch.zeros((2, 8), dtype=torch.float32, device=dev.device)
    strides = (dev.k_pool.stride(0), dev.k_pool.stride(1), dev.k_pool.stride(2))
    with pytest.raises(fi.Fi355Error) as ei:
        fi.fi_run(w.handle, dev.q, dev.k_pool, dev.v_pool, strides, dev.kv_indices, b.sm_scale, None, lse, None, 0)
    assert ei.value.code == fi.FI_ERR_INVALID_ARG
    w.close()
