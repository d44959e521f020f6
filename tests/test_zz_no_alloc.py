"""fi_run_composed_static (the entry point for callers that cannot allocate: its pass state rows live in a
static device array of the library) against fi_run_composed with caller buffers: two calls in a row on one
GPU, the second over fewer query rows, so that the array still holds the first call's rows."""
import dataclasses

import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, assert_close, make_wrapper

pytestmark = pytest.mark.gpu


def first_requests(case, n):
    """The shared-prefix case restricted to its first n requests (same pools, same prefix pages)."""
    def cut(b, qo_indptr, kv_indptr, last):
        return dataclasses.replace(b, qo_indptr=np.asarray(qo_indptr, dtype=np.int32),
                                   kv_indptr=np.asarray(kv_indptr, dtype=np.int32),
                                   last_page_len=np.asarray(last, dtype=np.int32), q_bits=b.q_bits[:n])
    p, s, o = case.prefix, case.suffix, case.single
    return workloads.SharedPrefixCase(
        prefix=cut(p, [0, n], p.kv_indptr, p.last_page_len),
        suffix=cut(s, s.qo_indptr[:n + 1], s.kv_indptr[:n + 1], s.last_page_len[:n]),
        single=cut(o, o.qo_indptr[:n + 1], o.kv_indptr[:n + 1], o.last_page_len[:n]))


def test_static_scratch_entry_point_equals_the_one_with_caller_buffers():
    import torch
    import paper_2501_01005_amd as fi
    big = workloads.config5(small=True)
    for case, what in ((big, "8 requests"), (first_requests(big, 3), "then 3 requests")):
        c = case
        print(f"[case] fi_run_composed_static, {what}: prefix {int(c.prefix.kv_lens()[0])} tokens, "
              f"suffixes {c.suffix.kv_lens().tolist()}", flush=True)
        dev_p, dev_s = DeviceBatch(c.prefix), DeviceBatch(c.suffix)
        wp, ws = make_wrapper(c.prefix, "append", min_chunk=64), make_wrapper(c.suffix, "decode", min_chunk=32)
        wp.plan(c.prefix.qo_indptr, c.prefix.kv_indptr, c.prefix.last_page_len, causal=False)
        ws.plan(c.suffix.qo_indptr, c.suffix.kv_indptr, c.suffix.last_page_len, causal=False)
        view_p, view_s = fi.fi_plan_view(wp.handle), fi.fi_plan_view(ws.handle)
        assert view_p["n_merge"] > 0, "the prefix tile must be split, so that both kinds of state rows are read"
        n, H, D = dev_p.q.shape[0], c.prefix.num_qo_heads, 128
        o_ref_gpu, lse_ref_gpu = wp.run_composed(ws, dev_p.q, dev_p.k_pool, dev_p.v_pool, dev_p.kv_indices,
                                                 dev_s.kv_indices, c.prefix.sm_scale)
        o = torch.full((n, H, D), float("nan"), dtype=torch.float32, device="cuda:0")
        lse = torch.full((n, H), float("nan"), dtype=torch.float32, device="cuda:0")
        strides = (dev_p.k_pool.stride(0), dev_p.k_pool.stride(1), dev_p.k_pool.stride(2))
        fi.fi_run_composed_static(wp.handle, ws.handle, dev_p.q, dev_p.k_pool, dev_p.v_pool, strides, dev_p.kv_indices,
                                  dev_s.kv_indices, c.prefix.sm_scale, n, o, lse, None,
                                  torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        # the same kernels on the same plans: the same bits
        assert torch.equal(o.view(torch.int32), o_ref_gpu.view(torch.int32)), what
        assert torch.equal(lse.view(torch.int32), lse_ref_gpu.view(torch.int32)), what
        o_ref, lse_ref = oracle.run_batch(c.single)
        e = assert_close(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, what)
        print(f"[ok] {what}: bit-identical to fi_run_composed; vs oracle err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
        wp.close(); ws.close()


def test_static_scratch_entry_point_rejects_more_rows_than_it_holds():
    import torch
    import paper_2501_01005_amd as fi
    c = workloads.config5(small=True)
    wp, ws = make_wrapper(c.prefix, "append"), make_wrapper(c.suffix, "decode")
    dummy = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    with pytest.raises(fi.Fi355Error) as err:
        fi.fi_run_composed_static(wp.handle, ws.handle, dummy, dummy, dummy, (2048 * 8, 2048, 128), dummy, dummy, 0.1,
                                  4096 // 32 + 1, dummy, dummy, None, 0)
    assert err.value.code == fi.FI_ERR_WORKSPACE_TOO_SMALL and "4096" in err.value.message
    wp.close(); ws.close()
