"""GPU parity for fi_run_composed (Sec. 3.1.2 composable formats, Sec. 2.2 merge): two planned passes over the
same query rows and one contraction launch.  Checked against the oracle on the single-format problem and, bit for
bit, against fi_run on each handle followed by fi_merge_state_pair."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, assert_close, make_wrapper

pytestmark = pytest.mark.gpu


def separate(wa, wb, dev_a, dev_b, sm_scale):
    import torch
    import paper_2501_01005_amd as fi
    o_a, l_a = wa.run(dev_a.q, dev_a.k_pool, dev_a.v_pool, dev_a.kv_indices, sm_scale)
    o_b, l_b = wb.run(dev_b.q, dev_b.k_pool, dev_b.v_pool, dev_b.kv_indices, sm_scale)
    o = torch.empty_like(o_a); l = torch.empty_like(l_a)
    fi.fi_merge_state_pair(o_a, l_a, o_b, l_b, l_a.numel(), 128, o, l, torch.cuda.current_stream().cuda_stream)
    return o, l


@pytest.mark.parametrize("kw_p,kw_s", [(dict(min_chunk=64), dict(min_chunk=32)),        # split tiles in both passes
                                       (dict(min_chunk=4096), dict(num_ctas=8, min_chunk=4096)),   # none split
                                       (dict(min_chunk=64), dict(num_ctas=8, min_chunk=4096))])
def test_shared_prefix_in_three_launches(kw_p, kw_s):
    import torch
    c = workloads.config5(small=True)
    print(f"[case] c5 small composed: prefix {kw_p} suffix {kw_s}", flush=True)
    o_ref, lse_ref = oracle.run_batch(c.single)
    dev_p, dev_s = DeviceBatch(c.prefix), DeviceBatch(c.suffix)
    wp = make_wrapper(c.prefix, "append", **kw_p)
    ws = make_wrapper(c.suffix, "decode", **kw_s)
    wp.plan(c.prefix.qo_indptr, c.prefix.kv_indptr, c.prefix.last_page_len, causal=False)
    ws.plan(c.suffix.qo_indptr, c.suffix.kv_indptr, c.suffix.last_page_len, causal=False)
    o_sep, l_sep = separate(wp, ws, dev_p, dev_s, c.prefix.sm_scale)
    for first, second, ia, ib in ((wp, ws, dev_p.kv_indices, dev_s.kv_indices), (ws, wp, dev_s.kv_indices, dev_p.kv_indices)):
        o = torch.full_like(o_sep, float("nan")); l = torch.full_like(l_sep, float("nan"))
        oc = torch.zeros(o.shape, dtype=dev_p.q.dtype, device=o.device)
        first.run_composed(second, dev_p.q, dev_p.k_pool, dev_p.v_pool, ia, ib, c.prefix.sm_scale, o=o, lse=l, o_cast=oc)
        torch.cuda.synchronize()
        e = assert_close(o.double().cpu().numpy(), l.double().cpu().numpy(), o_ref, lse_ref, "c5 composed in one contraction")
        if first is wp:
            assert torch.equal(o.view(torch.int32), o_sep.view(torch.int32)) and torch.equal(l.view(torch.int32), l_sep.view(torch.int32))
        assert torch.equal(oc.view(torch.int16), o.to(oc.dtype).view(torch.int16))
        # the rounded rows alone
        oc2 = torch.zeros_like(oc); l2 = torch.full_like(l, float("nan"))
        first.run_composed(second, dev_p.q, dev_p.k_pool, dev_p.v_pool, ia, ib, c.prefix.sm_scale, o=False, lse=l2, o_cast=oc2)
        torch.cuda.synchronize()
        assert torch.equal(oc2.view(torch.int16), oc.view(torch.int16)) and torch.equal(l2.view(torch.int32), l.view(torch.int32))
        print(f"[ok] c5 small composed: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    view_p = __import__("paper_2501_01005_amd").fi_plan_view(wp.handle)
    assert (int(view_p["n_merge"]) > 0) == (kw_p["min_chunk"] == 64)
    wp.close(); ws.close()


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
def test_two_decode_passes_over_halves_of_the_cache(dtype):
    """Each request's pages cut in two formats (the first k pages, the rest); requests whose second part is empty
    contribute the identity state there; long parts are split into chunks, short ones are not."""
    import torch
    kv = [3000, 700, 40, 16, 1, 333]
    cut_pages = [100, 20, 1, 1, 1, 0]          # pages of each request that go to the first format
    b = workloads.make_batch("halves", 400, dtype, 8, 2, 128, 16, [1] * len(kv), kv, False)
    o_ref, lse_ref = oracle.run_batch(b)
    ia, ib, pa, pb, la, lb = [], [], [0], [0], [], []
    for r in range(b.batch):
        pages = b.kv_indices[b.kv_indptr[r]:b.kv_indptr[r + 1]]
        k = min(cut_pages[r], len(pages))
        ia.append(pages[:k]); ib.append(pages[k:])
        pa.append(pa[-1] + k); pb.append(pb[-1] + len(pages) - k)
        # a format that holds the request's last page inherits its fill; full pages elsewhere
        la.append(int(b.last_page_len[r]) if k == len(pages) and k > 0 else (16 if k > 0 else 1))
        lb.append(int(b.last_page_len[r]) if len(pages) > k else 1)
    print(f"[case] two decode formats: dtype={dtype} kv={kv} first-format pages={cut_pages}", flush=True)
    dev = DeviceBatch(b)
    idx_a = torch.from_numpy(np.concatenate(ia).astype(np.int32)).to(dev.device)
    idx_b = torch.from_numpy(np.concatenate(ib).astype(np.int32)).to(dev.device)
    wa = make_wrapper(b, "decode", min_chunk=32)
    wb = make_wrapper(b, "decode", min_chunk=64)
    wa.plan(b.qo_indptr, np.asarray(pa, dtype=np.int32), np.asarray(la, dtype=np.int32), causal=False)
    wb.plan(b.qo_indptr, np.asarray(pb, dtype=np.int32), np.asarray(lb, dtype=np.int32), causal=False)
    for rep in range(2):
        o, l = wa.run_composed(wb, dev.q, dev.k_pool, dev.v_pool, idx_a, idx_b, b.sm_scale)
        torch.cuda.synchronize()
        e = assert_close(o.double().cpu().numpy(), l.double().cpu().numpy(), o_ref, lse_ref, f"two formats rep {rep}")
    print(f"[ok] two decode formats: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    wa.close(); wb.close()


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
def test_prefill_over_a_shared_prefix(dtype):
    """Two append-mode formats (Sec. 3.1.2 with multi-token queries): every request appends its own tokens after a
    common prefix.  Format a: all query rows as one row block over the prefix pages, not causal; format b: each
    request's own tokens, causal.  The single format (every request: prefix + own tokens, causal) is what the
    oracle computes; its copies of the prefix hold the same values as the shared pages."""
    import dataclasses
    import torch
    prefix, qo = 304, [70, 9, 130, 1, 64]
    n_pre = prefix // 16
    single = workloads.make_batch("sharedprefill", 450, dtype, 8, 2, 128, 16, qo, [prefix + q for q in qo], True)
    k_bits, v_bits = single.k_bits.copy(), single.v_bits.copy()
    shared = single.kv_indices[single.kv_indptr[0]:single.kv_indptr[0] + n_pre]
    own, own_indptr = [], [0]
    for r in range(len(qo)):
        pages = single.kv_indices[single.kv_indptr[r]:single.kv_indptr[r + 1]]
        k_bits[pages[:n_pre]] = k_bits[shared]
        v_bits[pages[:n_pre]] = v_bits[shared]
        own.append(pages[n_pre:])
        own_indptr.append(own_indptr[-1] + len(pages) - n_pre)
    single = dataclasses.replace(single, k_bits=k_bits, v_bits=v_bits)
    print(f"[case] prefill over a shared prefix: {dtype} prefix={prefix} qo={qo}", flush=True)
    o_ref, lse_ref = oracle.run_batch(single)
    dev = DeviceBatch(single)
    nnz = int(single.qo_indptr[-1])
    fmt_a = dataclasses.replace(single, qo_indptr=np.array([0, nnz], dtype=np.int32), kv_indptr=np.array([0, n_pre], dtype=np.int32),
                                kv_indices=shared.copy(), last_page_len=np.array([16], dtype=np.int32), causal=False)
    wa = make_wrapper(fmt_a, "append", num_ctas=2 * 4, min_chunk=64)
    wb = make_wrapper(single, "append", num_ctas=2 * 4, min_chunk=64)
    wa.plan(fmt_a.qo_indptr, fmt_a.kv_indptr, fmt_a.last_page_len, causal=False)
    wb.plan(single.qo_indptr, np.asarray(own_indptr, dtype=np.int32), single.last_page_len, causal=True)
    idx_a = torch.from_numpy(shared.astype(np.int32)).to(dev.device)
    idx_b = torch.from_numpy(np.concatenate(own).astype(np.int32)).to(dev.device)
    o, l = wa.run_composed(wb, dev.q, dev.k_pool, dev.v_pool, idx_a, idx_b, single.sm_scale)
    torch.cuda.synchronize()
    e = assert_close(o.double().cpu().numpy(), l.double().cpu().numpy(), o_ref, lse_ref, "prefill over a shared prefix")
    print(f"[ok] prefill over a shared prefix: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    wa.close(); wb.close()


def test_merge_lists_longer_than_a_wavefront():
    """150 requests, most of them split in both formats: the contraction looks a row's tile up in merge lists of
    more than 64 entries (searched 64 at a time).  Checked against the oracle and, bit for bit, against the
    separate launches."""
    import torch
    import paper_2501_01005_amd as fi
    rng = np.random.default_rng(77)
    B = 150
    kv = rng.integers(0, 1500, size=B)
    b = workloads.make_batch("longlists", 430, workloads.BF16, 8, 2, 128, 16, [1] * B, kv.tolist(), False)
    ia, ib, pa, pb, la, lb = [], [], [0], [0], [], []
    for r in range(B):
        pages = b.kv_indices[b.kv_indptr[r]:b.kv_indptr[r + 1]]
        k = int(rng.integers(0, len(pages) + 1))
        ia.append(pages[:k]); ib.append(pages[k:])
        pa.append(pa[-1] + k); pb.append(pb[-1] + len(pages) - k)
        la.append(int(b.last_page_len[r]) if k == len(pages) and k > 0 else (16 if k > 0 else 1))
        lb.append(int(b.last_page_len[r]) if len(pages) > k else 1)
    dev = DeviceBatch(b)
    cat = lambda xs: torch.from_numpy(np.concatenate(xs + [np.zeros(1, dtype=np.int32)]).astype(np.int32)).to(dev.device)
    idx_a, idx_b = cat(ia), cat(ib)
    wa, wb = make_wrapper(b, "decode", min_chunk=16), make_wrapper(b, "decode", min_chunk=16)
    wa.plan(b.qo_indptr, np.asarray(pa, dtype=np.int32), np.asarray(la, dtype=np.int32), causal=False)
    wb.plan(b.qo_indptr, np.asarray(pb, dtype=np.int32), np.asarray(lb, dtype=np.int32), causal=False)
    n_a, n_b = int(fi.fi_plan_view(wa.handle)["n_merge"]), int(fi.fi_plan_view(wb.handle)["n_merge"])
    print(f"[case] long merge lists: split tiles {n_a}, {n_b}", flush=True)
    assert n_a > 64 and n_b > 64
    o_ref, lse_ref = oracle.run_batch(b)
    o, l = wa.run_composed(wb, dev.q, dev.k_pool, dev.v_pool, idx_a, idx_b, b.sm_scale)
    torch.cuda.synchronize()
    assert_close(o.double().cpu().numpy(), l.double().cpu().numpy(), o_ref, lse_ref, "long merge lists")
    o_a, l_a = wa.run(dev.q, dev.k_pool, dev.v_pool, idx_a, b.sm_scale)
    o_b, l_b = wb.run(dev.q, dev.k_pool, dev.v_pool, idx_b, b.sm_scale)
    o2 = torch.empty_like(o_a); l2 = torch.empty_like(l_a)
    fi.fi_merge_state_pair(o_a, l_a, o_b, l_b, l_a.numel(), 128, o2, l2, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(o2.view(torch.int32), o.view(torch.int32)) and torch.equal(l2.view(torch.int32), l.view(torch.int32))
    wa.close(); wb.close()


def test_an_empty_format_is_the_identity():
    """A format in which no request has keys contributes the identity state: the composition equals fi_run on the
    other format bit for bit; two empty formats give zero rows with lse = -inf."""
    import torch
    kv = [900, 40, 1, 0, 333]
    b = workloads.make_batch("idstate", 420, workloads.BF16, 8, 2, 128, 16, [1] * len(kv), kv, False)
    dev = DeviceBatch(b)
    wa = make_wrapper(b, "decode", min_chunk=32)
    wb = make_wrapper(b, "decode")
    zeros = np.zeros(len(kv) + 1, dtype=np.int32)
    wa.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=False)
    wb.plan(b.qo_indptr, zeros, np.ones(len(kv), dtype=np.int32), causal=False)
    no_pages = torch.zeros(1, dtype=torch.int32, device=dev.device)
    o_a, l_a = wa.run(dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, b.sm_scale)
    for first, second, ia, ib in ((wa, wb, dev.kv_indices, no_pages), (wb, wa, no_pages, dev.kv_indices)):
        o, l = first.run_composed(second, dev.q, dev.k_pool, dev.v_pool, ia, ib, b.sm_scale)
        torch.cuda.synchronize()
        assert torch.equal(o.view(torch.int32), o_a.view(torch.int32)) and torch.equal(l.view(torch.int32), l_a.view(torch.int32))
    wa.plan(b.qo_indptr, zeros, np.ones(len(kv), dtype=np.int32), causal=False)
    o, l = wa.run_composed(wb, dev.q, dev.k_pool, dev.v_pool, no_pages, no_pages, b.sm_scale)
    torch.cuda.synchronize()
    assert torch.count_nonzero(o).item() == 0 and torch.isneginf(l).all().item()
    wa.close(); wb.close()


def test_composed_argument_errors():
    import torch
    import paper_2501_01005_amd as fi
    b = workloads.make_batch("cerr", 410, workloads.BF16, 8, 2, 128, 16, [1, 1], [40, 20], False)
    b3 = workloads.make_batch("cerr3", 411, workloads.BF16, 8, 2, 128, 16, [1, 1, 1], [40, 20, 16], False)
    dev = DeviceBatch(b)
    wa, wb, wc = make_wrapper(b, "decode"), make_wrapper(b, "decode"), make_wrapper(b3, "decode")
    for w, x in ((wa, b), (wb, b), (wc, b3)):
        w.plan(x.qo_indptr, x.kv_indptr, x.last_page_len, causal=False)
    with pytest.raises(fi.Fi355Error) as ei:
        wa.run_composed(wa, dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, dev.kv_indices, b.sm_scale)
    assert ei.value.code == fi.FI_ERR_INVALID_ARG
    with pytest.raises(fi.Fi355Error) as ei:   # the plans cover 2 and 3 query rows
        wa.run_composed(wc, dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, dev.kv_indices, b.sm_scale)
    assert ei.value.code == fi.FI_ERR_INVALID_ARG and "query rows" in ei.value.message
    torch.cuda.synchronize()
    for w in (wa, wb, wc):
        w.close()
