"""GPU parity of the 16-row and 64-row tile modes (query tile sizes that follow the query lengths, Sec. 3.2.2) and of
several formats planned and run as one work list (Sec. 3.1.2) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
import workloads
from oracle.plan_replica import plan_replica_formats
from gpu_util import DeviceBatch, assert_close, make_wrapper, run_gpu
from paper_2501_01005_amd.device import formats_of, make_formats_wrapper

pytestmark = pytest.mark.gpu

MODES = ["tile16", "tile64"]


def replica_kwargs(mode, g, min_chunk):
    """what fi_create sets for the planner in these modes (balance = 0)"""
    if mode == "tile16":
        return dict(t_pos=16 // g, min_chunk=min_chunk or 32, item_cost=64)
    return dict(t_pos=64 // g, min_chunk=min_chunk or 128, refine=True, light_rows=16, light_pct=30, kv_quantum=32,
                weighted_lkv=True)


def check(batch, what, mode, **kw):
    print(f"[case] {what}: {batch.name} qo={batch.qo_lens()[:8].tolist()} kv={batch.kv_lens()[:8].tolist()} "
          f"causal={batch.causal} kw={kw}", flush=True)
    o_ref, lse_ref = oracle.run_batch(batch)
    o, lse = run_gpu(batch, mode, **kw)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("seed", range(10))
def test_short_appends_causal_and_not(seed, mode):
    g = [1, 2, 4, 8, 16][seed % 5]
    dtype = workloads.F16 if seed % 2 else workloads.BF16
    causal = seed % 3 != 2
    b = workloads.random_case(700 + seed, dtype=dtype, num_qo_heads=2 * g, num_kv_heads=2, batch=2 + seed % 4,
                              max_qo=[3, 17, 40][seed % 3], max_kv=[90, 400, 900][seed % 3], causal=causal,
                              value_scale=[1.0, 0.5, 2.0][seed % 3])
    check(b, f"{mode} rand{seed}", mode, num_ctas=2 * [1, 3, 16, 64][seed % 4], min_chunk=[16, 32][seed % 2])


@pytest.mark.parametrize("mode", MODES)
def test_decode_batches_and_default_grid(mode):
    check(workloads.config2(small=True), f"c2 small as {mode}", mode)
    check(workloads.config1(), f"c1 as {mode}", mode)
    check(workloads.config3(small=True), f"c3 small (causal append) as {mode}", mode)


@pytest.mark.parametrize("mode", MODES)
def test_causal_edges(mode):
    # pure prefill over tile and step boundaries, more queries than keys (empty leading rows), an empty request
    for qo, kv in (([1], [1]), ([4], [4]), ([5], [5]), ([33], [33]), ([40], [25]), ([16, 3], [200, 0]), ([7], [71])):
        b = workloads.make_batch("edge", 19, workloads.BF16, 8, 2, 128, 16, qo, kv, True,
                                 num_pages=sum((k + 15) // 16 for k in kv) + 1)
        check(b, f"{mode} edge{qo}{kv}", mode, num_ctas=2 * 4, min_chunk=16)


@pytest.mark.parametrize("mode", MODES)
def test_one_format_at_a_time_with_the_small_workspace(mode):
    """fi_config.max_formats = 1: partial-state sections bounded by the CTAs; long requests split over many CTAs use
    them, with NaN everywhere else in the workspace"""
    b = workloads.make_batch("split", 23, workloads.BF16, 32, 8, 128, 16, [4, 1, 16, 3], [5000, 3000, 2500, 40], True)
    check(b, f"{mode} max_formats=1", mode, max_formats=1)
    check(b, f"{mode} max_formats=1, few CTAs", mode, max_formats=1, num_ctas=8 * 5, min_chunk=32)
    check(workloads.config2(small=True), f"c2 small as {mode}, max_formats=1", mode, max_formats=1)


def run_formats(case_batches, single, what, mode, **kw):
    import torch
    import paper_2501_01005_amd as fi
    print(f"[case] {what} ({mode}): formats {[(b.batch, int(b.kv_lens().sum())) for b in case_batches]}, kw={kw}", flush=True)
    formats, ids = formats_of(case_batches)
    w = make_formats_wrapper(case_batches, mode=mode, **kw)
    dev = DeviceBatch(case_batches[0])
    ids_dev = torch.from_numpy(ids).to("cuda:0")
    w.workspace.view(torch.float32)[w.pin_bytes // 4:].fill_(float("nan"))
    w.plan_formats(formats)
    view = fi.fi_plan_view(w.handle)
    g = case_batches[0].num_qo_heads // case_batches[0].num_kv_heads
    want = plan_replica_formats(formats, page_size=16, group=g, num_ctas=view["ctas_per_head"], causal=False,
                                **replica_kwargs(mode, g, kw.get("min_chunk")))
    for k in ("cta_indptr", "w_q_row0", "w_n_pos", "w_kv_page0", "w_kv_start", "w_kv_len", "w_out_slot", "row_indptr", "row_entry"):
        assert view[k].tobytes() == np.asarray(want[k], dtype=np.int32).tobytes(), k
    nnz, H = dev.q.shape[0], case_batches[0].num_qo_heads
    o = torch.full((nnz, H, 128), float("nan"), dtype=torch.float32, device="cuda:0")
    lse = torch.full((nnz, H), float("nan"), dtype=torch.float32, device="cuda:0")
    w.run(dev.q, dev.k_pool, dev.v_pool, ids_dev, case_batches[0].sm_scale, o=o, lse=lse)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.run_batch(single)
    e = assert_close(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, what)
    print(f"[ok] {what}: n_work={view['n_work']} L_kv={view['l_kv_chunk']} err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    w.close()
    return o, lse


@pytest.mark.parametrize("mode", MODES)
def test_shared_prefix_as_one_plan_small(mode):
    c = workloads.config5(small=True)
    run_formats([c.prefix, c.suffix], c.single, "c5 small, one plan", mode)
    run_formats([c.prefix, c.suffix], c.single, "c5 small, one plan, few CTAs", mode, num_ctas=8 * 3, min_chunk=16)
    # the other order of the formats folds the same states
    run_formats([c.suffix, c.prefix], c.single, "c5 small, suffix format first", mode)


@pytest.mark.parametrize("mode", MODES)
def test_shared_prefix_as_one_plan_full(mode):
    c = workloads.config5()
    run_formats([c.prefix, c.suffix], c.single, "c5 full, one plan", mode)


@pytest.mark.parametrize("mode", MODES)
def test_formats_with_empty_requests(mode):
    """A format whose request has no pages contributes the empty state; a row that is empty in every format gets
    o = 0, lse = -inf."""
    import dataclasses
    c = workloads.config5(small=True)
    s = c.suffix
    # the suffix of request 2 loses its pages
    n_pg = np.diff(s.kv_indptr).copy()
    n_pg[2] = 0
    kv_indptr = np.concatenate([[0], np.cumsum(n_pg)]).astype(np.int32)
    keep = np.concatenate([s.kv_indices[s.kv_indptr[i]:s.kv_indptr[i + 1]] for i in range(s.batch) if i != 2])
    last = s.last_page_len.copy()
    last[2] = 0
    s2 = dataclasses.replace(s, kv_indptr=kv_indptr, kv_indices=keep.astype(np.int32), last_page_len=last)
    # single-format view of the same problem
    pre = c.prefix.kv_indices
    idx, indptr = [], [0]
    for i in range(s2.batch):
        own = s2.kv_indices[s2.kv_indptr[i]:s2.kv_indptr[i + 1]]
        idx += [pre, own]
        indptr.append(indptr[-1] + len(pre) + len(own))
    last1 = np.where(np.diff(s2.kv_indptr) > 0, s2.last_page_len, 16).astype(np.int32)
    single = dataclasses.replace(c.single, kv_indptr=np.array(indptr, dtype=np.int32),
                                 kv_indices=np.concatenate(idx).astype(np.int32), last_page_len=last1)
    run_formats([c.prefix, s2], single, "c5 small, one suffix empty", mode)
    # both formats empty for every row: prefix without pages too
    p0 = dataclasses.replace(c.prefix, kv_indptr=np.array([0, 0], dtype=np.int32), kv_indices=np.zeros(0, dtype=np.int32),
                             last_page_len=np.array([0], dtype=np.int32))
    s0 = dataclasses.replace(s, kv_indptr=np.zeros(s.batch + 1, dtype=np.int32), kv_indices=np.zeros(0, dtype=np.int32),
                             last_page_len=np.zeros(s.batch, dtype=np.int32))
    single0 = dataclasses.replace(c.single, kv_indptr=np.zeros(s.batch + 1, dtype=np.int32),
                                  kv_indices=np.zeros(0, dtype=np.int32), last_page_len=np.zeros(s.batch, dtype=np.int32))
    o, lse = run_formats([p0, s0], single0, "every row empty", mode)
    assert (o == 0).all() and np.isneginf(lse.cpu().numpy()).all()


@pytest.mark.parametrize("mode", MODES)
def test_one_captured_run_serves_every_plan_over_two_formats(mode):
    """fi_run of a handle planned over two formats, captured once in a HIP graph (one attention launch + one
    contraction launch, no memset, no copy), replayed after re-planning other shared-prefix batches into the same
    workspace: every replay equals the eager run bit for bit and the oracle within tolerance."""
    import dataclasses
    import torch
    import paper_2501_01005_amd as fi
    c = workloads.config5(small=True)
    n = c.suffix.batch

    def variant(keep_prefix_pages, drop):
        """the case with a shorter prefix and some suffixes cut to one page"""
        p = dataclasses.replace(c.prefix, kv_indptr=np.array([0, keep_prefix_pages], dtype=np.int32),
                                kv_indices=c.prefix.kv_indices[:keep_prefix_pages].copy())
        n_pg = np.diff(c.suffix.kv_indptr).copy()
        last = c.suffix.last_page_len.copy()
        for i in drop:
            n_pg[i], last[i] = 1, 16
        ids = np.concatenate([c.suffix.kv_indices[c.suffix.kv_indptr[i]:c.suffix.kv_indptr[i] + n_pg[i]] for i in range(n)])
        s = dataclasses.replace(c.suffix, kv_indptr=np.concatenate([[0], np.cumsum(n_pg)]).astype(np.int32),
                                kv_indices=ids.astype(np.int32), last_page_len=last)
        idx, indptr = [], [0]
        for i in range(n):
            own = s.kv_indices[s.kv_indptr[i]:s.kv_indptr[i + 1]]
            idx += [p.kv_indices, own]
            indptr.append(indptr[-1] + len(p.kv_indices) + len(own))
        single = dataclasses.replace(c.single, kv_indptr=np.array(indptr, dtype=np.int32),
                                     kv_indices=np.concatenate(idx).astype(np.int32), last_page_len=last)
        return [p, s], single

    cases = [([c.prefix, c.suffix], c.single), variant(7, [0, 3]), variant(32, [1, 2, 5, 6]), ([c.prefix, c.suffix], c.single)]
    w = make_formats_wrapper([c.prefix, c.suffix], mode=mode, num_ctas=8 * 5, min_chunk=32)
    dev = DeviceBatch(c.prefix)
    H = c.prefix.num_qo_heads
    ids_dev = torch.zeros(len(c.prefix.kv_indices) + len(c.suffix.kv_indices), dtype=torch.int32, device="cuda:0")
    o = torch.zeros((n, H, 128), dtype=torch.float32, device="cuda:0")
    lse = torch.zeros((n, H), dtype=torch.float32, device="cuda:0")

    def load(batches):
        formats, ids = formats_of(batches)
        ids_dev[:len(ids)].copy_(torch.from_numpy(ids))
        o.fill_(float("nan"))
        lse.fill_(float("nan"))
        w.plan_formats(formats)

    load(cases[0][0])
    w.run(dev.q, dev.k_pool, dev.v_pool, ids_dev, c.prefix.sm_scale, o=o, lse=lse)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        w.run(dev.q, dev.k_pool, dev.v_pool, ids_dev, c.prefix.sm_scale, o=o, lse=lse)
    torch.cuda.synchronize()
    for rep, (batches, single) in enumerate(cases):
        print(f"[case] graph replay {rep} over two formats: prefix {int(batches[0].kv_lens()[0])} tokens, "
              f"suffixes {batches[1].kv_lens().tolist()}", flush=True)
        load(batches)
        w.run(dev.q, dev.k_pool, dev.v_pool, ids_dev, c.prefix.sm_scale, o=o, lse=lse)
        torch.cuda.synchronize()
        o_eager, lse_eager = o.clone(), lse.clone()
        o.fill_(float("nan"))
        lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o.view(torch.int32), o_eager.view(torch.int32)) and torch.equal(lse.view(torch.int32), lse_eager.view(torch.int32))
        o_ref, lse_ref = oracle.run_batch(single)
        e = assert_close(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, f"replay {rep}")
        print(f"[ok] replay {rep}: equals the eager run; err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    w.close()
