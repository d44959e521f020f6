"""One captured launch of `run` serves every batch: the grid, the kernel arguments and the workspace
sections depend only on the configuration, never on the request lengths (Sec. 3.3.1 on the fixed
grid of the persistent kernel; App. D.1 on the fixed workspace sections).  The test captures
`run` once in a HIP graph, then re-plans different batches into the same workspace and replays
the graph, with eager work and synchronisations in between, checking every replay against the
oracle and against the eager launch of the same batch bit for bit."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import assert_close, bits_to_torch

pytestmark = pytest.mark.gpu

HQ, HKV, D, PS = 8, 2, 128, 16
POOL_PAGES = 160


def _batches(mode):
    if mode == "decode":
        shapes = [([1] * 5, [700, 33, 1, 260, 129]), ([1] * 2, [2000, 17]), ([1] * 6, [64, 0, 65, 500, 16, 301]),
                  ([1] * 5, [700, 33, 1, 260, 129])]
        causal = False
    else:
        shapes = [([70, 9, 130], [400, 9, 260]), ([200], [1500]), ([1, 64, 65, 3], [300, 64, 500, 3]),
                  ([70, 9, 130], [400, 9, 260])]
        causal = True
    return [workloads.make_batch(f"graph_{mode}_{i}", 900 + 7 * i, workloads.BF16, HQ, HKV, D, PS, qo, kv, causal,
                                 num_pages=POOL_PAGES) for i, (qo, kv) in enumerate(shapes)]


@pytest.mark.parametrize("mode", ["decode", "append", "decode, contraction inside the launch"])
def test_one_captured_run_serves_every_plan(mode):
    import torch
    import paper_2501_01005_amd as fi

    dev = torch.device("cuda:0")
    merge = 2 if "inside" in mode else 0   # then the captured graph holds one kernel, and its arrival counters
    mode = mode.split(",")[0]              # must be back at zero after every replay
    batches = _batches(mode)
    t_pos = 1 if mode == "decode" else 256 // (HQ // HKV)
    max_batch = max(b.batch for b in batches)
    max_tiles = max(int(sum(-(-int(l) // t_pos) for l in b.qo_lens())) for b in batches)
    nnz_max = max(int(b.qo_indptr[-1]) for b in batches)
    idx_max = max(len(b.kv_indices) for b in batches)
    # few CTAs and a small minimum chunk: long requests are split, so the replays also cover partial slots and merge
    w = fi.PagedAttention(dtype=workloads.BF16, num_qo_heads=HQ, num_kv_heads=HKV, head_dim=D, page_size=PS, mode=mode,
                          max_batch=max_batch, max_qo_tiles=max_tiles, num_ctas=HKV * 6, min_chunk=128, merge=merge)
    q_s = torch.zeros((nnz_max, HQ, D), dtype=torch.bfloat16, device=dev)
    k_s = torch.zeros((POOL_PAGES, HKV, PS, D), dtype=torch.bfloat16, device=dev)
    v_s = torch.zeros_like(k_s)
    idx_s = torch.zeros(max(idx_max, 1), dtype=torch.int32, device=dev)
    o_s = torch.zeros((nnz_max, HQ, D), dtype=torch.float32, device=dev)
    lse_s = torch.zeros((nnz_max, HQ), dtype=torch.float32, device=dev)
    sm_scale = batches[0].sm_scale

    def load(b):
        nnz = int(b.qo_indptr[-1])
        q_s[:nnz].copy_(bits_to_torch(b.q_bits, b.dtype, dev))
        k_s.copy_(bits_to_torch(b.k_bits, b.dtype, dev))
        v_s.copy_(bits_to_torch(b.v_bits, b.dtype, dev))
        if len(b.kv_indices):
            idx_s[:len(b.kv_indices)].copy_(torch.from_numpy(np.ascontiguousarray(b.kv_indices, dtype=np.int32)))
        o_s.fill_(float("nan"))
        lse_s.fill_(float("nan"))
        w.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=b.causal)
        return nnz

    # eager once (also loads the code objects), then the capture
    load(batches[0])
    w.run(q_s, k_s, v_s, idx_s, sm_scale, o=o_s, lse=lse_s)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        w.run(q_s, k_s, v_s, idx_s, sm_scale, o=o_s, lse=lse_s)
    torch.cuda.synchronize()

    for rep, b in enumerate(batches):
        print(f"[case] graph replay {rep}: {b.name} qo={b.qo_lens().tolist()} kv={b.kv_lens().tolist()}", flush=True)
        o_ref, lse_ref = oracle.run_batch(b)
        nnz = load(b)
        w.run(q_s, k_s, v_s, idx_s, sm_scale, o=o_s, lse=lse_s)
        torch.cuda.synchronize()
        o_eager, lse_eager = o_s[:nnz].clone(), lse_s[:nnz].clone()
        o_s.fill_(float("nan"))
        lse_s.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_s[:nnz].view(torch.int32), o_eager.view(torch.int32)), f"replay {rep}: o differs from eager"
        assert torch.equal(lse_s[:nnz].view(torch.int32), lse_eager.view(torch.int32)), f"replay {rep}: lse differs"
        e = assert_close(o_s[:nnz].double().cpu().numpy(), lse_s[:nnz].double().cpu().numpy(), o_ref, lse_ref,
                         f"replay {rep}")
        print(f"[ok] replay {rep}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    w.close()


def test_one_captured_composed_run_serves_every_plan():
    """fi_run_composed under capture: two decode formats over the same five query rows (each request's pages cut in
    two), both re-planned between the replays; the launch geometry depends on the configuration and on the number
    of query rows only."""
    import torch
    import paper_2501_01005_amd as fi

    dev = torch.device("cuda:0")
    shapes = [[700, 33, 1, 260, 129], [64, 0, 500, 16, 301], [1500, 17, 5, 600, 40], [700, 33, 1, 260, 129]]
    batches = [workloads.make_batch(f"graph_comp_{i}", 950 + i, workloads.BF16, HQ, HKV, D, PS, [1] * 5, kv, False,
                                    num_pages=POOL_PAGES) for i, kv in enumerate(shapes)]
    mk = lambda: fi.PagedAttention(dtype=workloads.BF16, num_qo_heads=HQ, num_kv_heads=HKV, head_dim=D, page_size=PS,
                                   mode="decode", max_batch=5, max_qo_tiles=5, num_ctas=HKV * 6, min_chunk=64)
    wa, wb = mk(), mk()
    q_s = torch.zeros((5, HQ, D), dtype=torch.bfloat16, device=dev)
    k_s = torch.zeros((POOL_PAGES, HKV, PS, D), dtype=torch.bfloat16, device=dev)
    v_s = torch.zeros_like(k_s)
    ia_s = torch.zeros(POOL_PAGES, dtype=torch.int32, device=dev)
    ib_s = torch.zeros(POOL_PAGES, dtype=torch.int32, device=dev)
    o_s = torch.zeros((5, HQ, D), dtype=torch.float32, device=dev)
    lse_s = torch.zeros((5, HQ), dtype=torch.float32, device=dev)
    sm_scale = batches[0].sm_scale

    def load(b):
        ia, ib, pa, pb, la, lb = [], [], [0], [0], [], []
        for r in range(b.batch):
            pages = b.kv_indices[b.kv_indptr[r]:b.kv_indptr[r + 1]]
            k = len(pages) // 2
            ia.append(pages[:k]); ib.append(pages[k:])
            pa.append(pa[-1] + k); pb.append(pb[-1] + len(pages) - k)
            la.append(16 if k > 0 else 1)
            lb.append(int(b.last_page_len[r]) if len(pages) > k else 1)
        for dst, parts in ((ia_s, ia), (ib_s, ib)):
            flat = np.concatenate(parts).astype(np.int32) if parts else np.zeros(0, dtype=np.int32)
            if len(flat):
                dst[:len(flat)].copy_(torch.from_numpy(flat))
        q_s.copy_(bits_to_torch(b.q_bits, b.dtype, dev))
        k_s.copy_(bits_to_torch(b.k_bits, b.dtype, dev))
        v_s.copy_(bits_to_torch(b.v_bits, b.dtype, dev))
        o_s.fill_(float("nan")); lse_s.fill_(float("nan"))
        wa.plan(b.qo_indptr, np.asarray(pa, dtype=np.int32), np.asarray(la, dtype=np.int32), causal=False)
        wb.plan(b.qo_indptr, np.asarray(pb, dtype=np.int32), np.asarray(lb, dtype=np.int32), causal=False)

    load(batches[0])
    wa.run_composed(wb, q_s, k_s, v_s, ia_s, ib_s, sm_scale, o=o_s, lse=lse_s)   # eager once: code objects, pass rows
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        wa.run_composed(wb, q_s, k_s, v_s, ia_s, ib_s, sm_scale, o=o_s, lse=lse_s)
    torch.cuda.synchronize()
    for rep, b in enumerate(batches):
        print(f"[case] composed graph replay {rep}: kv={b.kv_lens().tolist()}", flush=True)
        load(b)
        graph.replay()
        torch.cuda.synchronize()
        o_g, l_g = o_s.clone(), lse_s.clone()
        o_ref, lse_ref = oracle.run_batch(b)
        assert_close(o_g.double().cpu().numpy(), l_g.double().cpu().numpy(), o_ref, lse_ref, f"composed replay {rep}")
        o_s.fill_(float("nan")); lse_s.fill_(float("nan"))
        wa.run_composed(wb, q_s, k_s, v_s, ia_s, ib_s, sm_scale, o=o_s, lse=lse_s)
        torch.cuda.synchronize()
        assert torch.equal(o_g.view(torch.int32), o_s.view(torch.int32)) and torch.equal(l_g.view(torch.int32), lse_s.view(torch.int32))
    wa.close(); wb.close()
