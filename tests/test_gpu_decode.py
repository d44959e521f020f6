"""GPU parity: the decode path (plan -> persistent decode kernel -> merge of split
chunks) through the C ABI against the fp64 oracle, element by element."""
import dataclasses

import numpy as np
import pytest

import oracle
import workloads
from oracle.plan_replica import plan_replica
from gpu_util import DeviceBatch, assert_close, make_wrapper, run_gpu

pytestmark = pytest.mark.gpu


def check(batch, what, **kw):
    print(f"[case] {what}: {batch.name} kv_lens={batch.kv_lens()[:8].tolist()} kw={kw}", flush=True)
    o_ref, lse_ref = oracle.run_batch(batch)
    o, lse = run_gpu(batch, "decode", **kw)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)


def test_config1_mha_decode_fp16():
    check(workloads.config1(), "c1")


def test_config1_split_into_many_chunks():
    check(workloads.config1(), "c1 split", num_ctas=8 * 40, min_chunk=16)


def test_config2_small_gqa_decode_bf16():
    check(workloads.config2(small=True), "c2 small")
    check(workloads.config2(small=True), "c2 small split", num_ctas=8 * 64, min_chunk=32)


def test_config4_small_long_context_split():
    check(workloads.config4(small=True), "c4 small")


@pytest.mark.parametrize("seed", range(8))
def test_random_ragged_batches(seed):
    g = [1, 2, 4, 4][seed % 4]
    dtype = workloads.F16 if seed % 2 else workloads.BF16
    b = workloads.random_case(100 + seed, dtype=dtype, num_qo_heads=2 * g, num_kv_heads=2, batch=3 + seed,
                              max_kv=[40, 300, 1000][seed % 3], value_scale=[1.0, 0.5, 2.0][seed % 3])
    check(b, f"rand{seed}", num_ctas=2 * [1, 3, 16, 64][seed % 4], min_chunk=[16, 64][seed % 2])


def test_single_token_and_exact_page_multiples():
    for kv in ([1], [16], [32], [33], [15, 17, 31, 48, 64, 65]):
        b = workloads.make_batch("edge", 7, workloads.BF16, 8, 2, 128, 16, [1] * len(kv), kv, False,
                                 num_pages=sum((k + 15) // 16 for k in kv) + 2)
        check(b, f"edge{kv}", num_ctas=2 * 4, min_chunk=16)


def test_all_requests_empty():
    b = workloads.make_batch("empty", 8, workloads.BF16, 8, 2, 128, 16, [1, 1], [0, 0], False, num_pages=2)
    o, lse = run_gpu(b, "decode", num_ctas=8)
    assert np.array_equal(o, np.zeros_like(o)) and np.isneginf(lse).all()


def test_strided_pool_layout_gives_identical_bits():
    b = workloads.config2(small=True)
    o1, l1 = run_gpu(b, "decode", dev=DeviceBatch(b, kv_layout="HND"))
    o2, l2 = run_gpu(b, "decode", dev=DeviceBatch(b, kv_layout="NHD"))
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_rerun_is_bit_identical_and_cast_output_is_the_rounded_output():
    import torch
    b = workloads.config2(small=True)
    dev = DeviceBatch(b)
    w = make_wrapper(b, "decode", num_ctas=8 * 32, min_chunk=64)
    o1, l1, c1 = run_gpu(b, "decode", dev=dev, wrapper=w, with_cast=True)
    o2, l2, c2 = run_gpu(b, "decode", dev=dev, wrapper=w, with_cast=True)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2) and np.array_equal(c1, c2)
    want = torch.from_numpy(o1).float().to(torch.bfloat16).double().numpy()
    assert np.array_equal(c1, want)
    w.close()


def test_plan_on_device_box_equals_replica_with_default_grid():
    import paper_2501_01005_amd as fi
    b = workloads.config2(small=True)
    w = make_wrapper(b, "decode")                      # num_ctas = 0 -> library default for this GPU
    w.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=False)
    got = fi.fi_plan_view(w.handle)
    want = plan_replica(b.qo_indptr, b.kv_indptr, b.last_page_len, page_size=16, t_pos=1, group=4,
                        num_ctas=got["ctas_per_head"], causal=False, min_chunk=32, item_cost=64)
    for k in ("cta_indptr", "w_q_row0", "w_kv_page0", "w_kv_start", "w_kv_len", "w_out_slot", "m_slot_base", "m_n_chunks"):
        assert got[k].tobytes() == np.asarray(want[k], dtype=np.int32).tobytes(), k
    w.close()


def test_permuted_pool_gives_identical_bits():
    b = workloads.config2(small=True)
    rng = np.random.default_rng(5)
    perm = rng.permutation(b.num_pages)
    k2 = np.empty_like(b.k_bits); v2 = np.empty_like(b.v_bits)
    k2[perm] = b.k_bits; v2[perm] = b.v_bits
    b2 = dataclasses.replace(b, k_bits=k2, v_bits=v2, kv_indices=perm[b.kv_indices].astype(np.int32))
    o1, l1 = run_gpu(b, "decode")
    o2, l2 = run_gpu(b2, "decode")
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


@pytest.mark.parametrize("dtype,g", [(workloads.BF16, 4), (workloads.F16, 1), (workloads.BF16, 2)])
def test_contraction_inside_the_attention_launch(dtype, g):
    """fi_config.merge = 2 (Sec. 3.3.1: one launch): the wavefront that delivers a split tile's last partial state
    folds them all.  Many chunks per request, spread over all CUs; two runs with one plan (the arrival counters must
    be back at zero), then a new plan; the rounded copy of the output is written by the folding wavefront too."""
    import torch
    b = workloads.make_batch("fold", 95 + g, dtype, 2 * g, 2, 128, 16, [1] * 5, [3000, 700, 40, 1, 0], False)
    o_ref, lse_ref = oracle.run_batch(b)
    dev = DeviceBatch(b)
    w = make_wrapper(b, "decode", merge=2, min_chunk=32)
    for rep in range(3):
        print(f"[case] fold in launch: g={g} {dtype} rep={rep}", flush=True)
        if rep != 1:
            w.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=False)
        o = torch.full((5, 2 * g, 128), float("nan"), dtype=torch.float32, device=dev.device)
        lse = torch.full((5, 2 * g), float("nan"), dtype=torch.float32, device=dev.device)
        oc = torch.zeros((5, 2 * g, 128), dtype=dev.q.dtype, device=dev.device)
        w.run(dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, b.sm_scale, o=o, lse=lse, o_cast=oc)
        torch.cuda.synchronize()
        e = assert_close(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, f"fold rep {rep}")
        ulp = 2.0 ** -8 if dtype == workloads.BF16 else 2.0 ** -11
        assert np.all(np.abs(oc.double().cpu().numpy() - o.double().cpu().numpy())
                      <= np.maximum(np.abs(o.double().cpu().numpy()), 2.0 ** -14) * ulp)
        print(f"[ok] fold rep {rep}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    view = __import__("paper_2501_01005_amd").fi_plan_view(w.handle)
    assert int(view["n_merge"]) >= 2 and max(view["m_n_chunks"]) > 16
    w.close()


@pytest.mark.parametrize("g", [8, 16])
@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
def test_wide_head_groups(g, dtype):
    """8 and 16 query heads per kv head (the fused tile's 16 columns half or completely filled): split and unsplit
    chunks, the 8-bit KV cache, another page size, the variants with the rotary embedding."""
    import torch
    b = workloads.random_case(300 + g, dtype=dtype, num_qo_heads=2 * g, num_kv_heads=2, batch=5, max_kv=600, value_scale=2.0)
    check(b, f"g={g} {dtype}", num_ctas=2 * 16, min_chunk=32)
    check(b, f"g={g} {dtype}, unsplit", num_ctas=2 * 2, min_chunk=1024)
    b8 = workloads.random_case(310 + g, dtype=dtype, num_qo_heads=2 * g, num_kv_heads=2, batch=5, max_kv=600,
                               kv_dtype=workloads.FP8, k_scale=0.5, v_scale=2.0)
    check(b8, f"g={g} {dtype}, 8-bit KV", num_ctas=2 * 16, min_chunk=32)
    bp = workloads.random_case(320 + g, dtype=dtype, num_qo_heads=2 * g, num_kv_heads=2, batch=5, max_kv=600, page_size=4)
    check(bp, f"g={g} {dtype}, page size 4", num_ctas=2 * 16, min_chunk=32)
    # variants: through the wrapper directly
    dev = DeviceBatch(b)
    w = make_wrapper(b, "decode", num_ctas=2 * 16, min_chunk=32)
    w.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=False)
    var = dict(kv_indptr=torch.from_numpy(np.ascontiguousarray(b.kv_indptr, dtype=np.int32)).to(dev.device),
               last_page_len=torch.from_numpy(np.ascontiguousarray(b.last_page_len, dtype=np.int32)).to(dev.device),
               logits_soft_cap=6.0, window_left=200, rope_theta=1e4,
               alibi_slopes=torch.tensor([2.0 ** (-(i + 1) * 8.0 / (2 * g)) for i in range(2 * g)], dtype=torch.float32,
                                         device=dev.device))
    o, lse = w.run(dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, b.sm_scale, variant=var)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.run_batch(b, logits_soft_cap=6.0, window_left=200, rope_theta=1e4,
                                      alibi_slopes=np.array([2.0 ** (-(i + 1) * 8.0 / (2 * g)) for i in range(2 * g)]))
    assert_close(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, f"g={g} variants")
    w.close()
