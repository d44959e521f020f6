"""GPU parity: the append / prefill path (plan -> MFMA tile kernel -> merge) and the
shared-prefix composition (Sec. 3.1.2) through the C ABI against the fp64 oracle."""
import numpy as np
import pytest

import oracle
import workloads
from oracle.plan_replica import plan_replica
from gpu_util import DeviceBatch, assert_close, make_wrapper, run_gpu

pytestmark = pytest.mark.gpu


def check(batch, what, **kw):
    print(f"[case] {what}: {batch.name} qo={batch.qo_lens()[:8].tolist()} kv={batch.kv_lens()[:8].tolist()} "
          f"causal={batch.causal} kw={kw}", flush=True)
    o_ref, lse_ref = oracle.run_batch(batch)
    o, lse = run_gpu(batch, "append", **kw)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)


def test_config3_small_causal_append():
    check(workloads.config3(small=True), "c3 small")
    check(workloads.config3(small=True), "c3 small split", num_ctas=8 * 16, min_chunk=32)


@pytest.mark.parametrize("seed", range(8))
def test_random_causal_and_full_batches(seed):
    g = [1, 2, 4, 8][seed % 4]
    dtype = workloads.F16 if seed % 2 else workloads.BF16
    causal = seed % 3 != 2
    b = workloads.random_case(200 + seed, dtype=dtype, num_qo_heads=2 * g, num_kv_heads=2, batch=2 + seed % 3,
                              max_qo=[5, 70, 300][seed % 3], max_kv=[90, 400, 700][seed % 3], causal=causal,
                              value_scale=[1.0, 0.5, 2.0][seed % 3])
    check(b, f"rand{seed}", num_ctas=2 * [1, 3, 16, 64][seed % 4], min_chunk=[16, 64][seed % 2])


def test_prefix_zero_and_tile_edges():
    # l_qo = l_kv (pure prefill), lengths around the 32-position tile and the 64-token KV tile
    for qo, kv in (([1], [1]), ([31], [31]), ([32], [32]), ([33], [33]), ([64], [64]), ([65], [129]), ([128, 1], [128, 700])):
        b = workloads.make_batch("edge", 9, workloads.BF16, 8, 2, 128, 16, qo, kv, True,
                                 num_pages=sum((k + 15) // 16 for k in kv) + 1)
        check(b, f"edge{qo}{kv}", num_ctas=2 * 4, min_chunk=16)


def test_more_queries_than_keys_gives_empty_rows():
    b = workloads.make_batch("short", 10, workloads.BF16, 8, 2, 128, 16, [40, 3], [25, 0], True, num_pages=4)
    check(b, "short kv", num_ctas=2 * 4, min_chunk=16)


def test_shared_prefix_composition_matches_single_format():
    import torch
    import paper_2501_01005_amd as fi
    c = workloads.config5(small=True)
    o_ref, lse_ref = oracle.run_batch(c.single)
    print("[case] c5 small: prefix pass (append tile kernel) + suffix pass (decode) + merge_state_pair", flush=True)
    dev_p, dev_s = DeviceBatch(c.prefix), DeviceBatch(c.suffix)
    wp = make_wrapper(c.prefix, "append", min_chunk=64)
    ws = make_wrapper(c.suffix, "decode")
    wp.plan(c.prefix.qo_indptr, c.prefix.kv_indptr, c.prefix.last_page_len, causal=False)
    ws.plan(c.suffix.qo_indptr, c.suffix.kv_indptr, c.suffix.last_page_len, causal=False)
    o_p, l_p = wp.run(dev_p.q, dev_p.k_pool, dev_p.v_pool, dev_p.kv_indices, c.prefix.sm_scale)
    o_s, l_s = ws.run(dev_s.q, dev_s.k_pool, dev_s.v_pool, dev_s.kv_indices, c.suffix.sm_scale)
    n_rows = o_p.shape[0] * o_p.shape[1]
    fi.fi_merge_state_pair(o_p, l_p, o_s, l_s, n_rows, 128, o_p, l_p, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    e = assert_close(o_p.double().cpu().numpy(), l_p.double().cpu().numpy(), o_ref, lse_ref, "c5 composed")
    print(f"[ok] c5 composed: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)
    # and the single-format decode of the same problem
    o1, l1 = run_gpu(c.single, "decode")
    assert_close(o1, l1, o_ref, lse_ref, "c5 single")
    wp.close(); ws.close()


def test_plan_for_append_equals_replica_with_default_grid():
    import paper_2501_01005_amd as fi
    b = workloads.config3(small=True)
    w = make_wrapper(b, "append")
    w.plan(b.qo_indptr, b.kv_indptr, b.last_page_len, causal=True)
    got = fi.fi_plan_view(w.handle)
    want = plan_replica(b.qo_indptr, b.kv_indptr, b.last_page_len, page_size=16, t_pos=64, group=4,
                        num_ctas=got["ctas_per_head"], causal=True, min_chunk=256)
    for k in ("cta_indptr", "w_q_row0", "w_n_pos", "w_kv_page0", "w_kv_start", "w_kv_len", "w_diag0", "w_out_slot"):
        assert got[k].tobytes() == np.asarray(want[k], dtype=np.int32).tobytes(), k
    w.close()


def test_bf16_v_outside_the_fp16_range_behaves_as_documented():
    """Append mode converts bf16 V to fp16 on its way into LDS (include/fi355.h, fi_run): exact for
    2^-14 <= |v| <= 65504, larger magnitudes become +-65504, smaller ones are rounded toward zero to a multiple of
    2^-24.  Every V row of a request holds the same vector here, so that o equals that vector whatever the
    softmax weights are: the oracle on the in-range columns, the documented conversion on the others."""
    b = workloads.make_batch("vrange", 77, workloads.BF16, 8, 2, 128, 16, [200, 20], [300, 50], True, num_pages=24,
                             poison=False)
    special = np.array([65280.0, 65536.0, 99840.0, -65536.0, -3.0e38, 2.0 ** -14, 2.0 ** -20, 2.0 ** -20 * (1 + 1 / 128),
                        -(2.0 ** -15) * 1.5, 3 * 2.0 ** -26, 1.0, -2.5, 1000.0, 2.0 ** -24, 0.0, 6.1e-5], dtype=np.float32)
    vstar = np.tile(special, 128 // len(special))
    bits = workloads.f32_to_bits(vstar, workloads.BF16)
    vstar = workloads.widen(bits, workloads.BF16)                      # what the cache really holds
    b.v_bits[:] = bits[None, None, None, :]
    # documented conversion: clamp, then toward zero onto the fp16 grid (spacing 2^-24 below 2^-14)
    clamped = np.clip(vstar, -65504.0, 65504.0)
    with np.errstate(divide="ignore"):
        ulp = np.exp2(np.maximum(np.floor(np.log2(np.abs(clamped))), -14.0) - 10.0)
    expected = np.where(clamped == 0, 0.0, np.trunc(clamped / ulp) * ulp)
    in_range = (np.abs(vstar) >= 2.0 ** -14) & (np.abs(vstar) <= 65504.0) | (vstar == 0)
    assert np.array_equal(expected[in_range], vstar[in_range]) and (~in_range).sum() >= 40
    print(f"[case] bf16 V outside the fp16 range: {b.name}, {(~in_range).sum()} of 128 columns out of range", flush=True)
    o_ref, lse_ref = oracle.run_batch(b)
    assert np.allclose(o_ref[..., in_range], vstar[in_range], rtol=1e-12, atol=0)   # a convex combination of equal rows
    for kw in (dict(num_ctas=2 * 4, min_chunk=16), dict()):       # both paths: short chunks and the scheduled loop
        o, lse = run_gpu(b, "append", **kw)
        assert not np.isnan(o).any()
        assert np.abs(lse - lse_ref).max() <= 1e-3
        # fp32 accumulation over up to 300 keys: 1e-5 relative; for the values on the 2^-24 grid a thousandth of a step
        excess = np.abs(o - expected) - (1e-5 * np.abs(expected) + 1e-3 * 2.0 ** -24)
        small = np.abs(vstar) < 2.0 ** -14
        print(f"[ok] kw={kw}: deviation from the documented conversion: max relative {np.abs(o / np.where(expected == 0, 1, expected) - 1)[..., expected != 0].max():.2e}, "
              f"max |o - v| on the columns below 2^-14: {np.abs(o - vstar)[..., small].max():.2e}", flush=True)
        assert excess.max() <= 0, excess.max()
        assert np.abs(o - vstar)[..., small].max() < 2.0 ** -24
