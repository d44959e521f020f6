"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times
(library-default grid and chunk size).  Every output element of every request is compared with
the fp64 oracle (the long-context workload has two requests, both compared)."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, assert_close, make_wrapper, run_gpu

pytestmark = pytest.mark.gpu


def sampled_check(batch, mode, requests, what, **kw):
    print(f"[case] {what}: {batch.name} batch={batch.batch} tokens={int(batch.kv_lens().sum())} sample={list(requests)}",
          flush=True)
    o, lse = run_gpu(batch, mode, **kw)
    assert not np.isnan(o).any() and not np.isnan(lse).any(), "NaN in GPU output"
    o_ref, lse_ref = oracle.run_batch(batch, requests=requests)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)


def test_config2_full_gqa_decode_zipf():
    # the benchmarked workload: all 128 requests, i.e. every row that the 256 CTAs per kv head and the merge of
    # the split tiles write
    b = workloads.config2()
    sampled_check(b, "decode", list(range(b.batch)), "c2 full")


def test_config4_full_long_context_decode():
    b = workloads.config4()
    sampled_check(b, "decode", [0, 1], "c4 full")


def test_config4_full_with_the_contraction_inside_the_launch():
    # 171 and 86 partial states per request, written by wavefronts on every XCD and folded by whichever comes last
    sampled_check(workloads.config4(), "decode", [0, 1], "c4 full, merge = 2", merge=2)


def test_config2_full_with_8_bit_kv_cache():
    b = workloads.config2(kv_dtype=workloads.FP8)
    sampled_check(b, "decode", list(range(b.batch)), "c2 full, E4M3 K/V")


def test_config4_full_with_8_bit_kv_cache():
    sampled_check(workloads.config4(kv_dtype=workloads.FP8), "decode", [0, 1], "c4 full, E4M3 K/V")


def test_config3_full_causal_append():
    b = workloads.config3()
    # every request: each CTA's queue of work items is then checked end to end, seams included
    sampled_check(b, "append", list(range(b.batch)), "c3 full")


@pytest.mark.parametrize("mode", ["tile16", "tile64"])
def test_full_decode_and_append_batches_through_the_tile_modes(mode):
    """The benchmark's decode and causal-append batches through the 16-row and 64-row tile kernels at the library's
    default grid: one-position tiles with long split chunks (a 32 768-token request), and tiles of 16 / g and 64 / g
    positions over 16 requests of 128..1 024 new tokens (hundreds of work items per CTA queue); a sample of requests
    against the oracle, every row checked for NaN."""
    b = workloads.config2()
    sampled_check(b, mode, [0, 1, 5, 17, 64, 127], f"c2 full as {mode}")
    b = workloads.config3()
    sampled_check(b, mode, [0, 1, 2, 9, 15], f"c3 full as {mode}")
    b = workloads.config3(page_size=32)
    sampled_check(b, "append", [1, 2, 7, 12], "c3 full, page size 32 (the scheduled loop's page-size variant)")


def test_config5_full_shared_prefix():
    import torch
    import paper_2501_01005_amd as fi
    c = workloads.config5()
    print("[case] c5 full: composed (prefix append pass + suffix decode pass + pair merge) and single format", flush=True)
    o_ref, lse_ref = oracle.run_batch(c.single)
    dev_p, dev_s = DeviceBatch(c.prefix), DeviceBatch(c.suffix)
    wp, ws = make_wrapper(c.prefix, "append"), make_wrapper(c.suffix, "decode")
    wp.plan(c.prefix.qo_indptr, c.prefix.kv_indptr, c.prefix.last_page_len, causal=False)
    ws.plan(c.suffix.qo_indptr, c.suffix.kv_indptr, c.suffix.last_page_len, causal=False)
    o_p, l_p = wp.run(dev_p.q, dev_p.k_pool, dev_p.v_pool, dev_p.kv_indices, c.prefix.sm_scale)
    o_s, l_s = ws.run(dev_s.q, dev_s.k_pool, dev_s.v_pool, dev_s.kv_indices, c.suffix.sm_scale)
    fi.fi_merge_state_pair(o_p, l_p, o_s, l_s, o_p.shape[0] * o_p.shape[1], 128, o_p, l_p,
                           torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    e = assert_close(o_p.double().cpu().numpy(), l_p.double().cpu().numpy(), o_ref, lse_ref, "c5 composed")
    # the same composition with one contraction launch for both passes: the same bits
    o_c, l_c = wp.run_composed(ws, dev_p.q, dev_p.k_pool, dev_p.v_pool, dev_p.kv_indices, dev_s.kv_indices, c.prefix.sm_scale)
    torch.cuda.synchronize()
    assert torch.equal(o_c.view(torch.int32), o_p.view(torch.int32)) and torch.equal(l_c.view(torch.int32), l_p.view(torch.int32))
    o1, l1 = run_gpu(c.single, "decode")
    e1 = assert_close(o1, l1, o_ref, lse_ref, "c5 single")
    print(f"[ok] c5 full: composed err_o={e[0]:.2e} err_lse={e[1]:.2e}; single err_o={e1[0]:.2e}", flush=True)
    wp.close(); ws.close()


@pytest.mark.parametrize("kind", ["decode", "prefill"])
@pytest.mark.parametrize("dist", ["constant", "uniform", "zipf"])
def test_input_dynamism_workloads(kind, dist):
    """Batch 16 with constant, uniform and skewed lengths, decode and causal prefill (Sec. 4.2's kernel experiment)."""
    b = workloads.config_e2(kind, dist)
    sampled_check(b, "decode" if kind == "decode" else "append", list(range(b.batch)), f"e2 {kind} {dist}")
