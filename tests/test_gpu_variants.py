"""GPU parity of decode and causal append with attention variants (Sec. 3.2.3: soft cap of the logits, ALiBi
bias, sliding window; decode also the fused rotary embedding) against the oracle: each variant alone, all
together, windows that hide whole steps and whole split chunks (whose partial state is then the identity of
the merge), both query types."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import DeviceBatch, assert_close, make_wrapper

pytestmark = pytest.mark.gpu


def run_variant(batch, num_ctas=0, min_chunk=0, mode="decode", plan_window=0, merge=0, dev=None, **var):
    import torch
    dev = dev or DeviceBatch(batch)
    w = make_wrapper(batch, mode, num_ctas=num_ctas, min_chunk=min_chunk, plan_window=plan_window, merge=merge)
    w.plan(batch.qo_indptr, batch.kv_indptr, batch.last_page_len, causal=batch.causal)
    nnz = dev.q.shape[0]
    o = torch.full((nnz, batch.num_qo_heads, batch.head_dim), float("nan"), dtype=torch.float32, device=dev.device)
    lse = torch.full((nnz, batch.num_qo_heads), float("nan"), dtype=torch.float32, device=dev.device)
    v = dict(kv_indptr=torch.from_numpy(np.ascontiguousarray(batch.kv_indptr, dtype=np.int32)).to(dev.device),
             last_page_len=torch.from_numpy(np.ascontiguousarray(batch.last_page_len, dtype=np.int32)).to(dev.device))
    if "alibi_slopes" in var:
        v["alibi_slopes"] = torch.from_numpy(np.asarray(var["alibi_slopes"], dtype=np.float32)).to(dev.device)
    v.update({k: var[k] for k in ("logits_soft_cap", "window_left", "rope_theta", "rope_scale") if k in var})
    w.run(dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, batch.sm_scale, o=o, lse=lse, variant=v)
    torch.cuda.synchronize()
    w.close()
    return o.double().cpu().numpy(), lse.double().cpu().numpy()


def check(batch, what, num_ctas=0, min_chunk=0, mode="decode", plan_window=0, merge=0, **var):
    print(f"[case] {what}: {batch.name} {mode} dtype={batch.dtype} heads={batch.num_qo_heads}/{batch.num_kv_heads} "
          f"qo={batch.qo_lens()[:8].tolist()} kv={batch.kv_lens()[:8].tolist()} "
          f"variant={ {k: (v if np.isscalar(v) else 'array') for k, v in var.items()} }", flush=True)
    o_ref, lse_ref = oracle.run_batch(batch, **var)
    o, lse = run_variant(batch, num_ctas=num_ctas, min_chunk=min_chunk, mode=mode, plan_window=plan_window, merge=merge,
                         **var)
    e = assert_close(o, lse, o_ref, lse_ref, what)
    print(f"[ok] {what}: err_o={e[0]:.2e} err_lse={e[1]:.2e}", flush=True)


def slopes(h):
    return np.array([2.0 ** (-(i + 1) * 8.0 / h) for i in range(h)])


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
@pytest.mark.parametrize("g", [1, 4])
def test_each_variant_and_all_together(dtype, g):
    b = workloads.random_case(400 + g, dtype=dtype, num_qo_heads=2 * g, num_kv_heads=2, batch=6, max_kv=500,
                              value_scale=2.0)
    check(b, "no variant in effect", logits_soft_cap=0.0, window_left=-1)
    check(b, "soft cap", logits_soft_cap=3.0)
    check(b, "alibi", alibi_slopes=slopes(2 * g))
    check(b, "window", window_left=70)
    check(b, "all", logits_soft_cap=5.0, window_left=33, alibi_slopes=slopes(2 * g))


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
def test_fused_rotary_embedding(dtype):
    """Keys are stored unrotated; the kernel rotates key t by t and the query by l_kv - 1 (Sec. 4.3's fused
    kernel).  Short and long requests, split chunks (a chunk's first token is not token 0), positions beyond
    65536 (where a single-precision angle would have lost its low bits), a position divisor, other variants on top."""
    b = workloads.random_case(430, dtype=dtype, num_qo_heads=8, num_kv_heads=2, batch=6, max_kv=700, value_scale=1.0)
    check(b, "rope", rope_theta=1e4)
    check(b, "rope, split chunks", num_ctas=2 * 16, min_chunk=32, rope_theta=1e4)
    check(b, "rope, other base and divisor", rope_theta=5e5, rope_scale=4.0)
    check(b, "rope + cap + window + alibi", rope_theta=1e4, logits_soft_cap=4.0, window_left=100, alibi_slopes=slopes(8))
    far = workloads.make_batch("far", 431, dtype, 4, 1, 128, 16, [1, 1, 1], [70000, 1, 255], False, poison=False)
    check(far, "rope at positions up to 70000", rope_theta=1e4)


def test_window_hides_whole_steps_and_whole_chunks():
    # long requests split into many chunks; a short window leaves most chunks without a visible token
    b = workloads.make_batch("win", 410, workloads.BF16, 8, 2, 128, 16, [1, 1, 1, 1], [3000, 700, 40, 1], False)
    for W in (0, 1, 31, 32, 100, 5000):
        check(b, f"window {W}", num_ctas=2 * 16, min_chunk=64, window_left=W)
    # the same with the partial states folded inside the launch: most of them are empty (lse = -inf)
    for W in (0, 100):
        check(b, f"window {W}, contraction inside the launch", num_ctas=2 * 16, min_chunk=64, window_left=W, merge=2)
    check(b, "rope, contraction inside the launch", num_ctas=2 * 16, min_chunk=64, rope_theta=1e4, merge=2)


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
@pytest.mark.parametrize("g", [1, 4])
def test_causal_append_with_variants(dtype, g):
    """Query tiles of several positions: every row has its own position, so bias and window differ from row to
    row; chunks long enough for the scheduled loop run on the general path with ALiBi or a window; split chunks; a window that
    hides whole tiles and, for the early rows of a split tile, whole chunks."""
    qo = [70, 9, 130, 1, 64]
    kv = [400, 9, 260, 300, 64]
    b = workloads.make_batch("appvar", 440 + g, dtype, 2 * g, 2, 128, 16, qo, kv, True)
    kw = dict(mode="append", num_ctas=2 * 4, min_chunk=1024)
    check(b, "append, no variant in effect", logits_soft_cap=0.0, window_left=-1, **kw)
    check(b, "append, soft cap", logits_soft_cap=3.0, **kw)
    check(b, "append, alibi", alibi_slopes=slopes(2 * g), **kw)
    check(b, "append, window", window_left=50, **kw)
    check(b, "append, all", logits_soft_cap=5.0, window_left=33, alibi_slopes=slopes(2 * g), **kw)
    check(b, "append, all, split chunks", logits_soft_cap=5.0, window_left=100, alibi_slopes=slopes(2 * g),
          mode="append", num_ctas=2 * 16, min_chunk=64)


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
@pytest.mark.parametrize("g", [1, 4, 16])
def test_soft_cap_inside_the_scheduled_append_loop(dtype, g):
    """The soft cap alone has a variant of the append kernel's scheduled loop (the other hooks run on the general
    path): one CTA per kv head walks items of both paths (seams, idle wavefronts, chunks that end inside a tile,
    tiles cut by the diagonal); a cap that bites hard with large logits (the reference is raised on the capped
    values) and one that barely does; split chunks."""
    qo = [64, 3, 64, 130, 1, 64, 40, 64, 64, 7, 200]
    kv = [300, 50, 128, 700, 100, 129, 140, 64, 191, 400, 260]
    for scale, cap in ((3.0, 2.0), (1.0, 30.0)):
        b = workloads.make_batch("caploop", 460 + g, dtype, 2 * g, 2, 128, 16, qo, kv, True, value_scale=scale)
        check(b, f"append loop, soft cap {cap}, one CTA per head", mode="append", num_ctas=2, min_chunk=1024, logits_soft_cap=cap)
    check(b, "append loop, soft cap, split chunks", mode="append", num_ctas=2 * 16, min_chunk=128, logits_soft_cap=4.0)


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
@pytest.mark.parametrize("g", [1, 4, 16])
def test_bias_and_window_inside_the_scheduled_append_loop(dtype, g):
    """ALiBi and the sliding window (without the soft cap) have a variant of the append kernel's scheduled loop too:
    one CTA per kv head walks items of both paths; steep and flat slopes with large logits (the reference is raised
    on the biased values); windows that hide whole steps, whole tiles and, in split tiles, whole chunks from some
    rows (their partial state is the empty one) or from every row of a wavefront; windows wider than the context;
    with and without the window in the plan."""
    qo = [64, 3, 64, 130, 1, 64, 40, 64, 64, 7, 200]
    kv = [300, 50, 128, 700, 100, 129, 140, 64, 191, 400, 260]
    one_cta = dict(mode="append", num_ctas=2, min_chunk=1024)
    for scale in (3.0, 1.0):
        b = workloads.make_batch("varloop", 470 + g, dtype, 2 * g, 2, 128, 16, qo, kv, True, value_scale=scale)
        check(b, f"append loop, alibi, value scale {scale}", alibi_slopes=slopes(2 * g), **one_cta)
        check(b, f"append loop, steep alibi, value scale {scale}", alibi_slopes=8.0 * slopes(2 * g), **one_cta)
    for W in (0, 7, 40, 64, 150, 100000):
        check(b, f"append loop, window {W}", window_left=W, **one_cta)
    check(b, "append loop, alibi + window", alibi_slopes=slopes(2 * g), window_left=90, **one_cta)
    for W in (10, 130):
        check(b, f"append loop, window {W}, split chunks", mode="append", num_ctas=2 * 16, min_chunk=128, window_left=W)
        check(b, f"append loop, planned window {W}, alibi", mode="append", num_ctas=2 * 8, min_chunk=128, plan_window=W + 1,
              window_left=W, alibi_slopes=slopes(2 * g))


@pytest.mark.parametrize("dtype", [workloads.BF16, workloads.F16])
@pytest.mark.parametrize("g", [1, 4])
def test_fused_rotary_embedding_in_causal_append(dtype, g):
    """Append / prefill with the rotary embedding fused in (Sec. 3.2.3 query / key transform; Sec. 4.3): query j is
    rotated by its position l_kv - l_qo + j, key t by t, the cache holds unrotated keys.  Prefixes of several tiles,
    split chunks (a chunk's first key is not key 0), partial tiles, a request with more queries than keys, a position
    divisor, the other hooks on top, large values (peaked rows are where a rotated operand rounded once would miss
    the tolerance), positions beyond 65536."""
    qo = [70, 9, 130, 1, 64, 40]
    kv = [400, 9, 260, 300, 64, 25]
    b = workloads.make_batch("approp", 480 + g, dtype, 2 * g, 2, 128, 16, qo, kv, True, value_scale=2.0)
    kw = dict(mode="append", num_ctas=2 * 4, min_chunk=1024)
    check(b, "append, rope", rope_theta=1e4, **kw)
    check(b, "append, rope, split chunks", rope_theta=1e4, mode="append", num_ctas=2 * 16, min_chunk=64)
    check(b, "append, rope, other base and divisor", rope_theta=5e5, rope_scale=4.0, **kw)
    check(b, "append, rope + cap + window + alibi", rope_theta=1e4, logits_soft_cap=4.0, window_left=100,
          alibi_slopes=slopes(2 * g), **kw)
    far = workloads.make_batch("far", 485, dtype, 2 * g, 2, 128, 16, [40], [70000], True, poison=False)
    check(far, "append, rope at positions up to 70000", rope_theta=1e4, mode="append", num_ctas=2 * 64, min_chunk=256)


@pytest.mark.parametrize("mode", ["decode", "append"])
def test_window_known_to_the_planner(mode):
    """fi_config.plan_window: the keys before a tile's window are not in its work items at all (chunks start in
    the middle of a request), the kernel masks the rest token by token.  Windows narrower than the plan's are
    allowed; rotary embedding on top (decode): positions stay absolute."""
    if mode == "decode":
        b = workloads.make_batch("pw", 450, workloads.BF16, 8, 2, 128, 16, [1] * 5, [3000, 700, 40, 1, 0], False)
        kw = dict(num_ctas=2 * 16, min_chunk=32)
    else:
        b = workloads.make_batch("pw", 451, workloads.F16, 8, 2, 128, 16, [70, 9, 130, 1, 64], [900, 9, 260, 300, 64], True)
        kw = dict(mode="append", num_ctas=2 * 4, min_chunk=64)
    for W in (0, 5, 31, 100, 1000, 5000):
        check(b, f"{mode}, planned window {W}", plan_window=W + 1, window_left=W, **kw)
    check(b, f"{mode}, planned window 200, run with 77", plan_window=201, window_left=77, **kw)
    check(b, f"{mode}, planned window 100 + cap + alibi", plan_window=101, window_left=100, logits_soft_cap=4.0,
          alibi_slopes=slopes(8), **kw)
    if mode == "decode":
        check(b, "decode, planned window 100 + rope", plan_window=101, window_left=100, rope_theta=1e4, **kw)


def test_refused_where_not_built():
    import paper_2501_01005_amd as fi
    dummy = np.zeros(64, dtype=np.uint8)
    ok = dict(dtype=fi.FI_DTYPE_BF16, num_qo_heads=8, num_kv_heads=2, head_dim=128, page_size=16, mode=fi.FI_MODE_DECODE,
              num_ctas=8, max_batch=4, max_qo_tiles=4)
    # the rotary embedding in decode mode at other page sizes; append mode without a causal plan (also for the rotary embedding)
    for bad, var in (({"page_size": 8}, dict(rope_theta=1e4)), ({"mode": fi.FI_MODE_APPEND}, dict(window_left=3)),
                     ({"mode": fi.FI_MODE_APPEND}, dict(rope_theta=1e4))):
        causal_plan = bad.pop("causal_plan", False)
        h = fi.fi_create(**{**ok, **bad})
        if causal_plan:
            fi.fi_plan(h, np.array([0, 2], dtype=np.int32), np.array([0, 1], dtype=np.int32), np.array([5], dtype=np.int32), True)
        with pytest.raises(fi.Fi355Error) as e:
            fi.fi_run_variant(h, dummy, dummy, dummy, (8, 8, 8), dummy, dummy, dummy, 1.0, dummy, dummy, **var)
        assert e.value.code == fi.FI_ERR_UNSUPPORTED
        fi.fi_destroy(h)
    h = fi.fi_create(**ok)
    with pytest.raises(fi.Fi355Error) as e:
        fi.fi_run_variant(h, dummy, dummy, dummy, (8, 8, 8), dummy, dummy, dummy, 1.0, dummy, dummy, window_left=-5)
    assert e.value.code == fi.FI_ERR_INVALID_ARG
    fi.fi_destroy(h)


@pytest.mark.parametrize("ps", [1, 8, 32])
def test_variants_at_other_page_sizes(ps):
    """The hooks on the general paths (decode: a page id per lane; append: a page id per staged row), with windows that
    hide whole steps of split chunks."""
    b = workloads.random_case(470 + ps, dtype=workloads.BF16, num_qo_heads=8, num_kv_heads=2, batch=5, max_kv=900, page_size=ps,
                              value_scale=2.0)
    check(b, f"decode ps={ps}: all hooks", logits_soft_cap=5.0, window_left=33, alibi_slopes=slopes(8))
    check(b, f"decode ps={ps}: window over split chunks", num_ctas=2 * 16, min_chunk=64, window_left=100)
    check(b, f"decode ps={ps}: alibi", alibi_slopes=slopes(8))
    a = workloads.make_batch("app", 480 + ps, workloads.F16, 8, 2, 128, ps, [70, 9, 130], [400, 9, 333], True)
    check(a, f"append ps={ps}: all hooks", mode="append", num_ctas=2 * 4, min_chunk=128, logits_soft_cap=5.0, window_left=50,
          alibi_slopes=slopes(8))
    check(a, f"append ps={ps}: window", mode="append", window_left=64)
    check(a, f"append ps={ps}: rotary embedding", mode="append", rope_theta=1e4)
