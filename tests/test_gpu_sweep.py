"""Seeded random sweep of the whole boundary against the fp64 oracle: every handle mode, both storage types, group
sizes 1..16, page sizes 1..64, causal or not, ragged lengths (empty requests, more queries than keys), grids from one
CTA per kv head up, chunk sizes from one page up; then the variants (soft cap, ALiBi, sliding window, rotary
embedding) in decode and causal append, the 8-bit KV cache and contiguous KV.  Each case prints what it is before it
runs."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import assert_close, run_gpu
from test_gpu_variants import run_variant

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12])
def test_random_batches_through_every_mode(seed):
    rng = np.random.default_rng(seed)
    for case in range(100):
        mode = str(rng.choice(["decode", "tile16", "tile64", "append"]))
        g = int(rng.choice([1, 2, 4, 8, 16]))
        hkv = int(rng.choice([1, 2, 3]))
        dtype = workloads.F16 if rng.integers(2) else workloads.BF16
        ps = 16 if mode in ("tile16", "tile64") else int(rng.choice([1, 2, 4, 8, 16, 16, 16, 32, 64]))
        batch = int(rng.integers(1, 9))
        causal = bool(rng.integers(2)) and mode != "decode"
        max_qo = 1 if mode == "decode" else int(rng.choice([1, 3, 17, 70, 300]))
        max_kv = int(rng.choice([40, 300, 1500, 4000]))
        qo = rng.integers(1, max_qo + 1, size=batch) if max_qo > 1 else np.ones(batch, dtype=np.int64)
        if causal:
            kv = qo + rng.integers(0, max_kv, size=batch)
            if rng.integers(3) == 0:
                kv[rng.integers(batch)] = max(1, int(qo[0]) - 3)   # more queries than keys: leading rows see nothing
        else:
            kv = rng.integers(0, max_kv + 1, size=batch)
        kw = {}
        if rng.integers(2):
            kw["num_ctas"] = hkv * int(rng.choice([1, 2, 5, 16, 64]))
        if rng.integers(2):
            kw["min_chunk"] = int(rng.choice([16, 32, 64, 128, 256]))
        data_seed = 5000 + int(rng.integers(100000))
        need = int(((kv + ps - 1) // ps).sum())
        b = workloads.make_batch("sweep", data_seed, dtype, g * hkv, hkv, 128, ps, qo, kv, causal, num_pages=need + 2,
                                 value_scale=float(rng.choice([0.5, 1.0, 2.0])))
        what = (f"sweep {seed}/{case}: mode={mode} g={g} hkv={hkv} {dtype} ps={ps} causal={causal} qo={qo.tolist()} "
                f"kv={kv.tolist()} kw={kw} data_seed={data_seed}")
        print("[case] " + what, flush=True)
        o_ref, lse_ref = oracle.run_batch(b)
        o, lse = run_gpu(b, mode, **kw)
        assert_close(o, lse, o_ref, lse_ref, what)


@pytest.mark.parametrize("seed", [21])
def test_random_variants_fp8_and_contiguous(seed):
    rng = np.random.default_rng(seed)
    for case in range(120):
        kind = str(rng.choice(["variant", "variant", "kv8", "contig"]))
        mode = str(rng.choice(["decode", "append"]))
        g = int(rng.choice([1, 2, 4, 8]))
        hkv = int(rng.choice([1, 2]))
        dtype = workloads.F16 if rng.integers(2) else workloads.BF16
        batch = int(rng.integers(1, 7))
        causal = mode == "append"
        max_qo = 1 if mode == "decode" else int(rng.choice([3, 40, 200, 400]))
        max_kv = int(rng.choice([60, 400, 1500, 3000]))
        qo = rng.integers(1, max_qo + 1, size=batch) if max_qo > 1 else np.ones(batch, dtype=np.int64)
        kv = qo + rng.integers(0, max_kv, size=batch)
        kw = {}
        if rng.integers(2):
            kw["num_ctas"] = hkv * int(rng.choice([1, 2, 5, 16, 64]))
        if rng.integers(2):
            kw["min_chunk"] = int(rng.choice([16, 32, 64, 128, 256]))
        data_seed = 9000 + int(rng.integers(100000))
        ps, var, extra = 16, {}, {}
        if kind == "kv8":
            mode, causal = "decode", False
            qo = np.ones(batch, dtype=np.int64)
            ps = int(rng.choice([16, 16, 8, 32]))
            extra = dict(kv_dtype=workloads.FP8, k_scale=float(rng.choice([0.25, 1.0])), v_scale=float(rng.choice([0.5, 2.0])))
        elif kind == "contig":
            ps = int(rng.choice([16, 16, 1, 8, 32]))
            extra = dict(permute_pages=False)
        else:
            if rng.integers(2):
                var["logits_soft_cap"] = float(rng.choice([2.0, 10.0, 30.0]))
            if rng.integers(2):
                var["alibi_slopes"] = np.array([2.0 ** (-(i + 1) * 8.0 / (g * hkv)) for i in range(g * hkv)])
            if rng.integers(2):
                var["window_left"] = int(rng.choice([0, 5, 31, 100, 1000]))
            if rng.integers(3) == 0:
                var["rope_theta"] = float(rng.choice([1e4, 5e5]))
            if not var:
                var["window_left"] = 64
            ps = int(rng.choice([16, 16, 1, 8, 32]))
            if ps != 16 and mode == "decode":
                var.pop("rope_theta", None)    # (the rotary embedding in decode mode is built for page size 16)
                var.setdefault("window_left", 64)
        need = int(((kv + ps - 1) // ps).sum())
        b = workloads.make_batch("sweep", data_seed, dtype, g * hkv, hkv, 128, ps, qo, kv, causal,
                                 num_pages=need + (0 if kind == "contig" else 2),
                                 value_scale=float(rng.choice([0.5, 1.0, 2.0])), **extra)
        what = (f"sweep {seed}/{case}: {kind} mode={mode} g={g} hkv={hkv} {dtype} ps={ps} qo={qo.tolist()} kv={kv.tolist()} "
                f"kw={kw} variant={ {k: (v if np.isscalar(v) else 'array') for k, v in var.items()} } data_seed={data_seed}")
        print("[case] " + what, flush=True)
        o_ref, lse_ref = oracle.run_batch(b, **var)
        if kind == "variant":
            o, lse = run_variant(b, mode=mode, num_ctas=kw.get("num_ctas", 0), min_chunk=kw.get("min_chunk", 0), **var)
        else:
            o, lse = run_gpu(b, mode, contiguous=(kind == "contig"), **kw)
        assert_close(o, lse, o_ref, lse_ref, what)


@pytest.mark.parametrize("mode", ["tile16", "tile64"])
def test_random_plans_over_two_and_three_formats(mode):
    """Random row partitions and page lists per format (Sec. 3.1.2), planned as one work list and run in one launch;
    expected: each format's attention by the oracle, then the oracle's merge of the states (Sec. 2.2: the merged state
    is the attention over the union of the formats' keys)."""
    import dataclasses
    import torch
    from oracle.attention import merge_pair
    from gpu_util import DeviceBatch
    from paper_2501_01005_amd.device import formats_of, make_formats_wrapper
    rng = np.random.default_rng(31 if mode == "tile16" else 32)
    for case in range(40):
        g = int(rng.choice([1, 2, 4, 8]))
        hkv = int(rng.choice([1, 2]))
        dtype = workloads.F16 if rng.integers(2) else workloads.BF16
        n_rows = int(rng.integers(1, 50))
        n_formats = int(rng.integers(2, 4))
        cuts_of, kv_of = [], []
        for f in range(n_formats):
            if f == 0 and rng.integers(2):
                cuts = [0, n_rows]                                      # a shared prefix: one row block
            else:
                cuts = sorted(set(rng.integers(0, n_rows + 1, size=int(rng.integers(0, n_rows + 1))).tolist()) | {0, n_rows})
            cuts_of.append(np.array(cuts))
            kv_of.append(rng.integers(0, int(rng.choice([50, 400, 2000])), size=len(cuts) - 1))
        # one pool for all formats: the requests of all formats one after the other; the query rows ride on the first
        # format's requests
        qo_all = np.concatenate([np.diff(cuts_of[0])] + [np.zeros(len(k), dtype=np.int64) for k in kv_of[1:]])
        kv_all = np.concatenate(kv_of)
        data_seed = 7000 + int(rng.integers(100000))
        base = workloads.make_batch("formats_pool", data_seed, dtype, g * hkv, hkv, 128, 16, qo_all, kv_all, False,
                                    num_pages=int(((kv_all + 15) // 16).sum()) + 2, value_scale=float(rng.choice([0.5, 1.0, 2.0])))
        batches, first = [], 0
        for f in range(n_formats):
            n_req = len(kv_of[f])
            p0 = int(base.kv_indptr[first])
            batches.append(dataclasses.replace(
                base, name=f"format{f}", qo_indptr=cuts_of[f].astype(np.int32),
                kv_indptr=(base.kv_indptr[first:first + n_req + 1] - p0).astype(np.int32),
                kv_indices=base.kv_indices[p0:int(base.kv_indptr[first + n_req])].copy(),
                last_page_len=base.last_page_len[first:first + n_req].copy()))
            first += n_req
        kw = {}
        if rng.integers(2):
            kw["num_ctas"] = hkv * int(rng.choice([1, 3, 16, 64]))
        if rng.integers(2):
            kw["min_chunk"] = int(rng.choice([16, 32, 128]))
        what = (f"formats {mode}/{case}: g={g} hkv={hkv} {dtype} rows={n_rows} cuts={[c.tolist() for c in cuts_of]} "
                f"kv={[k.tolist() for k in kv_of]} kw={kw} data_seed={data_seed}")
        print("[case] " + what, flush=True)
        o_ref, lse_ref = oracle.run_batch(batches[0])
        for b in batches[1:]:
            o_f, lse_f = oracle.run_batch(b)
            o_ref, lse_ref = merge_pair(o_ref, lse_ref, o_f, lse_f)
        formats, ids = formats_of(batches)
        w = make_formats_wrapper(batches, mode=mode, **kw)
        dev = DeviceBatch(batches[0])
        ids_dev = torch.from_numpy(ids).to("cuda:0")
        w.workspace.view(torch.float32)[w.pin_bytes // 4:].fill_(float("nan"))
        w.plan_formats(formats)
        H = g * hkv
        o = torch.full((n_rows, H, 128), float("nan"), dtype=torch.float32, device="cuda:0")
        lse = torch.full((n_rows, H), float("nan"), dtype=torch.float32, device="cuda:0")
        w.run(dev.q, dev.k_pool, dev.v_pool, ids_dev, base.sm_scale, o=o, lse=lse)
        torch.cuda.synchronize()
        w.close()
        assert_close(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, what)
