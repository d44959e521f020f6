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
