"""Host logic of the C-ABI library, runnable without a GPU: the exported symbols, the
planner (bit-exact against the replica of Algorithm 1), argument errors."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2501_01005_amd as fi
from oracle.plan_replica import plan_replica

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PLAN_KEYS = ("cta_indptr", "w_request", "w_q_row0", "w_n_pos", "w_kv_page0", "w_kv_start", "w_kv_len", "w_diag0",
             "w_out_slot", "w_merge", "m_q_row0", "m_n_pos", "m_slot_base", "m_n_chunks")


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fi355.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(fi_[a-z0-9_]+)\s*\(", header))
    assert {"fi_create", "fi_destroy", "fi_workspace_bytes", "fi_plan", "fi_plan_view", "fi_run", "fi_run_kv8", "fi_run_variant",
            "fi_run_composed", "fi_merge_states", "fi_merge_state_pair", "fi_check_indices", "fi_set_timing_events",
            "fi_last_error"} <= names
    L = ctypes.CDLL(fi.library_path())
    for n in names:
        assert hasattr(L, n), n


def make(mode, g, C, Hkv=2, max_batch=64, max_tiles=4096, **kw):
    return fi.fi_create(dtype=fi.FI_DTYPE_BF16, num_qo_heads=g * Hkv, num_kv_heads=Hkv, head_dim=128, page_size=16,
                        mode=mode, num_ctas=C * Hkv, max_batch=max_batch, max_qo_tiles=max_tiles, **kw)


def indptrs(qo, kv, ps=16):
    qo_indptr = np.concatenate([[0], np.cumsum(qo)]).astype(np.int32)
    n_pg = (np.asarray(kv) + ps - 1) // ps
    kv_indptr = np.concatenate([[0], np.cumsum(n_pg)]).astype(np.int32)
    last = np.where(n_pg > 0, np.asarray(kv) - (n_pg - 1) * ps, 0).astype(np.int32)
    return qo_indptr, kv_indptr, last


def compare(h, qo, kv, causal, t_pos, g, C, alpha, beta, min_chunk, literal=False, refine=False, light_rows=0,
            plan_window=0, item_cost=0):
    qo_indptr, kv_indptr, last = indptrs(qo, kv)
    fi.fi_plan(h, qo_indptr, kv_indptr, last, causal)
    got = fi.fi_plan_view(h)
    want = plan_replica(qo_indptr, kv_indptr, last, page_size=16, t_pos=t_pos, group=g, num_ctas=C, causal=causal,
                        alpha=alpha, beta=beta, min_chunk=min_chunk, literal_lkv=literal, refine=refine,
                        light_rows=light_rows, light_pct=64, kv_quantum=64 if light_rows else 1,
                        plan_window=plan_window, item_cost=item_cost)
    assert got["l_kv_chunk"] == want["L_kv"] and got["n_work"] == want["n_work"]
    assert got["n_merge"] == want["n_merge"] and got["n_slots"] == want["n_slots"]
    assert got["t_pos"] == t_pos and got["group"] == g and got["ctas_per_head"] == C
    for k in PLAN_KEYS:
        assert got[k].dtype == np.int32
        assert got[k].tobytes() == np.asarray(want[k], dtype=np.int32).tobytes(), k


@pytest.mark.parametrize("mode", ["decode", "append"])
def test_planner_equals_replica_on_random_length_sets(mode):
    rng = np.random.default_rng(7 if mode == "decode" else 8)
    n_cases = 0
    for g in (1, 4):
        for C in (1, 5, 32, 256):
            # (alpha, beta, min_chunk, balance): 1 = Algorithm 1 as printed, 2 = with the refinement
            for (alpha, beta, min_chunk, balance) in ((1, 1, 16, 1), (0, 1, 256, 1), (3, 2, 64, 2), (8, 5, 128, 2)):
                t_pos = 1 if mode == "decode" else 256 // g
                h = make(fi.FI_MODE_DECODE if mode == "decode" else fi.FI_MODE_APPEND, g, C, alpha=alpha, beta=beta,
                         min_chunk=min_chunk, balance=balance)
                refine = balance == 2
                light_rows = 128 if (refine and mode == "append") else 0
                for trial in range(20):
                    B = int(rng.integers(1, 48))
                    if mode == "decode":
                        qo = np.ones(B, dtype=np.int64)
                        kv = rng.integers(0, 4000, size=B)
                        r = rng.random()
                        if r < 0.25:
                            kv[rng.integers(0, B)] = int(rng.integers(30000, 300000))
                        elif r < 0.4:
                            kv[:] = int(rng.integers(1, 700))
                        elif r < 0.5:
                            B = 1; qo = qo[:1]; kv = kv[:1]
                    else:
                        qo = rng.integers(0, 600, size=B)
                        kv = qo + rng.integers(0, 3000, size=B)
                        if rng.random() < 0.2:
                            kv = np.maximum(kv - rng.integers(0, 100, size=B), 0)
                    compare(h, qo, kv, mode == "append", t_pos, g, C, alpha, beta, min_chunk, refine=refine,
                            light_rows=light_rows)
                    n_cases += 1
                fi.fi_destroy(h)
    assert n_cases >= 600


@pytest.mark.parametrize("mode", ["decode", "append"])
def test_planner_equals_replica_with_a_sliding_window(mode):
    rng = np.random.default_rng(17 if mode == "decode" else 18)
    for g in (1, 4):
        t_pos = 1 if mode == "decode" else 256 // g
        for C in (3, 32, 256):
            for window in (1, 16, 100, 1025, 100000):
                h = make(fi.FI_MODE_DECODE if mode == "decode" else fi.FI_MODE_APPEND, g, C, min_chunk=32, balance=1,
                         plan_window=window)
                for trial in range(8):
                    B = int(rng.integers(1, 24))
                    if mode == "decode":
                        qo = np.ones(B, dtype=np.int64)
                        kv = rng.integers(0, 5000, size=B)
                        if trial % 3 == 0:
                            kv[0] = int(rng.integers(30000, 200000))
                    else:
                        qo = rng.integers(0, 600, size=B)
                        kv = qo + rng.integers(0, 3000, size=B)
                    compare(h, qo, kv, mode == "append", t_pos, g, C, 1, 1, 32, plan_window=window)
                fi.fi_destroy(h)


def test_default_decode_plan_weighs_the_fixed_cost_of_a_work_item():
    """balance = 0 in decode mode: Algorithm 1's chunk length, unless the batch is so small that a slightly longer
    chunk saves every CTA a second work item (64 requests of 64..512 tokens on 256 CTAs: 80 -> 96 tokens)."""
    rng = np.random.default_rng(23)
    for C in (8, 64, 256):
        h = make(fi.FI_MODE_DECODE, 4, C, max_batch=128)
        h1 = make(fi.FI_MODE_DECODE, 4, C, max_batch=128, balance=1)
        for trial in range(12):
            B = int(rng.integers(1, 100))
            kv = rng.integers(0, (64, 513, 3000)[trial % 3], size=B)
            compare(h, np.ones(B, dtype=np.int64), kv, False, 1, 4, C, 1, 1, 32, item_cost=64)
            compare(h1, np.ones(B, dtype=np.int64), kv, False, 1, 4, C, 1, 1, 32)
        fi.fi_destroy(h); fi.fi_destroy(h1)
    g5 = np.random.Generator(np.random.PCG64(1005))
    kv = g5.integers(64, 513, size=64)
    h = make(fi.FI_MODE_DECODE, 4, 256, Hkv=8, max_batch=64)
    qo_indptr, kv_indptr, last = indptrs(np.ones(64, dtype=np.int64), kv)
    fi.fi_plan(h, qo_indptr, kv_indptr, last, False)
    got = fi.fi_plan_view(h)
    as_printed = plan_replica(qo_indptr, kv_indptr, last, page_size=16, t_pos=1, group=4, num_ctas=256, causal=False, min_chunk=32)
    assert as_printed["n_work"] > 256 and got["n_work"] <= 256 and got["l_kv_chunk"] > as_printed["L_kv"]
    fi.fi_destroy(h)


def test_planner_equals_replica_on_the_benchmark_length_sets():
    import workloads
    g2 = np.random.Generator(np.random.PCG64(1002))
    kv2 = workloads.zipf_lengths(g2, 128, 256, 32768, 1.2); kv2[0] = 32768
    h = make(fi.FI_MODE_DECODE, 4, 256, Hkv=8, max_batch=128, min_chunk=256)
    compare(h, np.ones(128, dtype=np.int64), kv2, False, 1, 4, 256, 1, 1, 256)
    compare(h, [1, 1], [131072, 65536], False, 1, 4, 256, 1, 1, 256)
    fi.fi_destroy(h)
    g3 = np.random.Generator(np.random.PCG64(1003))
    qo = g3.integers(128, 1025, size=16); pre = g3.integers(0, 4097, size=16)
    # append defaults: refined assignment with the measured cost (alpha, beta) = (8, 5), light tiles at 64 %
    for C in (32, 64):
        h = make(fi.FI_MODE_APPEND, 4, C, Hkv=8, max_batch=16, max_tiles=1024, min_chunk=256)
        compare(h, qo, qo + pre, True, 64, 4, C, 8, 5, 256, refine=True, light_rows=128)
        fi.fi_destroy(h)
    h = make(fi.FI_MODE_APPEND, 4, 64, Hkv=8, max_batch=16, max_tiles=1024, min_chunk=256, balance=1)
    compare(h, qo, qo + pre, True, 64, 4, 64, 1, 1, 256)
    fi.fi_destroy(h)
    h = make(fi.FI_MODE_APPEND, 4, 64, Hkv=8, max_batch=16, max_tiles=1024, min_chunk=256, literal_lkv=1, balance=1)
    compare(h, qo, qo + pre, True, 64, 4, 64, 1, 1, 256, literal=True)
    fi.fi_destroy(h)


def test_plan_is_deterministic_and_sections_do_not_move():
    h = make(fi.FI_MODE_DECODE, 4, 16)
    sizes = fi.fi_workspace_bytes(h)
    rng = np.random.default_rng(3)
    kv = rng.integers(1, 9000, size=20)
    qo_indptr, kv_indptr, last = indptrs(np.ones(20, dtype=np.int64), kv)
    fi.fi_plan(h, qo_indptr, kv_indptr, last, False)
    a = fi.fi_plan_view(h)
    fi.fi_plan(h, *indptrs(np.ones(3, dtype=np.int64), [5, 6, 7]), False)
    assert fi.fi_workspace_bytes(h) == sizes                 # layout depends on the config only (App. D.1)
    fi.fi_plan(h, qo_indptr, kv_indptr, last, False)
    b = fi.fi_plan_view(h)
    for k in PLAN_KEYS:
        assert a[k].tobytes() == b[k].tobytes()
    fi.fi_destroy(h)


def expect(code, fn, *a, **kw):
    with pytest.raises(fi.Fi355Error) as e:
        fn(*a, **kw)
    assert e.value.code == code and e.value.message


def test_argument_errors():
    ok = dict(dtype=fi.FI_DTYPE_BF16, num_qo_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
              mode=fi.FI_MODE_DECODE, num_ctas=64, max_batch=4, max_qo_tiles=4)
    expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "head_dim": 64})
    expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "page_size": 12})
    expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "page_size": 128})
    expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "num_qo_heads": 24})       # g = 3
    expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "num_qo_heads": 64, "merge": 2})   # in-launch contraction: g <= 4
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_create, **{**ok, "num_qo_heads": 30})
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_create, **{**ok, "dtype": 7})
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_create, **{**ok, "max_batch": 0})
    h = fi.fi_create(**ok)
    expect(fi.FI_ERR_NOT_PLANNED, fi.fi_plan_view, h)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_plan, h, [1, 2], [0, 1], [3], False)            # indptr[0] != 0
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_plan, h, [0, 1, 0], [0, 1, 2], [3, 3], False)   # decreasing
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_plan, h, [0, 1], [0, 1], [0], False)            # last_page_len = 0
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_plan, h, [0, 1], [0, 1], [17], False)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_plan, h, np.arange(6), np.arange(6), [1] * 5, False)   # batch > max_batch
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_plan, h, [0, 9], [0, 1], [3], False)            # 9 tiles > max_qo_tiles
    expect(fi.FI_ERR_NOT_PLANNED, fi.fi_plan_view, h)                                   # a failed plan leaves none
    fi.fi_plan(h, [0, 1], [0, 0], [0], False)                                           # empty request is fine
    assert fi.fi_plan_view(h)["n_work"] == 1
    # fi_run needs a plan that went to a device workspace
    dummy = np.zeros(64, dtype=np.uint8)
    expect(fi.FI_ERR_NOT_PLANNED, fi.fi_run, h, dummy, dummy, dummy, (1, 1, 1), dummy, 1.0, dummy, dummy)
    expect(fi.FI_ERR_NOT_PLANNED, fi.fi_run_kv8, h, dummy, dummy, dummy, (8, 8, 8), dummy, 1.0, 1.0, 1.0, dummy, dummy)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_run_kv8, h, dummy, dummy, dummy, (8, 8, 8), dummy, 1.0, 0.0, 1.0, dummy, dummy)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_create, **{**ok, "balance": 3})
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_create, **{**ok, "merge": 3})
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_create, **{**ok, "plan_window": -1})
    hw = fi.fi_create(**{**ok, "plan_window": 65})          # a window-planned handle runs with a matching window only
    dummy = np.zeros(64, dtype=np.uint8)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_run, hw, dummy, dummy, dummy, (8, 8, 8), dummy, 1.0, dummy, dummy)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_run_variant, hw, dummy, dummy, dummy, (8, 8, 8), dummy, dummy, dummy, 1.0, dummy, dummy,
           window_left=65)
    fi.fi_destroy(hw)
    expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "merge": 2, "mode": fi.FI_MODE_APPEND})   # in-launch contraction: decode only
    ha = fi.fi_create(**{**ok, "mode": fi.FI_MODE_APPEND})
    expect(fi.FI_ERR_UNSUPPORTED, fi.fi_run_kv8, ha, dummy, dummy, dummy, (8, 8, 8), dummy, 1.0, 1.0, 1.0, dummy, dummy)
    fi.fi_destroy(ha)
    # workspace too small is detected before anything is touched
    expect(fi.FI_ERR_WORKSPACE_TOO_SMALL, fi.fi_plan, h, [0, 1], [0, 1], [3], False, workspace=dummy,
           workspace_bytes=64)
    fi.fi_destroy(h)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_check_indices, [0, 5, 2], 5)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_check_indices, [0, -1], 5)
    fi.fi_check_indices([0, 4, 2], 5)
    expect(fi.FI_ERR_UNSUPPORTED, fi.fi_merge_states, dummy, dummy, 1, 1, 64, dummy, dummy)
    # the tile modes: page size 16 only, no planned window, no in-launch contraction, no variants, no 8-bit cache
    for mode in (fi.FI_MODE_TILE16, fi.FI_MODE_TILE64):
        expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "mode": mode, "page_size": 8})
        expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "mode": mode, "plan_window": 9})
        expect(fi.FI_ERR_UNSUPPORTED, fi.fi_create, **{**ok, "mode": mode, "merge": 2})
        ht = fi.fi_create(**{**ok, "mode": mode})
        expect(fi.FI_ERR_UNSUPPORTED, fi.fi_run_variant, ht, dummy, dummy, dummy, (8, 8, 8), dummy, dummy, dummy, 1.0, dummy, dummy,
               window_left=5)
        expect(fi.FI_ERR_UNSUPPORTED, fi.fi_run_kv8, ht, dummy, dummy, dummy, (8, 8, 8), dummy, 1.0, 1.0, 1.0, dummy, dummy)
        fi.fi_destroy(ht)
    expect(fi.FI_ERR_INVALID_ARG, fi.fi_create, **{**ok, "mode": 4})


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 on its own (no C++, no HIP types)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    header = os.path.join(os.path.dirname(__file__), "..", "include", "fi355.h")
    r = subprocess.run([gcc, "-fsyntax-only", "-x", "c", "-std=c99", "-Wall", "-Werror", header], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_committed_append_loops_are_what_the_generator_writes(tmp_path):
    """The scheduled loops of the append kernel (csrc/append_loop_*.inc) are generated assembly that is committed
    and compiled as is: regenerate them and compare, so that an edit by hand, or a generator change without
    regeneration, fails here."""
    import subprocess
    import sys
    csrc = os.path.join(ROOT, "paper_2501_01005_amd", "csrc")
    subprocess.run([sys.executable, os.path.join(csrc, "gen", "gen_append_loop.py"), str(tmp_path)], check=True,
                   capture_output=True)
    generated = sorted(os.listdir(tmp_path))
    committed = sorted(f for f in os.listdir(csrc) if f.startswith("append_loop_") and f.endswith(".inc"))
    assert generated == committed and len(generated) >= 5
    for f in generated:
        assert open(os.path.join(tmp_path, f)).read() == open(os.path.join(csrc, f)).read(), f


@pytest.mark.parametrize("name", ["plan_decode_example.txt", "plan_item_cost_example.txt", "plan_window_decode_example.txt",
                                  "plan_window_causal_example.txt", "plan_refine_example.txt"])
def test_planner_reproduces_the_hand_worked_examples(name):
    """The pencil-worked fixtures (those whose tile shape the library can be configured to: decode, or append with
    g = 4) through fi_plan: the planner itself against the hand-worked arrays, not only against the replica."""
    from test_oracle_plan import FIXTURE_KEYS, load_fixture
    fx = load_fixture(name)
    opt = lambda k, d: fx.get(k, [d])[0]
    g, C, t_pos = fx["group"][0], fx["num_ctas"][0], fx["t_pos"][0]
    decode = t_pos == 1
    assert decode or (t_pos == 64 and g == 4)
    if opt("refine", 0):
        assert (opt("light_rows", 0), opt("light_pct", 100), opt("kv_quantum", 1)) == (128, 64, 64)   # the library's constants
        balance = 2
    elif opt("item_cost", 0):
        assert decode and opt("item_cost", 0) == 64                                                 # the library's constant
        balance = 0
    else:
        balance = 1
    h = make(fi.FI_MODE_DECODE if decode else fi.FI_MODE_APPEND, g, C, alpha=opt("alpha", 1), beta=opt("beta", 1),
             min_chunk=opt("min_chunk", 16), balance=balance, plan_window=opt("plan_window", 0))
    qo_indptr, kv_indptr, last = indptrs(fx["qo_len"], fx["kv_len"])
    fi.fi_plan(h, qo_indptr, kv_indptr, last, bool(fx["causal"][0]))
    got = fi.fi_plan_view(h)
    assert got["l_kv_chunk"] == fx["L_kv"][0]
    for key in FIXTURE_KEYS:
        if key in fx and key != "cta_cost":
            assert got[key].tolist() == fx[key], key
    fi.fi_destroy(h)


def make_tile16(g, C, Hkv=2, max_batch=256, max_tiles=1024, **kw):
    return fi.fi_create(dtype=fi.FI_DTYPE_BF16, num_qo_heads=g * Hkv, num_kv_heads=Hkv, head_dim=128, page_size=16,
                        mode=fi.FI_MODE_TILE16, num_ctas=C * Hkv, max_batch=max_batch, max_qo_tiles=max_tiles, **kw)


def compare_formats(h, formats, want):
    fi.fi_plan_formats(h, formats)
    got = fi.fi_plan_view(h)
    assert got["l_kv_chunk"] == want["L_kv"] and got["n_work"] == want["n_work"]
    assert got["n_merge"] == want["n_merge"] and got["n_slots"] == want["n_slots"]
    keys = PLAN_KEYS + (("row_indptr", "row_entry") if len(formats) > 1 else ())
    assert got["n_rows"] == want.get("n_rows", 0)
    for k in keys:
        assert got[k].tobytes() == np.asarray(want[k], dtype=np.int32).tobytes(), k


def test_planner_reproduces_the_hand_worked_plan_over_two_formats():
    from test_oracle_plan import FIXTURE_KEYS, formats_of_fixture, load_fixture
    fx = load_fixture("plan_formats_example.txt")
    h = make_tile16(fx["group"][0], fx["num_ctas"][0], alpha=1, beta=1, min_chunk=16, balance=1)
    fi.fi_plan_formats(h, formats_of_fixture(fx))
    got = fi.fi_plan_view(h)
    assert got["l_kv_chunk"] == fx["L_kv"][0] and got["n_slots"] == fx["n_slots"][0] and got["n_merge"] == 0
    assert got["t_pos"] == fx["t_pos"][0] and got["n_rows"] == 6
    for key in FIXTURE_KEYS + ("row_indptr", "row_entry"):
        if key in fx and key != "cta_cost":
            assert got[key].tolist() == fx[key], key
    fi.fi_destroy(h)


def test_planner_equals_replica_over_several_formats():
    from oracle.plan_replica import plan_replica_formats
    rng = np.random.default_rng(41)
    n_cases = 0
    for g in (1, 4, 16):
        for C in (1, 7, 256):
            for (alpha, beta, min_chunk, balance) in ((1, 1, 16, 1), (2, 3, 32, 0)):
                h = make_tile16(g, C, alpha=alpha, beta=beta, min_chunk=min_chunk, balance=balance)
                for trial in range(12):
                    n_rows = int(rng.integers(1, 70))
                    n_formats = int(rng.integers(1, 4))
                    formats, base = [], 0
                    for f in range(n_formats):
                        if f == 0 and trial % 2 == 0:
                            cuts = [0, n_rows]                      # a shared prefix: one row block
                        else:
                            cuts = sorted(set(rng.integers(0, n_rows + 1, size=int(rng.integers(0, n_rows + 1))).tolist()) | {0, n_rows})
                        qo = np.diff(cuts)
                        kv = rng.integers(0, 3000 if f == 0 else 600, size=len(qo))
                        qo_indptr, kv_indptr, last = indptrs(qo, kv)
                        formats.append((qo_indptr, kv_indptr, last, base))
                        base += int(kv_indptr[-1])
                    want = plan_replica_formats(formats, page_size=16, t_pos=16 // g, group=g, num_ctas=C, causal=False,
                                                alpha=alpha, beta=beta, min_chunk=min_chunk,
                                                item_cost=64 if balance == 0 else 0)
                    compare_formats(h, formats, want)
                    n_cases += 1
                fi.fi_destroy(h)
    assert n_cases >= 200


def test_tile16_single_format_plans_equal_the_replica_causal_and_not():
    rng = np.random.default_rng(43)
    for g in (2, 4):
        for C in (3, 64):
            h = make_tile16(g, C, alpha=1, beta=1, min_chunk=16, balance=1)
            for trial in range(10):
                B = int(rng.integers(1, 20))
                qo = rng.integers(0, 40, size=B)
                kv = qo + rng.integers(0, 900, size=B)
                for causal in (False, True):
                    compare(h, qo, kv, causal, 16 // g, g, C, 1, 1, 16)
            fi.fi_destroy(h)


def make_tile64(g, C, Hkv=2, max_batch=256, max_tiles=1024, **kw):
    return fi.fi_create(dtype=fi.FI_DTYPE_BF16, num_qo_heads=g * Hkv, num_kv_heads=Hkv, head_dim=128, page_size=16,
                        mode=fi.FI_MODE_TILE64, num_ctas=C * Hkv, max_batch=max_batch, max_qo_tiles=max_tiles, **kw)


# what fi_create sets for the planner in the 64-row tile mode with balance = 0: refined assignment, a tile of at most
# 16 fused rows counts 30 percent per token, in the costs and in the sum behind the chunk length; costs in steps of 32
TILE64_PLAN = dict(refine=True, light_rows=16, light_pct=30, kv_quantum=32, weighted_lkv=True)


def test_planner_reproduces_the_hand_worked_weighted_plan():
    from test_oracle_plan import FIXTURE_KEYS, formats_of_fixture, load_fixture
    fx = load_fixture("plan_weighted_formats_example.txt")
    h = make_tile64(fx["group"][0], fx["num_ctas"][0], min_chunk=16)
    fi.fi_plan_formats(h, formats_of_fixture(fx))
    got = fi.fi_plan_view(h)
    assert got["l_kv_chunk"] == fx["L_kv"][0] and got["n_slots"] == fx["n_slots"][0] and got["n_merge"] == 0
    assert got["t_pos"] == fx["t_pos"][0] and got["n_rows"] == 8
    for key in FIXTURE_KEYS + ("row_indptr", "row_entry"):
        if key in fx and key != "cta_cost":
            assert got[key].tolist() == fx[key], key
    fi.fi_destroy(h)


def test_tile64_plans_equal_the_replica():
    """64-row tile mode: plans over several formats and over one (causal and not), default and as-printed balance;
    the workspace sections hold every such plan (the weighted chunk length allows more chunks than #CTA extra)."""
    from oracle.plan_replica import plan_replica_formats
    rng = np.random.default_rng(47)
    n_cases = 0
    for g in (1, 4, 16):
        for C in (1, 7, 64):
            for (min_chunk, balance) in ((16, 0), (128, 0), (32, 1)):
                h = make_tile64(g, C, min_chunk=min_chunk, balance=balance)
                kw = dict(page_size=16, t_pos=64 // g, group=g, num_ctas=C, min_chunk=min_chunk,
                          **(TILE64_PLAN if balance == 0 else {}))
                for trial in range(10):
                    n_rows = int(rng.integers(1, 90))
                    n_formats = int(rng.integers(1, 4))
                    formats, base = [], 0
                    for f in range(n_formats):
                        if f == 0 and trial % 2 == 0:
                            cuts = [0, n_rows]                      # a shared prefix: one row block
                        else:
                            cuts = sorted(set(rng.integers(0, n_rows + 1, size=int(rng.integers(0, n_rows + 1))).tolist()) | {0, n_rows})
                        qo = np.diff(cuts)
                        kv = rng.integers(0, 3000 if f == 0 else 600, size=len(qo))
                        qo_indptr, kv_indptr, last = indptrs(qo, kv)
                        formats.append((qo_indptr, kv_indptr, last, base))
                        base += int(kv_indptr[-1])
                    compare_formats(h, formats, plan_replica_formats(formats, causal=False, **kw))
                    n_cases += 1
                    B = int(rng.integers(1, 20))
                    qo = rng.integers(0, 80, size=B)
                    kv = qo + rng.integers(0, 900, size=B)
                    for causal in (False, True):
                        qo_indptr, kv_indptr, last = indptrs(qo, kv)
                        fi.fi_plan(h, qo_indptr, kv_indptr, last, causal)
                        got = fi.fi_plan_view(h)
                        want = plan_replica(qo_indptr, kv_indptr, last, causal=causal, **kw)
                        assert got["l_kv_chunk"] == want["L_kv"] and got["n_work"] == want["n_work"]
                        for k in PLAN_KEYS:
                            assert got[k].tobytes() == np.asarray(want[k], dtype=np.int32).tobytes(), k
                        n_cases += 1
                fi.fi_destroy(h)
    assert n_cases >= 800


def test_plan_formats_argument_errors():
    h = make_tile16(4, 4)
    qo, kv, last = indptrs([3], [40])
    qo2, kv2, last2 = indptrs([1, 1], [5, 6])
    with pytest.raises(fi.Fi355Error) as e:
        fi.fi_plan_formats(h, [(qo, kv, last, 0), (qo2, kv2, last2, 3)])       # 3 rows against 2
    assert e.value.code == fi.FI_ERR_INVALID_ARG and "query rows" in e.value.message
    with pytest.raises(fi.Fi355Error) as e:
        fi.fi_plan_formats(h, [(qo, kv, last, -1)])
    assert e.value.code == fi.FI_ERR_INVALID_ARG
    fi.fi_destroy(h)
    hd = make(fi.FI_MODE_DECODE, 4, 4)
    with pytest.raises(fi.Fi355Error) as e:
        fi.fi_plan_formats(hd, [(qo2, kv2, last2, 0)])
    assert e.value.code == fi.FI_ERR_UNSUPPORTED
    fi.fi_destroy(hd)


def test_suggested_mode_follows_the_mean_query_length():
    assert fi.fi_suggest_mode(32, 8, 1.0) == "decode" and fi.fi_suggest_mode(8, 8, 0.5) == "decode"
    assert fi.fi_suggest_mode(32, 8, 4.0) == "tile64" and fi.fi_suggest_mode(8, 8, 16.0) == "tile64"
    assert fi.fi_suggest_mode(32, 8, 5.0) == "append" and fi.fi_suggest_mode(32, 2, 2.0) == "append"
    with pytest.raises(fi.Fi355Error) as e:
        fi.fi_suggest_mode(6, 4, 1.0)
    assert e.value.code == fi.FI_ERR_INVALID_ARG


@pytest.mark.parametrize("mode", [fi.FI_MODE_TILE16, fi.FI_MODE_TILE64])
def test_one_format_at_a_time_takes_the_small_workspace(mode):
    """fi_config.max_formats = 1 on a tile handle: the partial-state sections are bounded by the CTAs (App. D.3), not by
    the work items; single-format plans are the same arrays; several formats at once are refused."""
    any_formats = make(mode, 4, 8, max_batch=64, max_tiles=20000)
    one_format = make(mode, 4, 8, max_batch=64, max_tiles=20000, max_formats=1)
    assert fi.fi_workspace_bytes(one_format)[0] < fi.fi_workspace_bytes(any_formats)[0] // 8
    rng = np.random.default_rng(31)
    for trial in range(20):
        B = int(rng.integers(1, 40))
        qo = rng.integers(1, 20, size=B)
        qo_indptr, kv_indptr, last = indptrs(qo, qo + rng.integers(0, 3000, size=B))
        views = []
        for h in (any_formats, one_format):
            fi.fi_plan(h, qo_indptr, kv_indptr, last, True)
            views.append(fi.fi_plan_view(h))
        assert views[0]["n_work"] == views[1]["n_work"] and views[0]["n_slots"] == views[1]["n_slots"]
        for k in PLAN_KEYS:
            assert views[0][k].tobytes() == views[1][k].tobytes(), k
    qo2, kv2, last2 = indptrs([1, 1], [5, 6])
    fi.fi_plan_formats(one_format, [(qo2, kv2, last2, 0)])
    with pytest.raises(fi.Fi355Error) as e:
        fi.fi_plan_formats(one_format, [(qo2, kv2, last2, 0), (qo2, kv2, last2, 2)])
    assert e.value.code == fi.FI_ERR_UNSUPPORTED
    fi.fi_plan_formats(any_formats, [(qo2, kv2, last2, 0), (qo2, kv2, last2, 2)])
    fi.fi_destroy(any_formats)
    fi.fi_destroy(one_format)
    with pytest.raises(fi.Fi355Error) as e:
        make(fi.FI_MODE_DECODE, 4, 8, max_formats=2)
    assert e.value.code == fi.FI_ERR_UNSUPPORTED
    with pytest.raises(fi.Fi355Error) as e:
        make(mode, 4, 8, max_formats=-1)
    assert e.value.code == fi.FI_ERR_INVALID_ARG
