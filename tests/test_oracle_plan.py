"""Pins for the replica of the paper's scheduling algorithm (Algorithm 1, Sec. 3.3.1):
pencil-worked examples stored as text fixtures (two of the algorithm as printed, four of the
planner's additions: fixed item cost, sliding window, refined assignment), and the invariants the paper
states (App. D.2 write-through, App. D.3 partial-output bound, determinism)."""
import os

import numpy as np
import pytest

from oracle.plan_replica import NO_DIAG, plan_replica

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def load_fixture(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


def indptrs_from_lengths(qo_len, kv_len, page_size):
    qo_indptr = np.concatenate([[0], np.cumsum(qo_len)]).astype(np.int64)
    n_pg = [(l + page_size - 1) // page_size for l in kv_len]
    kv_indptr = np.concatenate([[0], np.cumsum(n_pg)]).astype(np.int64)
    last = [0 if l == 0 else l - (n - 1) * page_size for l, n in zip(kv_len, n_pg)]
    return qo_indptr, kv_indptr, last


# as printed in the paper (the first two) and the planner's additions: the fixed cost per work item of the default
# decode plan, the sliding window known to the planner, the refined assignment (one move and two swaps fire)
HAND_WORKED = ["plan_decode_example.txt", "plan_causal_example.txt", "plan_item_cost_example.txt",
               "plan_window_decode_example.txt", "plan_window_causal_example.txt", "plan_refine_example.txt"]
FIXTURE_KEYS = ("cta_indptr", "w_request", "w_q_row0", "w_n_pos", "w_kv_page0", "w_kv_start", "w_kv_len", "w_diag0",
                "w_out_slot", "w_merge", "cta_cost", "m_q_row0", "m_n_pos", "m_slot_base", "m_n_chunks")


def replica_args(fx):
    ps = fx["page_size"][0]
    opt = lambda k, d: fx.get(k, [d])[0]
    return dict(page_size=ps, t_pos=fx["t_pos"][0], group=fx["group"][0], num_ctas=fx["num_ctas"][0],
                causal=bool(fx["causal"][0]), alpha=opt("alpha", 1), beta=opt("beta", 1), min_chunk=opt("min_chunk", ps),
                refine=bool(opt("refine", 0)), light_rows=opt("light_rows", 0), light_pct=opt("light_pct", 100),
                kv_quantum=opt("kv_quantum", 1), plan_window=opt("plan_window", 0), item_cost=opt("item_cost", 0),
                weighted_lkv=bool(opt("weighted_lkv", 0)))


@pytest.mark.parametrize("name", HAND_WORKED)
def test_hand_worked_examples(name):
    fx = load_fixture(name)
    qo_indptr, kv_indptr, last = indptrs_from_lengths(fx["qo_len"], fx["kv_len"], fx["page_size"][0])
    p = plan_replica(qo_indptr, kv_indptr, last, **replica_args(fx))
    assert p["L_kv"] == fx["L_kv"][0]
    for key in FIXTURE_KEYS:
        if key in fx:
            assert list(p[key]) == fx[key], key


def test_item_cost_example_differs_from_the_algorithm_as_printed():
    # the same lengths without the fixed item cost: Algorithm 1's own chunk length (64) and five work items
    fx = load_fixture("plan_item_cost_example.txt")
    qo_indptr, kv_indptr, last = indptrs_from_lengths(fx["qo_len"], fx["kv_len"], 16)
    p = plan_replica(qo_indptr, kv_indptr, last, **{**replica_args(fx), "item_cost": 0})
    assert p["L_kv"] == 64 and p["n_work"] == 5 and p["w_kv_len"] == [64, 64, 60, 50, 2]


def random_lengths(rng, kind):
    B = int(rng.integers(1, 40))
    if kind == "decode":
        qo = np.ones(B, dtype=np.int64)
        kv = rng.integers(0, 3000, size=B)
        if rng.random() < 0.3:
            kv[rng.integers(0, B)] = int(rng.integers(20000, 200000))      # one giant request
        if rng.random() < 0.2:
            kv[:] = int(rng.integers(1, 500))                              # all equal
    else:
        qo = rng.integers(0, 300, size=B)
        pre = rng.integers(0, 2000, size=B)
        kv = qo + pre
        if rng.random() < 0.3:
            kv = np.maximum(kv - rng.integers(0, 50, size=B), 0)           # fewer keys than queries allowed
    return qo, kv


@pytest.mark.parametrize("kind", ["decode", "append"])
def test_invariants_random(kind):
    rng = np.random.default_rng(2024 if kind == "decode" else 2025)
    for trial in range(150):
        qo, kv = random_lengths(rng, kind)
        ps = int(rng.choice([1, 4, 16]))
        C = int(rng.choice([1, 3, 8, 32, 128]))
        t_pos = 1 if kind == "decode" else int(rng.choice([16, 32, 128]))
        g = int(rng.choice([1, 4]))
        causal = kind == "append"
        alpha, beta = int(rng.integers(0, 4)), int(rng.integers(1, 4))
        min_chunk = ps * int(rng.choice([1, 4, 16]))
        qo_indptr, kv_indptr, last = indptrs_from_lengths(qo, kv, ps)
        kw = dict(page_size=ps, t_pos=t_pos, group=g, num_ctas=C, causal=causal, alpha=alpha, beta=beta,
                  min_chunk=min_chunk)
        if trial % 3 == 2:
            # a fixed cost per work item may lengthen the chunks of a small batch, never beyond twice the length
            # of Algorithm 1 and never to more rounds of work items; everything below holds for that plan too
            kw["item_cost"] = int(rng.choice([16, 64, 1000]))
            printed = plan_replica(qo_indptr, kv_indptr, last, **{**kw, "item_cost": 0})
            longer = plan_replica(qo_indptr, kv_indptr, last, **kw)
            assert printed["L_kv"] <= longer["L_kv"] <= 2 * printed["L_kv"]
            assert -(-longer["n_work"] // C) <= -(-printed["n_work"] // C)
            if printed["L_kv"] > 4 * kw["item_cost"]:
                assert longer == printed
        p = plan_replica(qo_indptr, kv_indptr, last, **kw)
        assert p == plan_replica(qo_indptr, kv_indptr, last, **kw)          # deterministic (Sec. 3.3.1)
        L = p["L_kv"]
        assert L % ps == 0 and L >= min_chunk and L * C >= p["S"]
        n_work = p["n_work"]
        assert p["cta_indptr"][0] == 0 and p["cta_indptr"][-1] == n_work and len(p["cta_indptr"]) == C + 1
        assert sorted(p["work_order"]) == list(range(n_work))               # each item assigned once
        # chunks of a tile partition [0, kv_eff) and every chunk is <= L_kv
        tiles = {}
        for k in range(n_work):
            key = (p["w_request"][k], p["w_q_row0"][k])
            tiles.setdefault(key, []).append(k)
            assert 0 <= p["w_kv_len"][k] <= L
            assert p["w_kv_start"][k] % ps == 0
            i = p["w_request"][k]
            assert p["w_kv_page0"][k] == kv_indptr[i] + p["w_kv_start"][k] // ps
        n_tiles_expected = int(sum(-(-int(q) // t_pos) for q in qo))
        assert len(tiles) == n_tiles_expected
        n_slots = 0
        n_split = 0
        for (i, row0), items in tiles.items():
            items.sort(key=lambda k: p["w_kv_start"][k])
            start = row0 - int(qo_indptr[i])
            end = min(start + t_pos, int(qo[i]))
            kv_eff = max(0, min(int(kv[i]), int(kv[i]) - int(qo[i]) + end)) if causal else int(kv[i])
            pos = 0
            for k in items:
                assert p["w_kv_start"][k] == pos
                assert p["w_n_pos"][k] == end - start
                assert p["w_diag0"][k] == (int(kv[i]) - int(qo[i]) + start if causal else NO_DIAG)
                pos += p["w_kv_len"][k]
            assert pos == kv_eff
            assert (len(items) > 1) == (kv_eff > L)                           # split iff longer than L_kv
            if len(items) == 1:
                assert p["w_out_slot"][items[0]] == -1                        # write-through (App. D.2)
            else:
                slots = [p["w_out_slot"][k] for k in items]
                assert slots == list(range(slots[0], slots[0] + len(items)))
                assert all(p["w_kv_len"][k] == L for k in items[:-1])          # greedy: only the last is short
                n_slots += len(items)
                n_split += 1
        assert n_slots == p["n_slots"] <= 2 * C                                # App. D.3
        assert p["n_merge"] == n_split <= C
        assert sum(p["m_n_chunks"]) == n_slots
        # LPT property: no CTA exceeds the least-loaded one by more than one item's cost
        T_q = t_pos * g
        costs = p["cta_cost"]
        loads = [0] * C
        for c in range(C):
            for k in range(p["cta_indptr"][c], p["cta_indptr"][c + 1]):
                loads[c] += alpha * T_q + beta * p["w_kv_len"][k]
        assert loads == costs
        if n_work:
            max_item = max(alpha * T_q + beta * l for l in p["w_kv_len"])
            assert max(loads) - min(loads) <= max_item
        # queues hold items longest first
        for c in range(C):
            lens = p["w_kv_len"][p["cta_indptr"][c]:p["cta_indptr"][c + 1]]
            assert lens == sorted(lens, reverse=True)


@pytest.mark.parametrize("kind", ["decode", "append"])
def test_refined_assignment_keeps_the_partition_and_never_raises_the_maximum(kind):
    # the refinement (an addition of this build) moves whole work items between queues: the chunks, the slots and
    # the merge list are those of Algorithm 1; under its own cost the maximum load is never above the greedy one
    rng = np.random.default_rng(77 if kind == "decode" else 78)
    improved = 0
    for trial in range(120):
        qo, kv = random_lengths(rng, kind)
        ps, C = 16, int(rng.choice([2, 3, 8, 32]))
        t_pos = 1 if kind == "decode" else int(rng.choice([16, 64]))
        g = int(rng.choice([1, 4]))
        alpha, beta = int(rng.integers(0, 9)), int(rng.integers(1, 6))
        light_rows = 0 if kind == "decode" else (t_pos * g) // 2
        qo_indptr, kv_indptr, last = indptrs_from_lengths(qo, kv, ps)
        kw = dict(page_size=ps, t_pos=t_pos, group=g, num_ctas=C, causal=kind == "append", alpha=alpha, beta=beta,
                  min_chunk=16)
        base = plan_replica(qo_indptr, kv_indptr, last, **kw)
        ref = plan_replica(qo_indptr, kv_indptr, last, refine=True, light_rows=light_rows, light_pct=64, **kw)
        assert ref == plan_replica(qo_indptr, kv_indptr, last, refine=True, light_rows=light_rows, light_pct=64, **kw)
        for k in ("L_kv", "S", "n_work", "n_merge", "n_slots", "m_q_row0", "m_n_pos", "m_slot_base", "m_n_chunks"):
            assert ref[k] == base[k], k
        item = lambda p, k: (p["w_request"][k], p["w_q_row0"][k], p["w_n_pos"][k], p["w_kv_page0"][k],
                             p["w_kv_start"][k], p["w_kv_len"][k], p["w_diag0"][k], p["w_out_slot"][k])
        assert sorted(item(ref, k) for k in range(ref["n_work"])) == sorted(item(base, k) for k in range(base["n_work"]))
        assert ref["cta_indptr"][0] == 0 and ref["cta_indptr"][-1] == ref["n_work"]

        def cost(p, k):   # the refined cost, in percent
            light = light_rows > 0 and p["w_n_pos"][k] * g <= light_rows
            return 100 * alpha * t_pos * g + beta * p["w_kv_len"][k] * (64 if light else 100)

        def loads(p):
            return [sum(cost(p, k) for k in range(p["cta_indptr"][c], p["cta_indptr"][c + 1])) for c in range(C)]

        assert loads(ref) == ref["cta_cost"]
        assert max(loads(ref)) <= max(loads(base)) or light_rows > 0   # with light tiles the greedy pass itself differs
        improved += max(loads(ref)) < max(loads(base))
        for c in range(C):
            lens = ref["w_kv_len"][ref["cta_indptr"][c]:ref["cta_indptr"][c + 1]]
            assert lens == sorted(lens, reverse=True)
    assert improved > 10


def test_refined_assignment_balances_the_append_workload():
    # lengths of the causal-append benchmark workload: 154 items on 32 CTAs; greedy leaves 5.9 %, the refinement
    # well under 1 % (loads in the planner's own cost: 8 * T_q + 5 * l_kv, light tiles at 64 %)
    g3 = np.random.Generator(np.random.PCG64(1003))
    qo = g3.integers(128, 1025, size=16)
    pre = g3.integers(0, 4097, size=16)
    pre[1] = 0
    if qo[2] % 128 == 0:
        qo[2] += 37
    qo_indptr, kv_indptr, last = indptrs_from_lengths(qo, qo + pre, 16)
    kw = dict(page_size=16, t_pos=64, group=4, num_ctas=32, causal=True, alpha=8, beta=5, min_chunk=256)
    ref = plan_replica(qo_indptr, kv_indptr, last, refine=True, light_rows=128, light_pct=64, kv_quantum=64, **kw)
    base = plan_replica(qo_indptr, kv_indptr, last, **kw)

    def loads(p):
        out = []
        for c in range(32):
            t = 0
            for k in range(p["cta_indptr"][c], p["cta_indptr"][c + 1]):
                t += 100 * 8 * 256 + 5 * -(-p["w_kv_len"][k] // 64) * 64 * (64 if p["w_n_pos"][k] * 4 <= 128 else 100)
            out.append(t)
        return np.array(out, dtype=np.float64)

    lb, lr = loads(base), loads(ref)
    assert lb.max() / lb.mean() > 1.04
    assert lr.max() / lr.mean() < 1.01
    assert lr.sum() == lb.sum()


def test_long_context_split_is_balanced():
    # two long requests over 32 CTAs: greedy chunks give 31 full + two short pieces that share a CTA
    qo_indptr, kv_indptr, last = indptrs_from_lengths([1, 1], [131072, 65536], 16)
    p = plan_replica(qo_indptr, kv_indptr, last, page_size=16, t_pos=1, group=4, num_ctas=32, causal=False)
    assert p["L_kv"] == 6144
    assert p["n_work"] == 33 and p["n_slots"] == 33
    # 31 CTAs hold one full chunk (cost 4 + 6144); the last holds 4096 + 2048 (cost 2 * 4 + 6144)
    assert sorted(p["cta_cost"]) == [6148] * 31 + [6152]


def test_literal_lkv_flag_only_changes_chunk_size():
    qo_indptr, kv_indptr, last = indptrs_from_lengths([256], [256], 16)
    a = plan_replica(qo_indptr, kv_indptr, last, page_size=16, t_pos=32, group=4, num_ctas=4, causal=True)
    b = plan_replica(qo_indptr, kv_indptr, last, page_size=16, t_pos=32, group=4, num_ctas=4, causal=True,
                     literal_lkv=True)
    assert a["S"] == sum(32 * (t + 1) for t in range(8)) and b["S"] == 8 * 256
    assert b["L_kv"] > a["L_kv"]


def test_empty_and_degenerate_inputs():
    # no requests with queries -> no work, L_kv = min_chunk
    p = plan_replica([0, 0], [0, 3], [5], page_size=16, t_pos=1, group=1, num_ctas=4, causal=False)
    assert p["n_work"] == 0 and p["L_kv"] == 16 and p["cta_indptr"] == [0, 0, 0, 0, 0]
    # a request with no pages still gets one empty work item (its rows must be written)
    p = plan_replica([0, 1], [0, 0], [0], page_size=16, t_pos=1, group=1, num_ctas=2, causal=False)
    assert p["n_work"] == 1 and p["w_kv_len"] == [0] and p["w_out_slot"] == [-1]


def test_sliding_window_leaves_out_exactly_the_pages_no_row_sees():
    """plan_window = W + 1: the chunks of a tile cover [kv_begin, kv_eff) without gaps, kv_begin is a page boundary, no
    row of the tile sees a key before it, and it is the last page boundary with that property; a window wider
    than the context changes nothing."""
    rng = np.random.default_rng(23)
    for causal, t_pos in ((False, 1), (True, 64)):
        for trial in range(40):
            B = int(rng.integers(1, 12))
            qo = np.ones(B, dtype=np.int64) if not causal else rng.integers(1, 300, size=B)
            kv = qo + rng.integers(0, 3000, size=B)
            W = int(rng.integers(0, 1500))
            qo_indptr, kv_indptr, last = indptrs_from_lengths([int(x) for x in qo], [int(x) for x in kv], 16)
            kw = dict(page_size=16, t_pos=t_pos, group=4, num_ctas=int(rng.integers(1, 40)), causal=causal, min_chunk=32)
            p = plan_replica(qo_indptr, kv_indptr, last, plan_window=W + 1, **kw)
            by_tile = {}
            for k in range(p["n_work"]):
                by_tile.setdefault((p["w_request"][k], p["w_q_row0"][k]), []).append(k)
            for (i, q_row0), items in by_tile.items():
                items.sort(key=lambda k: p["w_kv_start"][k])
                start = q_row0 - int(qo_indptr[i])
                first_pos = int(kv[i]) - int(qo[i]) + start              # position of the tile's first row
                kv_begin = p["w_kv_start"][items[0]]
                assert kv_begin % 16 == 0 and kv_begin <= max(0, first_pos - W)
                assert kv_begin + 16 > max(0, first_pos - W) or p["w_kv_len"][items[0]] == 0
                end = kv_begin
                for k in items:
                    assert p["w_kv_start"][k] == end
                    assert p["w_kv_page0"][k] == int(kv_indptr[i]) + end // 16
                    end += p["w_kv_len"][k]
                n_pos = p["w_n_pos"][items[0]]
                assert end == (min(int(kv[i]), first_pos + n_pos) if causal else int(kv[i]))
            wide = plan_replica(qo_indptr, kv_indptr, last, plan_window=10 ** 7, **kw)
            none = plan_replica(qo_indptr, kv_indptr, last, **kw)
            assert all(wide[k] == none[k] for k in none)


def formats_of_fixture(fx):
    out = []
    for f in range(fx["n_formats"][0]):
        qo_indptr, kv_indptr, last = indptrs_from_lengths(fx[f"f{f}_qo_len"], fx[f"f{f}_kv_len"], fx["page_size"][0])
        out.append((qo_indptr, kv_indptr, last, fx[f"f{f}_kv_base"][0]))
    return out


# (the second: light tiles at 30 percent in the chunk length and in the costs, and one swap of the refinement)
@pytest.mark.parametrize("name", ["plan_formats_example.txt", "plan_weighted_formats_example.txt"])
def test_hand_worked_plan_over_two_formats(name):
    from oracle.plan_replica import plan_replica_formats
    fx = load_fixture(name)
    p = plan_replica_formats(formats_of_fixture(fx), **replica_args(fx))
    assert p["L_kv"] == fx["L_kv"][0] and p["n_slots"] == fx["n_slots"][0] and p["n_merge"] == 0
    for key in FIXTURE_KEYS + ("row_indptr", "row_entry"):
        if key in fx:
            assert list(p[key]) == fx[key], key


def test_plans_over_several_formats_keep_the_invariants():
    """Random shared-prefix style batches: one work list over all formats; every chunk of every tile owns exactly
    one slot; every query row lists, per format in order, the chunks of the tile that holds it, in ascending KV
    order; one format alone is the single-format plan."""
    from oracle.plan_replica import plan_replica_formats
    rng = np.random.default_rng(31)
    for trial in range(60):
        g = int(rng.choice([1, 2, 4, 8]))
        t_pos, ps = 16 // g, 16
        C = int(rng.choice([1, 3, 16, 64]))
        n_rows = int(rng.integers(1, 40))
        formats, lens = [], []
        n_formats = int(rng.integers(1, 4))
        base = 0
        for f in range(n_formats):
            # cut the rows into requests at random places
            cuts = sorted(set(rng.integers(0, n_rows + 1, size=int(rng.integers(0, n_rows + 1))).tolist()) | {0, n_rows})
            qo = np.diff(cuts)
            kv = rng.integers(0, 700, size=len(qo))
            qo_indptr, kv_indptr, last = indptrs_from_lengths(qo, kv, ps)
            formats.append((qo_indptr, kv_indptr, last, base))
            lens.append((qo, kv))
            base += int(kv_indptr[-1])
        kw = dict(page_size=ps, t_pos=t_pos, group=g, num_ctas=C, causal=False, min_chunk=16)
        p = plan_replica_formats(formats, **kw)
        assert p == plan_replica_formats(formats, **kw)
        if n_formats == 1:
            assert p == plan_replica(formats[0][0], formats[0][1], formats[0][2], **kw)
            continue
        assert p["n_merge"] == 0 and p["n_slots"] == p["n_work"] and sorted(p["w_out_slot"]) == list(range(p["n_work"]))
        assert p["n_rows"] == n_rows and len(p["row_indptr"]) == n_rows + 1
        # state (slot, position) -> the work item that writes it
        by_slot = {p["w_out_slot"][k]: k for k in range(p["n_work"])}
        req_base = np.concatenate([[0], np.cumsum([len(f[2]) for f in formats])])
        for r in range(n_rows):
            entries = p["row_entry"][p["row_indptr"][r]:p["row_indptr"][r + 1]]
            seen_formats = []
            covered = {}
            for e in entries:
                k = by_slot[e // t_pos]
                assert p["w_q_row0"][k] + e % t_pos == r and e % t_pos < p["w_n_pos"][k]
                f = int(np.searchsorted(req_base, p["w_request"][k], side="right")) - 1
                seen_formats.append(f)
                covered.setdefault(f, []).append((p["w_kv_start"][k], p["w_kv_len"][k]))
            assert seen_formats == sorted(seen_formats) and set(seen_formats) == set(range(n_formats))
            for f, chunks in covered.items():
                # the chunks of the row's tile in format f, in ascending order, cover its request's keys exactly
                i = int(np.searchsorted(formats[f][0], r, side="right")) - 1
                pos = 0
                for (start, length) in chunks:
                    assert start == pos
                    pos += length
                assert pos == int(lens[f][1][i])
