"""CPU replica of the load-balanced work partition (Algorithm 1, Sec. 3.3.1).

TEST INFRASTRUCTURE ONLY.  Pure Python integers, `sorted` and `heapq`; takes
the algorithm's steps in the paper's order.  Shares no code with the C++
planner of the GPU library; the planner's arrays must equal this replica's
bit for bit.

Steps (paper's notation):
  input   {l_qo(i), l_kv(i)}, query tile size T_q
  cost    cost(l_q, l_kv) = alpha * l_q + beta * l_kv
  L_kv    = sum_i ceil(l_qo(i)/T_q) * l_kv(i) / #CTA
  split   every query tile's KV range into chunks of at most L_kv; chunk w has length l_kv(w)
  sort    W = {(w, l_kv(w))} by descending length
  assign  pop the CTA with the least accumulated cost, give it the next chunk,
          add cost(T_q, l_kv(w)) to it, push it back
plus the output index map of Sec. 3.3.1 / App. D.2: a tile with one chunk
writes the final output directly (write-through), a split tile writes one
partial state per chunk into the workspace and is merged afterwards.

Readings where the paper is silent (each is a deliberate choice, listed in the
design notes):
  * heads are left out of the plan (as in Algorithm 1): every kv head runs the
    same work list; #CTA here is the number of CTAs per kv head;
  * a query tile holds T_pos consecutive positions of one request fused with
    the g = H_qo/H_kv heads of a group (App. A), so T_q = T_pos * g rows;
  * under causal masking a tile's KV range is what its last row can see,
    kv_eff = clamp(l_kv - l_qo + tile_end, 0, l_kv); that is the l_kv(i) of
    the tile in the L_kv formula and in the split (`literal_lkv=True` uses
    l_kv(i) for every tile in the L_kv formula as printed);
  * L_kv = max(min_chunk, round_up(ceil(S / #CTA), page_size)); S = 0 gives
    min_chunk.  Rounding up to whole pages keeps chunk starts page aligned and
    keeps the number of partial tiles <= 2 * #CTA (App. D.3);
  * greedy split: chunk c = [c*L_kv, min((c+1)*L_kv, kv_eff)); a tile with
    kv_eff = 0 still gets one (empty) chunk so its rows are written;
  * work indices w are given in (request, tile, chunk) order; sort key
    (-length, w); heap key (cost, cta); alpha, beta integers;
  * a CTA's queue keeps assignment order;
  * split tiles are numbered in (request, tile) order, slot_base is the running
    sum of their chunk counts, chunk c of a split tile owns slot slot_base + c,
    the merge folds slots in ascending c.

Refinement (``refine=True``; an addition of this build, not in the paper, used for
append where a CTA gets only a handful of long items): costs are taken in percent
(``unit = 100``); the chunk length is rounded up to whole tiles of ``kv_quantum``
tokens; an item whose fused rows ``n_pos * group`` fit in ``light_rows`` counts
``light_pct`` percent of its per-token term; after the greedy pass, unless there
are more than ``8 * #CTA`` work items (then the greedy result is kept), up to
``4 * #CTA + 64`` times: take the most loaded CTA (lowest index on ties), and among
all (other CTA, item of the loaded CTA, optional cheaper partner item of the other
CTA) candidates in that nesting order take the first one that gives the smallest new
maximum of the two loads, if it is below the current maximum; move (or swap) it;
stop when there is none.  Moved items go to the end of a queue; at the end every
queue is ordered by (-length, w) again.  ``weighted_lkv=True`` (with the refinement):
in the sum S of the L_kv formula a light tile's KV range counts ``light_pct`` percent
as well (rounded up, tile by tile), so that loads in cost units come out equal when
light and full tiles are planned together.
"""
from __future__ import annotations

import heapq
from typing import Dict, List, Sequence

NO_DIAG = 0x3FFFFFFF   # "row sees everything" marker for non-causal work items


def _requests_of(qo_indptr, kv_indptr, last_page_len, page_size, kv_base=0):
    """(first query row, l_qo, l_kv, index of the first page id) of every request of one format"""
    out = []
    for i in range(len(last_page_len)):
        n_pg = int(kv_indptr[i + 1]) - int(kv_indptr[i])
        l_kv = 0 if n_pg == 0 else (n_pg - 1) * page_size + int(last_page_len[i])
        out.append((int(qo_indptr[i]), int(qo_indptr[i + 1]) - int(qo_indptr[i]), l_kv, kv_base + int(kv_indptr[i])))
    return out


def plan_replica(qo_indptr: Sequence[int], kv_indptr: Sequence[int], last_page_len: Sequence[int], **kw) -> Dict[str, object]:
    """Algorithm 1 over one format (keyword arguments: see _plan)."""
    return _plan(_requests_of(qo_indptr, kv_indptr, last_page_len, kw["page_size"]), composed=False, **kw)


def plan_replica_formats(formats, **kw) -> Dict[str, object]:
    """Several formats over the same query rows (Sec. 3.1.2) planned as one work list: `formats` is a sequence of
    (qo_indptr, kv_indptr, last_page_len, kv_base), kv_base = where the format's page ids start in the one page-id
    array all formats share.  Requests are numbered through the formats in the given order, Algorithm 1 then runs
    unchanged over all their query tiles.  With more than one format (a reading of this build; the paper composes
    formats by merging the states of separate kernels, Sec. 2.2) no tile writes through: every work item writes a
    partial state into its own slot (slots numbered tile by tile, chunk c of a tile at slot_base + c), the merge
    list stays empty, and `row_indptr` / `row_entry` list for every query row the partial states it folds, formats
    in the given order, chunks in ascending KV order, each as slot * t_pos + (row - first row of the tile)."""
    reqs = []
    for (qo_indptr, kv_indptr, last_page_len, kv_base) in formats:
        reqs += _requests_of(qo_indptr, kv_indptr, last_page_len, kw["page_size"], kv_base)
    n_rows = int(formats[0][0][-1])
    assert all(int(f[0][-1]) == n_rows for f in formats), "the formats cover different numbers of query rows"
    return _plan(reqs, composed=len(formats) > 1, n_rows=n_rows, **kw)


def _plan(requests, *, composed: bool, n_rows: int = 0, page_size: int, t_pos: int, group: int, num_ctas: int, causal: bool,
          alpha: int = 1, beta: int = 1, min_chunk: int | None = None,
          literal_lkv: bool = False, refine: bool = False, light_rows: int = 0,
          light_pct: int = 100, kv_quantum: int = 1, plan_window: int = 0,
          item_cost: int = 0, weighted_lkv: bool = False) -> Dict[str, object]:
    B = len(requests)
    if min_chunk is None:
        min_chunk = page_size
    min_chunk = ((min_chunk + page_size - 1) // page_size) * page_size
    T_q = t_pos * group

    # -- lengths -----------------------------------------------------------
    q_row0_of = [r[0] for r in requests]
    l_qo = [r[1] for r in requests]
    l_kv = [r[2] for r in requests]
    page0_of = [r[3] for r in requests]

    # -- query tiles and the KV range each one needs -------------------------
    tiles = []        # (request, tile_start, n_pos, kv_eff, diag0)
    S = 0
    for i in range(B):
        n_tiles = -(-l_qo[i] // t_pos)
        for t in range(n_tiles):
            start = t * t_pos
            end = min(start + t_pos, l_qo[i])
            if causal:
                kv_eff = max(0, min(l_kv[i], l_kv[i] - l_qo[i] + end))
                diag0 = l_kv[i] - l_qo[i] + start
            else:
                kv_eff = l_kv[i]
                diag0 = NO_DIAG
            # sliding window (not in the paper's algorithm): with plan_window = W + 1 > 0 a query at position pos sees
            # keys pos - W .. pos only; the tile's first row sits at l_kv - l_qo + start, so no row of the tile sees
            # a key before kv_begin, which is rounded down to a page boundary (chunks start on pages)
            kv_begin = 0
            if plan_window > 0:
                kv_begin = max(0, l_kv[i] - l_qo[i] + start - (plan_window - 1))
                kv_begin = min(kv_begin, kv_eff) // page_size * page_size
            tiles.append((i, start, end - start, kv_eff, diag0, kv_begin))
            counted = l_kv[i] if literal_lkv else kv_eff - kv_begin
            if weighted_lkv and refine and light_rows > 0 and (end - start) * group <= light_rows:
                counted = -(-counted * light_pct // 100)   # a light tile counts light_pct percent, rounded up
            S += counted

    # -- maximum chunk size --------------------------------------------------
    L_kv = -(-S // num_ctas)
    L_kv = ((L_kv + page_size - 1) // page_size) * page_size
    L_kv = max(min_chunk, L_kv)
    # fixed cost per work item (not in the paper's algorithm): in a batch so small that the chunk length is at most
    # 4 * item_cost tokens, a longer chunk (up to twice, whole pages) is taken when it lowers
    # ceil(#chunks / #CTA) * (item_cost + L); ties keep the shorter chunk
    if item_cost > 0 and L_kv <= 4 * item_cost:
        def estimate(length):
            n = sum(max(1, -(-(t[3] - t[5]) // length)) for t in tiles)
            return -(-n // num_ctas) * (item_cost + length)
        best, best_est = L_kv, estimate(L_kv)
        for length in range(L_kv + page_size, 2 * L_kv + 1, page_size):
            est = estimate(length)
            if est < best_est:
                best, best_est = length, est
        L_kv = best

    # -- split ---------------------------------------------------------------
    work = []         # per w: dict
    tile_chunks = []  # per tile: number of chunks
    for (i, start, n_pos, kv_eff, diag0, kv_begin) in tiles:
        n_chunks = max(1, -(-(kv_eff - kv_begin) // L_kv))
        tile_chunks.append(n_chunks)
        for c in range(n_chunks):
            lo = kv_begin + c * L_kv
            hi = min(lo + L_kv, kv_eff)
            work.append(dict(request=i, q_row0=q_row0_of[i] + start, n_pos=n_pos,
                             kv_start=lo, kv_len=hi - lo,
                             kv_page0=page0_of[i] + lo // page_size,
                             diag0=diag0, tile=len(tile_chunks) - 1, chunk=c))

    # -- output index map ------------------------------------------------------
    slot_base_of_tile = []
    merge_index_of_tile = []
    merge = []        # per split tile: (q_row0, n_pos, slot_base, n_chunks)
    next_slot = 0
    row_lists: List[List[int]] = [[] for _ in range(n_rows)] if composed else []
    for ti, (i, start, n_pos, kv_eff, diag0, kv_begin) in enumerate(tiles):
        if composed:
            # several formats: no write-through, every chunk of every tile owns a slot, and every query row of the
            # tile notes the partial states it will fold
            slot_base_of_tile.append(next_slot)
            merge_index_of_tile.append(-1)
            for pos in range(n_pos):
                row_lists[q_row0_of[i] + start + pos] += [(next_slot + c) * t_pos + pos for c in range(tile_chunks[ti])]
            next_slot += tile_chunks[ti]
        elif tile_chunks[ti] > 1:
            slot_base_of_tile.append(next_slot)
            merge_index_of_tile.append(len(merge))
            merge.append((q_row0_of[i] + start, n_pos, next_slot, tile_chunks[ti]))
            next_slot += tile_chunks[ti]
        else:
            slot_base_of_tile.append(-1)
            merge_index_of_tile.append(-1)
    for w in work:
        base = slot_base_of_tile[w["tile"]]
        w["out_slot"] = -1 if base < 0 else base + w["chunk"]
        w["merge"] = merge_index_of_tile[w["tile"]]     # the split tile this chunk belongs to, for whoever folds it

    # -- sort by descending length, assign to the least-loaded CTA ------------
    order = sorted(range(len(work)), key=lambda w: (-work[w]["kv_len"], w))
    unit = 100 if refine else 1

    def item_cost(w):
        light = refine and light_rows > 0 and work[w]["n_pos"] * group <= light_rows
        l_kv = work[w]["kv_len"]
        if refine:   # the kernel works in whole tiles of kv_quantum tokens
            l_kv = -(-l_kv // kv_quantum) * kv_quantum
        return unit * alpha * T_q + beta * l_kv * (light_pct if light else unit)

    heap = [(0, c) for c in range(num_ctas)]
    heapq.heapify(heap)
    queues: List[List[int]] = [[] for _ in range(num_ctas)]
    for w in order:
        cost, c = heapq.heappop(heap)
        queues[c].append(w)
        heapq.heappush(heap, (cost + item_cost(w), c))
    cta_cost = [0] * num_ctas
    for cost, c in heap:
        cta_cost[c] = cost

    # -- refinement (not in the paper; see the module header) ------------------
    if refine and len(work) <= 8 * num_ctas:
        for _ in range(4 * num_ctas + 64):
            hi = max(range(num_ctas), key=lambda c: (cta_cost[c], -c))     # most loaded, lowest index on ties
            best_new, best = cta_cost[hi], None
            for lo in range(num_ctas):
                if lo == hi:
                    continue
                for ia, a in enumerate(queues[hi]):
                    ca = item_cost(a)
                    moved = max(cta_cost[hi] - ca, cta_cost[lo] + ca)
                    if moved < best_new:
                        best_new, best = moved, (lo, ia, -1)
                    for ib, b_ in enumerate(queues[lo]):
                        cb = item_cost(b_)
                        if cb >= ca:
                            continue
                        swapped = max(cta_cost[hi] - ca + cb, cta_cost[lo] + ca - cb)
                        if swapped < best_new:
                            best_new, best = swapped, (lo, ia, ib)
            if best is None:
                break
            lo, ia, ib = best
            wa = queues[hi].pop(ia)
            cta_cost[hi] -= item_cost(wa)
            cta_cost[lo] += item_cost(wa)
            if ib >= 0:
                wb = queues[lo].pop(ib)
                cta_cost[lo] -= item_cost(wb)
                cta_cost[hi] += item_cost(wb)
                queues[hi].append(wb)
            queues[lo].append(wa)
    if refine:
        for q in queues:
            q.sort(key=lambda w: (-work[w]["kv_len"], w))

    cta_indptr = [0]
    flat = []
    for c in range(num_ctas):
        flat.extend(queues[c])
        cta_indptr.append(len(flat))

    def col(name):
        return [work[w][name] for w in flat]

    rows = {}
    if composed:
        row_indptr = [0]
        for lst in row_lists:
            row_indptr.append(row_indptr[-1] + len(lst))
        rows = dict(n_rows=n_rows, row_indptr=row_indptr, row_entry=[e for lst in row_lists for e in lst])
    return dict(
        **rows,
        L_kv=L_kv, S=S, n_work=len(work), n_merge=len(merge), n_slots=next_slot,
        cta_indptr=cta_indptr,
        w_request=col("request"), w_q_row0=col("q_row0"), w_n_pos=col("n_pos"),
        w_kv_page0=col("kv_page0"), w_kv_start=col("kv_start"), w_kv_len=col("kv_len"),
        w_diag0=col("diag0"), w_out_slot=col("out_slot"), w_merge=col("merge"),
        m_q_row0=[m[0] for m in merge], m_n_pos=[m[1] for m in merge],
        m_slot_base=[m[2] for m in merge], m_n_chunks=[m[3] for m in merge],
        cta_cost=cta_cost, work_order=flat,
    )
