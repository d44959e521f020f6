// Load-balanced partition of KV ranges over a fixed number of CTAs: Algorithm 1 of
// Sec. 3.3.1, with the output index map of App. D.2 (write-through for unsplit tiles)
// and the slot bound of App. D.3.  Heads are left out, as in the paper: every kv head
// executes the same queues.
#include "plan.h"

#include <algorithm>
#include <utility>
#include <vector>

#include "../../include/fi355.h"

namespace fi355 {

static size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

void WorkspaceLayout::init(int32_t ctas, int32_t max_qo_tiles, int32_t t_pos, int32_t num_qo_heads,
                           int32_t num_kv_heads, int32_t head_dim, bool formats, int32_t chunk_factor) {
  ctas_per_head = ctas;
  // sum_t ceil(kv_eff(t) / L_kv) <= n_tiles + S / L_kv <= n_tiles + #CTA; with PlanParams::weighted_lkv the sum
  // that sets L_kv counts a light tile's tokens light_pct percent, so S / L_kv <= #CTA * 100 / light_pct
  // (chunk_factor = that ratio rounded up)
  max_work = max_qo_tiles + chunk_factor * ctas;
  max_merge = chunk_factor * ctas;
  // App. D.3: at most 2 * #CTA partial states when unsplit tiles write through; composed formats have no
  // write-through, there every work item owns a slot
  max_slots = formats ? max_work : 2 * chunk_factor * ctas;
  size_t o = 0;
  off_header = o;
  o += kHeaderInts;
  off_cta_indptr = o;
  o += static_cast<size_t>(ctas) + 1;
  for (int a = 0; a < kWorkArrays; ++a) {
    off_work[a] = o;
    o += static_cast<size_t>(max_work);
  }
  for (int a = 0; a < kMergeArrays; ++a) {
    off_merge[a] = o;
    o += static_cast<size_t>(max_merge);
  }
  off_counters = o;
  o += static_cast<size_t>(max_merge) * num_kv_heads;
  max_rows = 0;
  if (formats) {
    max_rows = max_qo_tiles * t_pos;
    off_row_indptr = o;
    o += static_cast<size_t>(max_rows) + 1;
    off_row_entry = o;
    o += static_cast<size_t>(max_work) * t_pos;
  }
  plan_ints = o;
  plan_bytes = round_up(o * sizeof(int32_t), 256);
  const size_t rows = static_cast<size_t>(max_slots) * t_pos * num_qo_heads;
  off_part_lse = plan_bytes;
  off_part_o = round_up(off_part_lse + rows * sizeof(float), 256);
  total_bytes = round_up(off_part_o + rows * head_dim * sizeof(float), 256);
}

namespace {
struct Tile {
  int32_t request, start, n_pos, kv_eff, kv_begin, diag0, q_row0, kv_page_base;
  int32_t n_chunks, slot_base, merge_index;
};
struct Chunk {
  int32_t tile, kv_start, kv_len, in_tile;
};
using Entry = std::pair<int64_t, int32_t>;  // (accumulated cost, cta)

// Working arrays of make_plan, kept per thread between calls: planning runs once per generation step on the
// host (Sec. 3.3.1), in front of every layer's launches, so it does not allocate once the sizes have settled.
struct Scratch {
  std::vector<Tile> tiles;
  std::vector<Chunk> chunks;
  std::vector<int32_t> order, cta_of, fill;
  std::vector<int64_t> cost, load;
  std::vector<uint64_t> keys;
  std::vector<Entry> heap;
  std::vector<std::vector<int32_t>> queues;
};
thread_local Scratch scratch;

// the root of a binary min-heap has grown: restore the heap order
void sift_down(std::vector<Entry>& heap) {
  const size_t n = heap.size();
  const Entry e = heap[0];
  size_t i = 0;
  for (;;) {
    size_t c = 2 * i + 1;
    if (c >= n) break;
    if (c + 1 < n && heap[c + 1] < heap[c]) ++c;
    if (!(heap[c] < e)) break;
    heap[i] = heap[c];
    i = c;
  }
  heap[i] = e;
}
}  // namespace

int32_t make_plan(const PlanParams& pp, const WorkspaceLayout& L, const int32_t* qo_indptr,
                  const int32_t* kv_indptr, const int32_t* last_page_len, int32_t batch,
                  int32_t* plan, std::string* err) {
  FormatView f;
  f.qo_indptr = qo_indptr;
  f.kv_indptr = kv_indptr;
  f.last_page_len = last_page_len;
  f.batch = batch;
  return make_plan_formats(pp, L, &f, 1, plan, err);
}

int32_t make_plan_formats(const PlanParams& pp, const WorkspaceLayout& L, const FormatView* formats,
                          int32_t n_formats, int32_t* plan, std::string* err) {
  auto fail = [&](int32_t code, const std::string& msg) {
    if (err) *err = msg;
    return code;
  };
  if (!formats || n_formats < 1 || !plan) return fail(FI_ERR_INVALID_ARG, "fi_plan: null array");
  const bool composed = n_formats > 1;
  if (composed && L.max_rows == 0)
    return fail(FI_ERR_UNSUPPORTED, "fi_plan_formats: the handle's mode plans one format at a time");
  int64_t batch_total = 0;
  for (int32_t f = 0; f < n_formats; ++f) {
    const FormatView& F = formats[f];
    if (!F.qo_indptr || !F.kv_indptr || (F.batch > 0 && !F.last_page_len)) return fail(FI_ERR_INVALID_ARG, "fi_plan: null array");
    if (F.batch < 0) return fail(FI_ERR_INVALID_ARG, "fi_plan: negative batch");
    if (F.qo_indptr[0] != 0 || F.kv_indptr[0] != 0) return fail(FI_ERR_INVALID_ARG, "fi_plan: indptr[0] must be 0");
    if (F.kv_base < 0) return fail(FI_ERR_INVALID_ARG, "fi_plan_formats: negative kv_indices_base");
    if (F.qo_indptr[F.batch] != formats[0].qo_indptr[formats[0].batch])
      return fail(FI_ERR_INVALID_ARG, "fi_plan_formats: the formats cover different numbers of query rows");
    batch_total += F.batch;
  }
  if (batch_total > pp.max_batch)
    return fail(FI_ERR_INVALID_ARG, "fi_plan: batch " + std::to_string(batch_total) + " outside [0, max_batch=" +
                                        std::to_string(pp.max_batch) + "]");
  const int64_t n_rows = formats[0].qo_indptr[formats[0].batch];
  if (composed && n_rows > L.max_rows)
    return fail(FI_ERR_INVALID_ARG, "fi_plan_formats: more query rows than max_qo_tiles * tile positions");

  const int32_t ps = pp.page_size;
  const int64_t C = pp.ctas_per_head;

  // ---- lengths, query tiles, and the KV range each tile needs ----
  std::vector<Tile>& tiles = scratch.tiles;
  tiles.clear();
  int64_t S = 0;
  int32_t request_base = 0;  // requests are counted through all formats
  for (int32_t f = 0; f < n_formats; request_base += formats[f].batch, ++f) {
    const int32_t* qo_indptr = formats[f].qo_indptr;
    const int32_t* kv_indptr = formats[f].kv_indptr;
    const int32_t* last_page_len = formats[f].last_page_len;
    const int32_t batch = formats[f].batch;
    for (int32_t i = 0; i < batch; ++i) {
      const int64_t l_qo = static_cast<int64_t>(qo_indptr[i + 1]) - qo_indptr[i];
      const int64_t n_pg = static_cast<int64_t>(kv_indptr[i + 1]) - kv_indptr[i];
      if (l_qo < 0 || n_pg < 0)
        return fail(FI_ERR_INVALID_ARG, "fi_plan: indptr decreases at request " + std::to_string(i));
      if (n_pg > 0 && (last_page_len[i] < 1 || last_page_len[i] > ps))
        return fail(FI_ERR_INVALID_ARG, "fi_plan: last_page_len[" + std::to_string(i) + "] = " +
                                            std::to_string(last_page_len[i]) + " outside [1, page_size]");
      const int64_t l_kv = n_pg == 0 ? 0 : (n_pg - 1) * ps + last_page_len[i];
      if (l_kv >= kNoDiag) return fail(FI_ERR_INVALID_ARG, "fi_plan: request too long");
      const int64_t n_tiles = (l_qo + pp.t_pos - 1) / pp.t_pos;
      if (static_cast<int64_t>(tiles.size()) + n_tiles > pp.max_qo_tiles)
        return fail(FI_ERR_INVALID_ARG, "fi_plan: more query tiles than max_qo_tiles=" + std::to_string(pp.max_qo_tiles));
      for (int64_t t = 0; t < n_tiles; ++t) {
        Tile tl;
        tl.request = request_base + i;
        tl.start = static_cast<int32_t>(t * pp.t_pos);
        const int64_t end = std::min<int64_t>(tl.start + pp.t_pos, l_qo);
        tl.n_pos = static_cast<int32_t>(end - tl.start);
        if (pp.causal) {
          tl.kv_eff = static_cast<int32_t>(std::max<int64_t>(0, std::min<int64_t>(l_kv, l_kv - l_qo + end)));
          tl.diag0 = static_cast<int32_t>(l_kv - l_qo + tl.start);
        } else {
          tl.kv_eff = static_cast<int32_t>(l_kv);
          tl.diag0 = kNoDiag;
        }
        tl.kv_begin = 0;
        if (pp.plan_window > 0) {
          const int64_t first_seen = std::max<int64_t>(0, l_kv - l_qo + tl.start - (pp.plan_window - 1));
          tl.kv_begin = static_cast<int32_t>(std::min<int64_t>(first_seen, tl.kv_eff) / ps * ps);
        }
        tl.q_row0 = qo_indptr[i] + tl.start;
        tl.kv_page_base = formats[f].kv_base + kv_indptr[i];
        tl.n_chunks = 1;
        tl.slot_base = -1;
        tl.merge_index = -1;
        tiles.push_back(tl);
        int64_t counted = pp.literal_lkv ? l_kv : tl.kv_eff - tl.kv_begin;
        if (pp.weighted_lkv && pp.refine && pp.light_rows > 0 && static_cast<int64_t>(tl.n_pos) * pp.group <= pp.light_rows)
          counted = (counted * pp.light_pct + 99) / 100;
        S += counted;
      }
    }
  }

  // ---- maximum chunk size L_kv: S / #CTA, whole pages, at least min_chunk ----
  const int64_t min_chunk = (static_cast<int64_t>(pp.min_chunk) + ps - 1) / ps * ps;
  int64_t Lkv = (S + C - 1) / C;
  Lkv = (Lkv + ps - 1) / ps * ps;
  Lkv = std::max(min_chunk, Lkv);
  if (pp.item_cost > 0 && Lkv <= 4 * static_cast<int64_t>(pp.item_cost)) {
    auto estimate = [&](int64_t len) {
      int64_t n = 0;
      for (const Tile& tl : tiles) n += std::max<int64_t>(1, (tl.kv_eff - tl.kv_begin + len - 1) / len);
      return (n + C - 1) / C * (pp.item_cost + len);
    };
    int64_t best = Lkv, best_est = estimate(Lkv);
    for (int64_t len = Lkv + ps; len <= 2 * Lkv; len += ps) {
      const int64_t est = estimate(len);
      if (est < best_est) {
        best = len;
        best_est = est;
      }
    }
    Lkv = best;
  }

  // ---- split every tile's KV range into chunks of at most L_kv; number the chunks ----
  std::vector<Chunk>& chunks = scratch.chunks;
  chunks.clear();
  int32_t next_slot = 0, n_merge = 0;
  for (size_t ti = 0; ti < tiles.size(); ++ti) {
    Tile& tl = tiles[ti];
    tl.n_chunks = static_cast<int32_t>(std::max<int64_t>(1, (tl.kv_eff - tl.kv_begin + Lkv - 1) / Lkv));
    if (composed) {  // every state is a partial state; the row lists below say who folds what
      tl.slot_base = next_slot;
      next_slot += tl.n_chunks;
    } else if (tl.n_chunks > 1) {
      tl.slot_base = next_slot;
      next_slot += tl.n_chunks;
      tl.merge_index = n_merge++;
    }
    for (int32_t c = 0; c < tl.n_chunks; ++c) {
      Chunk ch;
      ch.tile = static_cast<int32_t>(ti);
      ch.kv_start = static_cast<int32_t>(tl.kv_begin + c * Lkv);
      ch.kv_len = static_cast<int32_t>(std::min<int64_t>(ch.kv_start + Lkv, tl.kv_eff) - ch.kv_start);
      ch.in_tile = c;
      chunks.push_back(ch);
    }
  }
  const int32_t n_work = static_cast<int32_t>(chunks.size());
  if (n_work > L.max_work || next_slot > L.max_slots || n_merge > L.max_merge)
    return fail(FI_ERR_WORKSPACE_TOO_SMALL, "fi_plan: plan exceeds the workspace sections (internal bound)");

  // ---- descending length (ties: lower work index first) ----
  std::vector<uint64_t>& keys = scratch.keys;  // (largest length first, then the work index) as one integer
  keys.resize(n_work);
  for (int32_t w = 0; w < n_work; ++w)
    keys[w] = (static_cast<uint64_t>(0x7fffffff - chunks[w].kv_len) << 32) | static_cast<uint32_t>(w);
  std::sort(keys.begin(), keys.end());
  std::vector<int32_t>& order = scratch.order;
  order.resize(n_work);
  for (int32_t i = 0; i < n_work; ++i) order[i] = static_cast<int32_t>(keys[i] & 0xffffffffu);

  // ---- least-loaded CTA first (ties: lower CTA index) ----
  std::vector<Entry>& heap = scratch.heap;  // binary min-heap, least (cost, cta) at the root
  heap.resize(static_cast<size_t>(C));
  for (int32_t c = 0; c < C; ++c) heap[c] = {0, c};  // ascending, hence already in heap order
  const int64_t t_q = static_cast<int64_t>(pp.t_pos) * pp.group;
  // cost(l_q, l_kv) = alpha * T_q + beta * l_kv; with the refinement in percent, the per-token term of a
  // light tile weighted by light_pct
  const int64_t unit = pp.refine ? 100 : 1;
  std::vector<int64_t>& cost = scratch.cost;
  cost.resize(static_cast<size_t>(n_work));
  for (int32_t w = 0; w < n_work; ++w) {
    const Tile& tl = tiles[chunks[w].tile];
    const bool light = pp.refine && pp.light_rows > 0 && static_cast<int64_t>(tl.n_pos) * pp.group <= pp.light_rows;
    int64_t l_kv = chunks[w].kv_len;
    if (pp.refine) l_kv = (l_kv + pp.kv_quantum - 1) / pp.kv_quantum * pp.kv_quantum;
    cost[w] = unit * pp.alpha * t_q + static_cast<int64_t>(pp.beta) * l_kv * (light ? pp.light_pct : unit);
  }
  std::vector<int64_t>& load = scratch.load;
  load.assign(static_cast<size_t>(C), 0);
  std::vector<int32_t>& cta_of = scratch.cta_of;  // the CTA of work item w; a queue keeps the order of assignment
  cta_of.resize(static_cast<size_t>(n_work));
  for (int32_t w : order) {
    Entry& e = heap[0];
    cta_of[w] = e.second;
    e.first += cost[w];
    load[e.second] = e.first;
    sift_down(heap);
  }

  // ---- refinement: while it lowers the maximum, move one item out of the most loaded CTA or swap it for a
  //      cheaper one (first best candidate in (cta, item, partner) order; a fixed number of rounds at most) ----
  // (with more than 8 items per CTA on average the greedy pass is fine-grained enough, and the search, which
  // is quadratic in the queue lengths, is skipped)
  const bool refined = pp.refine && n_work <= 8 * C;
  std::vector<std::vector<int32_t>>& queues = scratch.queues;
  if (refined) {
    if (queues.size() < static_cast<size_t>(C)) queues.resize(static_cast<size_t>(C));
    for (int32_t c = 0; c < C; ++c) queues[c].clear();
    for (int32_t w : order) queues[cta_of[w]].push_back(w);
    for (int32_t round = 0; round < 4 * C + 64; ++round) {
      int32_t hi = 0;
      for (int32_t c = 1; c < C; ++c)
        if (load[c] > load[hi]) hi = c;
      int64_t best_new = load[hi];
      int32_t best_lo = -1, best_a = -1, best_b = -1;  // positions in the queues
      for (int32_t lo = 0; lo < C; ++lo) {
        if (lo == hi) continue;
        for (size_t ia = 0; ia < queues[hi].size(); ++ia) {
          const int64_t ca = cost[queues[hi][ia]];
          const int64_t moved = std::max(load[hi] - ca, load[lo] + ca);
          if (moved < best_new) {
            best_new = moved;
            best_lo = lo;
            best_a = static_cast<int32_t>(ia);
            best_b = -1;
          }
          for (size_t ib = 0; ib < queues[lo].size(); ++ib) {
            const int64_t cb = cost[queues[lo][ib]];
            if (cb >= ca) continue;
            const int64_t swapped = std::max(load[hi] - ca + cb, load[lo] + ca - cb);
            if (swapped < best_new) {
              best_new = swapped;
              best_lo = lo;
              best_a = static_cast<int32_t>(ia);
              best_b = static_cast<int32_t>(ib);
            }
          }
        }
      }
      if (best_lo < 0) break;
      const int32_t wa = queues[hi][best_a];
      queues[hi].erase(queues[hi].begin() + best_a);
      load[hi] -= cost[wa];
      load[best_lo] += cost[wa];
      if (best_b >= 0) {
        const int32_t wb = queues[best_lo][best_b];
        queues[best_lo].erase(queues[best_lo].begin() + best_b);
        load[best_lo] -= cost[wb];
        load[hi] += cost[wb];
        queues[hi].push_back(wb);
      }
      queues[best_lo].push_back(wa);
    }
    for (int32_t c = 0; c < C; ++c)
      for (int32_t w : queues[c]) cta_of[w] = c;
  }
  // A queue runs its longest chunk first, the lower work index first among equals: the items of its CTA in the
  // sequence of `order` (which is also the order in which the greedy pass assigned them).

  // ---- emit the plan section ----
  std::fill(plan, plan + L.plan_ints, 0);
  int32_t* hdr = plan + L.off_header;
  hdr[H_N_WORK] = n_work;
  hdr[H_N_MERGE] = n_merge;
  hdr[H_N_SLOTS] = next_slot;
  hdr[H_L_KV] = static_cast<int32_t>(Lkv);
  hdr[H_T_POS] = pp.t_pos;
  hdr[H_CTAS] = static_cast<int32_t>(C);
  int32_t* cta_indptr = plan + L.off_cta_indptr;
  for (int32_t w = 0; w < n_work; ++w) ++cta_indptr[cta_of[w] + 1];
  for (int32_t c = 0; c < C; ++c) cta_indptr[c + 1] += cta_indptr[c];
  std::vector<int32_t>& fill = scratch.fill;  // next free position of each CTA's queue
  fill.assign(cta_indptr, cta_indptr + C);
  for (int32_t w : order) {
    const int32_t k = fill[cta_of[w]]++;
    const Chunk& ch = chunks[w];
    const Tile& tl = tiles[ch.tile];
    plan[L.off_work[W_REQUEST] + k] = tl.request;
    plan[L.off_work[W_Q_ROW0] + k] = tl.q_row0;
    plan[L.off_work[W_N_POS] + k] = tl.n_pos;
    plan[L.off_work[W_KV_PAGE0] + k] = tl.kv_page_base + ch.kv_start / ps;
    plan[L.off_work[W_KV_START] + k] = ch.kv_start;
    plan[L.off_work[W_KV_LEN] + k] = ch.kv_len;
    plan[L.off_work[W_DIAG0] + k] = tl.diag0;
    plan[L.off_work[W_OUT_SLOT] + k] = tl.slot_base < 0 ? -1 : tl.slot_base + ch.in_tile;
    plan[L.off_work[W_MERGE] + k] = tl.merge_index;
  }
  if (composed) {
    // ---- per query row: the partial states it folds; tiles are in (format, request, tile) order, which within a
    //      format is ascending query rows ----
    hdr[H_N_ROWS] = static_cast<int32_t>(n_rows);
    int32_t* row_indptr = plan + L.off_row_indptr;
    int32_t* row_entry = plan + L.off_row_entry;
    for (const Tile& tl : tiles)
      for (int32_t p = 0; p < tl.n_pos; ++p) row_indptr[tl.q_row0 + p + 1] += tl.n_chunks;
    for (int64_t r = 0; r < n_rows; ++r) row_indptr[r + 1] += row_indptr[r];
    if (static_cast<size_t>(row_indptr[n_rows]) > static_cast<size_t>(L.max_work) * pp.t_pos)
      return fail(FI_ERR_WORKSPACE_TOO_SMALL, "fi_plan_formats: row lists exceed the workspace section (internal bound)");
    std::vector<int32_t>& at = scratch.fill;  // next free entry of each row's list
    at.assign(row_indptr, row_indptr + n_rows);
    for (const Tile& tl : tiles)
      for (int32_t p = 0; p < tl.n_pos; ++p)
        for (int32_t c = 0; c < tl.n_chunks; ++c) row_entry[at[tl.q_row0 + p]++] = (tl.slot_base + c) * pp.t_pos + p;
    return FI_OK;
  }
  int32_t mi = 0;
  for (const Tile& tl : tiles) {
    if (tl.slot_base < 0) continue;
    plan[L.off_merge[M_Q_ROW0] + mi] = tl.q_row0;
    plan[L.off_merge[M_N_POS] + mi] = tl.n_pos;
    plan[L.off_merge[M_SLOT_BASE] + mi] = tl.slot_base;
    plan[L.off_merge[M_N_CHUNKS] + mi] = tl.n_chunks;
    hdr[H_MERGE_POS] = std::max(hdr[H_MERGE_POS], tl.n_pos);
    ++mi;
  }
  return FI_OK;
}

}  // namespace fi355
