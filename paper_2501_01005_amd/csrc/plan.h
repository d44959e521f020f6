// Host-side scheduler (Algorithm 1, Sec. 3.3.1) and workspace layout (App. D).
// Integer-only C++; no HIP types here.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

namespace fi355 {

constexpr int32_t kNoDiag = 0x3FFFFFFF;
constexpr int kHeaderInts = 16;
constexpr int kWorkArrays = 9;   // request, q_row0, n_pos, kv_page0, kv_start, kv_len, diag0, out_slot, merge
constexpr int kMergeArrays = 4;  // q_row0, n_pos, slot_base, n_chunks

// Indices of the per-work-item arrays inside the plan section.
enum WorkField { W_REQUEST = 0, W_Q_ROW0, W_N_POS, W_KV_PAGE0, W_KV_START, W_KV_LEN, W_DIAG0, W_OUT_SLOT, W_MERGE };
enum MergeField { M_Q_ROW0 = 0, M_N_POS, M_SLOT_BASE, M_N_CHUNKS };
// (H_MERGE_POS: the largest number of positions of a split tile, which bounds the rows the contraction launch walks)
enum HeaderField { H_N_WORK = 0, H_N_MERGE, H_N_SLOTS, H_L_KV, H_T_POS, H_CTAS, H_N_ROWS, H_MERGE_POS };

// Section offsets depend only on the creation-time configuration, so the pointers a
// captured launch holds stay valid across plans (App. D.1).
struct WorkspaceLayout {
  int32_t ctas_per_head = 0;  // #CTA of Algorithm 1
  int32_t max_work = 0;       // max_qo_tiles + ctas_per_head
  int32_t max_merge = 0;      // ctas_per_head
  int32_t max_slots = 0;      // 2 * ctas_per_head (App. D.3)
  size_t off_header = 0;      // int32 offsets (in ints) inside the plan section
  size_t off_cta_indptr = 0;
  size_t off_work[kWorkArrays] = {};
  size_t off_merge[kMergeArrays] = {};
  size_t off_counters = 0;    // max_merge * num_kv_heads arrival counters of the split tiles, zero in every plan
  // Handles that can plan several formats over the same query rows (Sec. 3.1.2) also hold, per query row, the list
  // of partial states to fold: row r owns row_entry[row_indptr[r] .. row_indptr[r + 1]), each entry the partial row
  // slot * t_pos + position-in-tile of one state, in fold order.  max_rows = 0 without them.
  int32_t max_rows = 0;       // max_qo_tiles * t_pos
  size_t off_row_indptr = 0;  // [max_rows + 1]
  size_t off_row_entry = 0;   // [max_work * t_pos]
  size_t plan_ints = 0;       // ints in the plan section
  size_t plan_bytes = 0;      // rounded up to 256
  size_t off_part_lse = 0;    // byte offsets in the device workspace
  size_t off_part_o = 0;
  size_t total_bytes = 0;

  // formats: the handle may plan several formats at once: every work item then owns a partial slot
  void init(int32_t ctas, int32_t max_qo_tiles, int32_t t_pos, int32_t num_qo_heads, int32_t num_kv_heads,
            int32_t head_dim, bool formats = false, int32_t chunk_factor = 1);
};

struct PlanParams {
  int32_t page_size = 16;
  int32_t t_pos = 1;
  int32_t group = 1;
  int32_t ctas_per_head = 1;
  int32_t alpha = 1, beta = 1;
  int32_t min_chunk = 16;
  bool causal = false;
  bool literal_lkv = false;
  // Load balance beyond the greedy assignment of Algorithm 1 (off = the algorithm as printed):
  // a work item whose fused rows (n_pos * group) fit in `light_rows` costs `light_pct` percent of
  // the per-token term (such a tile leaves wavefronts of the append kernel idle), and after the
  // greedy pass items are moved or swapped out of the most loaded CTA while that lowers the maximum.
  // With the refinement the chunk length is also rounded up to whole tiles of kv_quantum tokens.
  bool refine = false;
  int32_t light_rows = 0;
  int32_t light_pct = 100;
  int32_t kv_quantum = 1;
  int32_t max_batch = 0;
  int32_t max_qo_tiles = 0;
  // Sliding window: > 0 = W + 1, a query at position pos sees keys pos - W .. pos only, and the keys that no row
  // of a tile sees (before its first row's window, rounded down to a page) are left out of the tile's KV range.
  int32_t plan_window = 0;
  // Fixed cost of a work item in tokens (0 = off, the chunk length as printed).  When the chunk length of
  // Algorithm 1 is at most 4 * item_cost (a batch so small that a CTA gets about one short chunk), chunk lengths
  // L up to twice that, in whole pages, are tried and the one with the smallest ceil(#chunks / #CTA) * (item_cost + L)
  // is taken (ties: the shorter): a slightly longer chunk can save every CTA a second work item.
  int32_t item_cost = 0;
  // With the refinement: a light tile's KV range also counts light_pct percent (rounded up, tile by tile) in the
  // sum S that sets the chunk length L_kv = S / #CTA, so that the CTAs' loads in cost units, not in tokens, come out
  // equal when light and full tiles are planned together (the 64-row tile kernel walks a light tile's chunk with
  // four wavefronts side by side).
  bool weighted_lkv = false;
};

// One format (Sec. 3.1.1, Sec. 3.1.2): a block-sparse-row view of the KV pool over the query rows, given by its
// row partition (qo_indptr), its page lists (kv_indptr into the page-id array, starting at element kv_base of
// the array the kernels get) and the fill of every request's last page.
struct FormatView {
  const int32_t* qo_indptr = nullptr;
  const int32_t* kv_indptr = nullptr;
  const int32_t* last_page_len = nullptr;
  int32_t batch = 0;
  int32_t kv_base = 0;
};

// Runs the partition and writes the plan section (header, queues, work items, merge list)
// into `plan` (layout.plan_ints ints).  Returns 0 or a negative FI_ERR_* with `err` set.
int32_t make_plan(const PlanParams& pp, const WorkspaceLayout& layout, const int32_t* qo_indptr,
                  const int32_t* kv_indptr, const int32_t* last_page_len, int32_t batch,
                  int32_t* plan, std::string* err);

// The same over n_formats >= 1 formats that cover the same query rows (every qo_indptr ends at the same row count):
// the work items of all formats share the chunk size, the queues and the launch.  With more than one format every
// work item writes a partial state (no write-through: a row's final state is the merge of one state per format at
// least), the merge list is empty and the row lists say which partial states each query row folds, formats in the
// given order, chunks of a tile in ascending KV order.  Work indices run over (format, request, tile, chunk);
// w_request counts requests through all formats.  Needs a layout made with formats = true.
int32_t make_plan_formats(const PlanParams& pp, const WorkspaceLayout& layout, const FormatView* formats,
                          int32_t n_formats, int32_t* plan, std::string* err);

}  // namespace fi355
