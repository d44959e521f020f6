// Launch interface between the C-ABI layer and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace fi355 {

// Everything a persistent attention launch reads.  The plan arrays live in the
// fixed plan section of the device workspace (App. D.1).
struct RunParams {
  const int32_t* cta_indptr;
  const int32_t* w_q_row0;
  const int32_t* w_n_pos;
  const int32_t* w_kv_page0;
  const int32_t* w_kv_start;
  const int32_t* w_kv_len;
  const int32_t* w_diag0;
  const int32_t* w_out_slot;
  const int32_t* kv_indices;
  const void* q;
  const void* k_pool;
  const void* v_pool;
  int64_t stride_page, stride_head, stride_tok;  // elements
  float* o;
  float* lse;
  void* o_cast;     // may be null
  float* part_o;    // [max_slots * t_pos * H_qo, D]
  float* part_lse;  // [max_slots * t_pos * H_qo]
  float scale_log2; // sm_scale * log2(e) (times the K scale of an 8-bit KV cache)
  float out_scale;  // 8-bit KV cache: the V scale; 1 otherwise
  int32_t num_qo_heads, num_kv_heads, group, t_pos;
  int32_t ctas_per_head;
  int32_t page_log2;  // log2 of the page size (tokens per page)
  // contraction inside the decode launch (Sec. 3.3.1): w_merge != null switches it on
  const int32_t* w_merge;      // per work item: index of its split tile in the m_* arrays, -1 if not split
  const int32_t* m_slot_base;  // per split tile: first partial slot
  const int32_t* m_n_chunks;   //                 number of partial states
  int32_t* merge_counters;     // [split tile][kv head] partial states delivered so far; zero between launches
  // attention variants (Sec. 3.2.3), read by the variant kernels only
  const int32_t* w_request;      // request of each work item
  const int32_t* kv_indptr;      // DEVICE copies of the plan inputs: a request's total KV length gives the
  const int32_t* last_page_len;  //   absolute position of its query
  const float* alibi_slopes;     // [num_qo_heads] or null
  float soft_cap;                // > 0: logits <- cap * tanh(logits / cap)
  float cap_k1, cap_a;           // with a soft cap: 2 * scale_log2 / cap and cap * log2(e) (the append loop's constants)
  int32_t window_left;           // >= 0: tokens more than this far behind the query are hidden
};

// Rotary position embedding fused into the decode kernel (query / key transform, Sec. 3.2.3): the angle of
// component pair (d, d + 64) at position t is t * rev[d] revolutions.  A second table holds fract(256 * rev[d]),
// rounded from double precision, so that the kernel can reduce t = 256 t1 + t0 to a fraction of a revolution
// without losing the low bits of large positions: fract(t1 * rev256[d] + t0 * rev[d]).
struct RopeTable {
  float rev[64];
  float rev256[64];
};

struct MergeParams {
  const int32_t* header;  // plan header: [H_N_MERGE] read on the device
  const int32_t* m_q_row0;
  const int32_t* m_n_pos;
  const int32_t* m_slot_base;
  const int32_t* m_n_chunks;
  const float* part_o;
  const float* part_lse;
  float* o;
  float* lse;
  void* o_cast;
  int32_t num_qo_heads, t_pos, is_bf16;
  int32_t max_merge;  // entries the merge list arrays hold (readable past n_merge)
};

// Two passes over the same query rows: a.o / a.lse (b.o / b.lse) hold the states of the pass's unsplit tiles.
struct ComposeParams {
  MergeParams a, b;
  float* o;  // may be null when o_cast is not
  float* lse;
  void* o_cast;
  int64_t nnz_qo;
};

// decode.hip: query tile = 1 position x g fused heads, one wavefront per CTA.
// kv8: the pools hold OCP E4M3 codes (App. F) instead of the query type.  variant: the logits hooks of
// RunParams are applied (16-bit pools, page size 16 only).
// rope != null (variant launches only): queries and keys are rotated by their positions first.
hipError_t launch_decode(const RunParams& p, bool is_bf16, bool kv8, bool variant, const RopeTable* rope,
                         hipStream_t stream);
// tile.hip: query tiles of up to 16 fused rows = RunParams::t_pos positions x g heads, one wavefront per CTA,
// causal or not; 16-bit pools, page size 16, no variants; grid = ctas_per_head * num_kv_heads with the kv head as
// the fast index.
hipError_t launch_tiles(const RunParams& p, bool is_bf16, hipStream_t stream);
// tile64.hip: query tiles of up to 64 fused rows, CTAs of four wavefronts: tiles of more than 16 rows share every
// K/V row through LDS, tiles of at most 16 rows are walked by the four wavefronts side by side; same limits and grid.
hipError_t launch_tiles64(const RunParams& p, bool is_bf16, hipStream_t stream);
// append.hip: query tile = append_tile_rows()/g positions x g fused heads, 8 wavefronts per CTA.
// variant: the logits hooks of RunParams are applied (causal batches only; with ALiBi or a window every item takes
// the generic path, the soft cap alone has a variant of the scheduled loop).
// rope != null (variant launches only): queries and keys are rotated by their positions first (general path).
hipError_t launch_append(const RunParams& p, bool is_bf16, bool variant, const RopeTable* rope, hipStream_t stream);
int append_tile_rows();  // fused rows (positions x group) of one append query tile
// upload.hip: staging (device view of page-locked host memory) -> plan section
hipError_t launch_plan_upload(const int32_t* staging_dev_view, int32_t* plan_section, int32_t n_ints,
                              hipStream_t stream);
// merge.hip
hipError_t launch_merge_planned(const MergeParams& p, int32_t grid, hipStream_t stream);
hipError_t launch_compose(const ComposeParams& p, hipStream_t stream);
// Contraction of a plan over several formats: query row r folds the partial states listed in
// row_entry[row_indptr[r] .. row_indptr[r + 1]) (entry = partial row of the state before the head is added).
struct RowMergeParams {
  const int32_t* header;  // [H_N_ROWS] read on the device
  const int32_t* row_indptr;
  const int32_t* row_entry;
  const float* part_o;
  const float* part_lse;
  float* o;  // may be null when o_cast is not
  float* lse;
  void* o_cast;
  int32_t num_qo_heads, is_bf16;
};
hipError_t launch_merge_rows(const RowMergeParams& p, int32_t grid, hipStream_t stream);
hipError_t launch_merge_states(const float* o_parts, const float* lse_parts, int64_t n_rows, int32_t n_states,
                               float* o, float* lse, hipStream_t stream);
hipError_t launch_merge_pair(const float* o_a, const float* lse_a, const float* o_b, const float* lse_b,
                             int64_t n_rows, float* o, float* lse, hipStream_t stream);

constexpr int kNoDiagMarker = 0x3FFFFFFF;  // w_diag0 of a non-causal work item
constexpr int kHeadDim = 128;
constexpr int kPageSize = 16;  // the page size the fast paths are specialised for
constexpr int kMergeGrid = 1024;  // fixed grid of the planned merge launch

}  // namespace fi355
