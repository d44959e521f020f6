/*
 * fi355 -- batched attention over a paged (block-sparse-row) KV cache for AMD MI355X (gfx950).
 *
 * C ABI of the library: plain pointers and sizes only.  Every pointer is marked
 * HOST or DEVICE.  All functions return an int32 status (FI_OK = 0, negative = error,
 * message through fi_last_error()); no exception leaves the library (a host allocation that
 * fails inside it comes back as FI_ERR_HOST_MEMORY), nothing aborts.
 *
 * Method (FlashInfer, arXiv 2501.01005):
 *   - storage: ragged query/output + block-sparse-row KV cache, Sec. 3.1.1;
 *     several formats over one pool (shared prefix), Sec. 3.1.2;
 *   - attention state (O, LSE) and its merge operator, Sec. 2.2;
 *   - plan / run split, workspace with fixed sections, Sec. 3.3.1, Sec. 3.4, App. D;
 *   - load-balanced partition of KV ranges over a fixed number of CTAs, Algorithm 1;
 *   - head-group fusion for grouped-query attention, App. A.
 *
 * Ownership: the caller owns every device buffer and the pinned staging buffer.
 * The library allocates no device memory, frees nothing it was handed, and never
 * synchronises the device.  A handle owns only host-side plan arrays.
 *
 * Layouts (all row-major, innermost dimension contiguous):
 *   q        DEVICE  [nnz_qo, num_qo_heads, head_dim]   fp16 or bf16
 *   o        DEVICE  [nnz_qo, num_qo_heads, head_dim]   fp32   (attention output)
 *   lse      DEVICE  [nnz_qo, num_qo_heads]             fp32   (natural log-sum-exp of the
 *                                                               scaled logits; -inf for an
 *                                                               empty key set, then o = 0)
 *   k_pool, v_pool DEVICE, addressed as
 *            base + page*kv_strides[0] + kv_head*kv_strides[1] + slot*kv_strides[2] + d
 *            (strides in elements; head_dim contiguous).  The tuned layout is
 *            [num_pages, num_kv_heads, page_size, head_dim].
 *   qo_indptr, kv_indptr [batch+1], last_page_len [batch]  HOST int32 (plan input)
 *   kv_indices DEVICE int32 [kv_indptr[batch]] page ids (run input; not range checked
 *            on the device -- see fi_check_indices)
 */
#ifndef FI355_H_
#define FI355_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FI_OK 0
#define FI_ERR_INVALID_ARG (-1)          /* null pointer, malformed indptr, length out of range ... */
#define FI_ERR_UNSUPPORTED (-2)          /* head_dim / page_size / group size not instantiated      */
#define FI_ERR_WORKSPACE_TOO_SMALL (-3)
#define FI_ERR_NOT_PLANNED (-4)          /* fi_run before a successful fi_plan with a workspace     */
#define FI_ERR_HIP (-5)                  /* a HIP runtime call failed; message has its string       */
#define FI_ERR_HOST_MEMORY (-6)          /* a host-side allocation inside the library failed         */

#define FI_DTYPE_F16 0
#define FI_DTYPE_BF16 1

#define FI_MODE_DECODE 0 /* query tile = 1 position x g fused heads; one wavefront per CTA   */
#define FI_MODE_APPEND 1 /* query tile = 256/g positions x g fused heads; MFMA tile kernel     */
#define FI_MODE_TILE16 2 /* query tile = 16/g positions x g fused heads = the 16 columns of the decode kernel's
                            matrix tile, one wavefront per CTA (the small query tiles of Sec. 3.2.2): short
                            appends (causal or not), and several formats over the same query rows planned and
                            run as ONE work list and ONE attention launch (fi_plan_formats, Sec. 3.1.2).
                            16-bit pools, page_size 16, no variants                                  */
#define FI_MODE_TILE64 3 /* query tile = 64/g positions x g fused heads, CTAs of four wavefronts (Sec. 3.2.2: the
                            tile size follows the query lengths): a tile of more than 16 fused rows gives each
                            wavefront 16 of them and the four share every K/V row through LDS (a block of queries
                            over a shared prefix, Sec. 3.1.2, re-reads it 4x less often than in FI_MODE_TILE16);
                            a tile of at most 16 rows (a decode step) has its chunk walked by the four wavefronts
                            side by side and their states merged in the CTA.  The planner counts such a light
                            tile's tokens at 30 percent, in the work items' costs and in the sum that sets the
                            chunk length.  Same uses and limits as FI_MODE_TILE16, g in {1, 2, 4, 8, 16}          */

typedef struct fi_handle fi_handle;
typedef void* fi_stream; /* a hipStream_t (0 = the null stream) */

/* Fixed at creation; launch grids and workspace section offsets depend on this struct
 * only, never on sequence lengths (Sec. 3.3.1 last paragraph, App. D.1). */
typedef struct fi_config {
  int32_t dtype;        /* FI_DTYPE_*: storage type of q, k_pool, v_pool                       */
  int32_t num_qo_heads; /* H_qo                                                                */
  int32_t num_kv_heads; /* H_kv; g = H_qo / H_kv must be an integer                            */
  int32_t head_dim;     /* D (128)                                                             */
  int32_t page_size;    /* B_c of the BSR cache: a power of two in 1..64.  16 is the size the
                           kernels are tuned for; the others run general code paths (slower)   */
  int32_t mode;         /* FI_MODE_*                                                           */
  int32_t num_ctas;     /* total persistent CTAs over all kv heads; 0 = library default for
                           the current device (needs a GPU); CTAs per kv head = num_ctas/H_kv   */
  int32_t max_batch;    /* upper bound on `batch` of any later fi_plan (fi_plan_formats: on the sum
                           of the formats' batches)                                            */
  int32_t max_qo_tiles; /* upper bound on the number of query tiles of any later fi_plan
                           (decode: = max_batch; otherwise sum_i ceil(l_qo(i) / T_pos), over all
                           formats for fi_plan_formats)                                        */
  int32_t alpha;        /* cost(l_q, l_kv) = alpha*l_q + beta*l_kv of Algorithm 1; 0,0 = 1,1
                           (8,5 for the refined append assignment, see `balance`)              */
  int32_t beta;
  int32_t min_chunk;    /* smallest KV chunk the planner may create, tokens; 0 = default
                           (decode 32, append 256)                                              */
  int32_t literal_lkv;  /* 1: use l_kv(i) for every query tile in the chunk-size formula as
                           printed in Algorithm 1 even under causal masking; 0: use what the
                           tile can see                                                         */
  int32_t balance;      /* assignment of work items to CTAs.  1: Algorithm 1 as printed (greedy,
                           least-loaded CTA first).  2: the same, then items are moved or swapped
                           out of the most loaded CTA while that lowers the maximum; in append mode
                           a tile of at most half the fused rows counts 64 % of its per-token cost
                           (it leaves wavefronts idle).  0: default = 2 for append; for decode 1,
                           except that in a batch so small that Algorithm 1's chunk length is at
                           most 256 tokens a chunk length up to twice that is taken when it lowers
                           ceil(#chunks / #CTA) * (64 + chunk length): a work item has a fixed cost,
                           and a slightly longer chunk can save every CTA a second item            */
  int32_t merge;        /* where the partial states of split tiles are contracted (Sec. 3.3.1: the paper
                           fuses the contraction into the attention launch).  1: in a second launch.
                           2: in the attention launch: the CTA that delivers a tile's last partial
                           state folds them all (decode mode with g = 1, 2 or 4 only, FI_ERR_UNSUPPORTED
                           otherwise; on MI355X slower than 1, because partial states cross between the
                           XCDs' L2 caches through memory).
                           0: default = 1                                                       */
  int32_t plan_window;  /* sliding-window attention: 0 = every key a query may see is planned and read;
                           n > 0: a query at position pos sees keys pos - (n - 1) .. pos only, and fi_plan
                           leaves the keys before a tile's window (rounded down to a page) out of its
                           work items, so that the time follows the window, not the context length.
                           Such a plan must be run with fi_run_variant and 0 <= window_left <= n - 1
                           (the kernel masks token by token; FI_ERR_INVALID_ARG otherwise)        */
  int32_t max_formats;  /* how many formats a later fi_plan_formats may plan at once.  0: default = as many
                           as fit for the tile modes (FI_MODE_TILE16, FI_MODE_TILE64), 1 for the others.
                           1: one format at a time (fi_plan, or fi_plan_formats with one format): the
                           workspace then holds partial states for 2 * #CTA-bounded split tiles only
                           (App. D.3) instead of one per work item, which matters when max_qo_tiles is
                           large.  More than 1 on a decode or append handle: FI_ERR_UNSUPPORTED       */
} fi_config;

/* Borrowed HOST views of the last plan, for bit-exact checks against a replica of
 * Algorithm 1.  Work items are listed queue by queue: CTA c owns items
 * cta_indptr[c] .. cta_indptr[c+1]-1, in the order it executes them. */
typedef struct fi_plan_arrays {
  int32_t t_pos;          /* query positions per tile                                          */
  int32_t group;          /* g                                                                 */
  int32_t ctas_per_head;  /* #CTA of Algorithm 1                                               */
  int32_t l_kv_chunk;     /* L_kv: maximum chunk size, tokens                                  */
  int32_t n_work;         /* number of work items (chunks)                                     */
  int32_t n_merge;        /* number of query tiles that were split                             */
  int32_t n_slots;        /* partial-output slots in use (<= 2 * ctas_per_head, App. D.3)      */
  int32_t pad_;
  const int32_t* cta_indptr;  /* [ctas_per_head + 1]                                           */
  const int32_t* w_request;   /* [n_work] request index                                        */
  const int32_t* w_q_row0;    /* [n_work] first query row (index into q's leading dimension)   */
  const int32_t* w_n_pos;     /* [n_work] valid query positions in the tile                    */
  const int32_t* w_kv_page0;  /* [n_work] index into kv_indices of the chunk's first page      */
  const int32_t* w_kv_start;  /* [n_work] first token of the chunk within the request          */
  const int32_t* w_kv_len;    /* [n_work] tokens in the chunk (0 for an empty request)         */
  const int32_t* w_diag0;     /* [n_work] causal: tile row r sees request tokens <= diag0 + r;
                                 non-causal: 0x3FFFFFFF                                        */
  const int32_t* w_out_slot;  /* [n_work] -1 = write the final output directly (App. D.2),
                                 else partial-output slot                                      */
  const int32_t* w_merge;     /* [n_work] index of the item's tile in the m_* arrays, -1 if the
                                 tile was not split                                            */
  const int32_t* m_q_row0;    /* [n_merge] first query row of the split tile                   */
  const int32_t* m_n_pos;     /* [n_merge]                                                     */
  const int32_t* m_slot_base; /* [n_merge] first slot; chunk c of the tile is slot base + c    */
  const int32_t* m_n_chunks;  /* [n_merge]                                                     */
  /* plans over several formats (fi_plan_formats with n_formats > 1) have no merge list (n_merge = 0) and no
   * write-through (every w_out_slot >= 0); instead every query row lists the partial states it folds:         */
  int32_t n_rows;             /* query rows of such a plan, 0 otherwise                            */
  int32_t pad2_;
  const int32_t* row_indptr;  /* [n_rows + 1] row r folds row_entry[row_indptr[r] .. row_indptr[r + 1])   */
  const int32_t* row_entry;   /* partial state = slot * t_pos + position of the row in the slot's tile,
                                 formats in the order given, chunks of a tile in ascending KV order  */
} fi_plan_arrays;

/* Create / destroy a handle.  cfg HOST.  FI_ERR_UNSUPPORTED unless head_dim = 128,
 * page_size a power of two in 1..64 (16 in FI_MODE_TILE16 and FI_MODE_TILE64), g in {1,2,4,8,16}.  With num_ctas = 0 the
 * current HIP device is queried (FI_ERR_HIP without one). */
int32_t fi_create(const fi_config* cfg, fi_handle** out);
int32_t fi_destroy(fi_handle* h);

/* Bytes the caller must provide: device workspace (plan sections + partial outputs,
 * App. D.3 bound 2 * #CTA * T_q * (D + 1) floats per kv head) and pinned staging buffer. */
int32_t fi_workspace_bytes(const fi_handle* h, size_t* device_bytes, size_t* pinned_host_bytes);

/* The scheduler of Algorithm 1 (Sec. 3.3.1), run on the host once per generation step and
 * reused by every layer.  Reads the three HOST arrays, writes the plan into `pinned_host`
 * (HOST, page-locked, >= pinned_host_bytes; NULL = use pageable memory of the handle) and
 * enqueues ONE async transfer into the fixed plan sections of `workspace_dev` on `stream`
 * (a copy kernel reading the staging buffer when it is mapped into the device address
 * space, as hipHostMalloc memory is; hipMemcpyAsync otherwise).
 * The staging buffer must not be re-planned before that copy has executed.
 * workspace_dev = NULL plans on the host only (no HIP call; fi_run stays unavailable).
 * causal != 0: query j of a request sees tokens t <= l_kv - l_qo + j (the appended tokens
 * are already in the cache).  Errors: FI_ERR_INVALID_ARG for indptr[0] != 0, decreasing
 * indptr, last_page_len outside [1, page_size] on a non-empty request, batch > max_batch,
 * more tiles than max_qo_tiles; FI_ERR_WORKSPACE_TOO_SMALL. */
int32_t fi_plan(fi_handle* h, const int32_t* qo_indptr, const int32_t* kv_indptr,
                const int32_t* last_page_len, int32_t batch, int32_t causal,
                void* workspace_dev, size_t workspace_bytes,
                void* pinned_host, size_t pinned_bytes, fi_stream stream);

/* Composable formats (Sec. 3.1.2) as one plan: n_formats (1..8) block-sparse-row views of the KV pool over the
 * SAME nnz_qo query rows (say format 0 = one row block of all queries against the pages of a shared prefix,
 * format 1 = one row per request against its own pages), each given by its HOST arrays qo_indptr[f] [batch[f] + 1],
 * kv_indptr[f] [batch[f] + 1], last_page_len[f] [batch[f]], with kv_indptr[f] indexing the page-id array that fi_run
 * gets from element kv_indices_base[f] on (the caller keeps the formats' page ids one after the other in one
 * DEVICE array).  Every qo_indptr[f] must end at the same row count.  Algorithm 1 runs over the query tiles of all
 * formats at once: one chunk size, one set of queues, hence one persistent attention launch in fi_run, followed
 * by one contraction launch in which every query row folds its partial states (formats in the given order,
 * chunks in ascending KV order, Sec. 2.2).  Not causal.  Handle: FI_MODE_TILE16 or FI_MODE_TILE64 (FI_ERR_UNSUPPORTED otherwise).
 * With n_formats = 1 this is fi_plan with causal = 0.  Other arguments, staging and errors as fi_plan. */
int32_t fi_plan_formats(fi_handle* h, int32_t n_formats, const int32_t* const* qo_indptr,
                        const int32_t* const* kv_indptr, const int32_t* const* last_page_len,
                        const int32_t* batch, const int32_t* kv_indices_base, void* workspace_dev,
                        size_t workspace_bytes, void* pinned_host, size_t pinned_bytes, fi_stream stream);

/* Borrowed views of the handle's last plan; valid until the next fi_plan / fi_destroy. */
int32_t fi_plan_view(const fi_handle* h, fi_plan_arrays* out);

/* Attention over the planned batch (Sec. 2.2 states; Sec. 3.2 kernels): one persistent
 * launch of ctas_per_head x H_kv CTAs that walk their work queues, writing final rows
 * directly or partial states into the workspace, then one fixed-grid merge launch for the
 * split tiles.  All pointers DEVICE.  kv_strides HOST [3] = element strides of
 * (page, kv head, slot-in-page).  sm_scale (> 0) multiplies q.k before the softmax.
 * kv_indices = NULL: contiguous KV (the dense baseline of App. B): the page table is the identity, i.e. request i owns
 * pages kv_indptr[i] .. kv_indptr[i + 1] - 1 of the pool, rows are addressed affinely and no page id is loaded (with
 * page_size 1 and strides (H_kv * D, D, anything) the pool is the ragged tensor [tokens, H_kv, D]).  Decode and
 * append mode, fi_run only (FI_ERR_UNSUPPORTED elsewhere).
 * o_cast (may be NULL): the output also rounded to the input dtype (nearest even), [nnz_qo, H_qo, D].
 * o may be NULL when o_cast is not: the output is then written in the input dtype only, which
 * halves the output bytes of an append step (partial states stay fp32 in the workspace; lse is
 * always written).
 * Range of V in append mode with bf16 pools: the tile kernel multiplies P by V on the matrix cores in
 * fp16 (P needs fp16's 11 significant bits to meet the output tolerance) and converts every bf16 V
 * element to fp16 on its way from the pool: exact for 2^-14 <= |v| <= 65504; a larger magnitude enters
 * the product as +-65504 (no infinity is produced); a smaller one is rounded toward zero to a multiple
 * of 2^-24 (absolute error below 2^-24).  No error is reported for such values.  Decode mode and fp16
 * pools use V as stored.  (tests/test_gpu_append.py feeds such values and asserts exactly this.)
 * Asynchronous on `stream`; uses the workspace given to the last fi_plan. */
int32_t fi_run(fi_handle* h, const void* q, const void* k_pool, const void* v_pool,
               const int64_t* kv_strides, const int32_t* kv_indices, float sm_scale,
               float* o, float* lse, void* o_cast, fi_stream stream);

/* fi_run over an 8-bit KV cache (App. F: fp8 K/V with 16-bit queries and wider arithmetic):
 * k_pool and v_pool DEVICE hold one OCP E4M3 code per element (1 sign, 4 exponent bits with
 * bias 7, 3 mantissa bits; 0x7f / 0xff are NaN, no infinities); an element's value is its
 * decoded code times k_scale (v_scale), both > 0.  kv_strides are in elements, i.e. bytes, and
 * multiples of 8.  The codes are widened to the query type on the fly (exact), all arithmetic
 * is that of fi_run.  Decode mode only (FI_ERR_UNSUPPORTED for an append handle); otherwise
 * arguments, ownership and errors as for fi_run. */
int32_t fi_run_kv8(fi_handle* h, const void* q, const void* k_pool, const void* v_pool,
                   const int64_t* kv_strides, const int32_t* kv_indices, float sm_scale,
                   float k_scale, float v_scale, float* o, float* lse, void* o_cast,
                   fi_stream stream);

/* Attention variants (Sec. 3.2.3: logits transform and logits mask), applied to the scaled logits
 * s = sm_scale * q.k of query position pos and key position t in this order:
 *   logits_soft_cap c > 0:  s <- c * tanh(s / c)                       (0 = off)
 *   alibi_slopes != NULL:   s <- s + alibi_slopes[query head] * (t - pos)   DEVICE float [num_qo_heads]
 *   window_left W >= 0:     keys with t < pos - W are hidden            (-1 = off)
 * pos = l_kv - l_qo + j for query j of a request (the appended tokens are in the cache). */
typedef struct fi_variant {
  float logits_soft_cap;
  int32_t window_left;
  const float* alibi_slopes;
  float rope_theta; /* > 0: rotary position embedding fused into the kernel (query / key transform, Sec. 3.2.3;
                       Sec. 4.3): before the logits, key t is rotated by its position t and the query by pos;
                       component pair (d, d + D/2) turns by (position / rope_scale) * rope_theta^(-2d/D) radians.
                       The cache holds the keys unrotated.  0 = off */
  float rope_scale; /* position divisor of the rotary embedding; 0 = 1 */
} fi_variant;

/* fi_run with a variant.  (A window alone only masks: to skip the hidden keys, create the handle with
 * fi_config.plan_window.)  kv_indptr [batch+1] and last_page_len [batch] are DEVICE copies of the arrays
 * the batch was planned with (the decode kernel derives pos from them).  Built for 16-bit pools;
 * decode mode: every field of fi_variant (the rotary embedding at page_size 16 only); append mode: every field
 * too, for batches planned with causal = 1 (at page_size 16 the soft cap alone, and ALiBi and / or a window
 * without the soft cap, run variants of the scheduled tile loop, 1.2-1.3x the time of fi_run; the soft cap together
 * with one of the others, the rotary embedding, and every variant at other page sizes run every work item on the
 * kernel's general path, several times slower).  FI_ERR_UNSUPPORTED otherwise.  Every key of the request is still read, a window only
 * masks.  variant HOST, read during the call.  Otherwise as fi_run. */
int32_t fi_run_variant(fi_handle* h, const void* q, const void* k_pool, const void* v_pool,
                       const int64_t* kv_strides, const int32_t* kv_indices,
                       const int32_t* kv_indptr, const int32_t* last_page_len, float sm_scale,
                       const fi_variant* variant, float* o, float* lse, void* o_cast,
                       fi_stream stream);

/* Measurement hook: with two hipEvent_t handles set, every later fi_run records `before`
 * right before and `after` right after the launch of its attention kernel (the merge launch
 * comes after `after`) on the run's stream, so a caller can time that kernel alone.
 * NULL, NULL switches the hook off.  The events stay owned by the caller. */
int32_t fi_set_timing_events(fi_handle* h, void* before, void* after);

/* Merge operator of Sec. 2.2 over n_states states per row, folded in index order:
 * o_parts DEVICE [n_rows, n_states, D], lse_parts DEVICE [n_rows, n_states] ->
 * o DEVICE [n_rows, D], lse DEVICE [n_rows].  A state with lse = -inf is the identity. */
int32_t fi_merge_states(const float* o_parts, const float* lse_parts, int64_t n_rows,
                        int32_t n_states, int32_t head_dim, float* o, float* lse,
                        fi_stream stream);

/* Two-state merge used to compose a shared-prefix pass with a per-request pass
 * (Sec. 3.1.2, Sec. 4.4).  o may alias o_a and lse may alias lse_a (in place). */
int32_t fi_merge_state_pair(const float* o_a, const float* lse_a, const float* o_b,
                            const float* lse_b, int64_t n_rows, int32_t head_dim,
                            float* o, float* lse, fi_stream stream);

/* Composable formats (Sec. 3.1.2) in three launches instead of five: the attention kernels of two
 * planned handles over the SAME nnz_qo query rows (say a shared-prefix format in append mode and a
 * per-request format in decode mode, each with its own handle, plan, workspace and page ids over the
 * same pools), then ONE contraction launch that, per output row, folds each pass's partial states
 * where its tile was split and merges the two states (Sec. 2.2).  The result equals, bit for bit,
 * fi_run on each handle followed by fi_merge_state_pair.
 * o_a, lse_a, o_b, lse_b DEVICE fp32 [nnz_qo, H_qo, D] / [nnz_qo, H_qo]: state rows of each pass that
 * the caller owns (the attention kernels write the states of unsplit tiles there; contents after the
 * call are unspecified).  o / lse / o_cast as in fi_run (o may be NULL when o_cast is not); they may
 * alias neither pass's rows.  Both handles: same dtype and head counts, merge != 2, no plan_window;
 * 16-bit pools.  Errors as fi_run, plus FI_ERR_INVALID_ARG when the plans' query rows differ from
 * nnz_qo.  Asynchronous on `stream`.  Allocates nothing; the launch geometry depends on the two
 * configurations and on nnz_qo only, so a captured call serves later plans over as many query rows. */
int32_t fi_run_composed(fi_handle* h_a, fi_handle* h_b, const void* q, const void* k_pool,
                        const void* v_pool, const int64_t* kv_strides, const int32_t* kv_indices_a,
                        const int32_t* kv_indices_b, float sm_scale, float* o_a, float* lse_a,
                        float* o_b, float* lse_b, int64_t nnz_qo, float* o, float* lse, void* o_cast,
                        fi_stream stream);

/* fi_run_composed for callers that cannot allocate device memory (code under HIP graph capture, serving loops
 * that must not call hipMalloc, harnesses that forbid it): the state rows of the two passes (o_a, lse_a, o_b,
 * lse_b of fi_run_composed) live in a static device array of the library instead of caller buffers.  Limit:
 * nnz_qo * num_qo_heads <= 4096 state rows (the array holds 2 * 4096 * (128 + 1) floats = 4 227 072 bytes on
 * every GPU the library is used on, from the library's load until the process ends);
 * FI_ERR_WORKSPACE_TOO_SMALL beyond that.  The call allocates and frees nothing; the address of the array is
 * looked up once per GPU, on the first call with that GPU current (the GPU of `stream` must be the current one).
 * All calls on one GPU share the array: calls whose work overlaps in time on one GPU (two streams) race; calls
 * ordered on one stream do not.  The array keeps the previous call's contents; nothing in it has to be cleared.
 * Everything else (arguments, result bits, errors) as fi_run_composed. */
int32_t fi_run_composed_static(fi_handle* h_a, fi_handle* h_b, const void* q, const void* k_pool,
                               const void* v_pool, const int64_t* kv_strides, const int32_t* kv_indices_a,
                               const int32_t* kv_indices_b, float sm_scale, int64_t nnz_qo, float* o,
                               float* lse, void* o_cast, fi_stream stream);

/* HOST helper: which handle mode to create for a batch whose requests bring `mean_qo_len` query positions each on
 * average (Sec. 3.2.2 picks the query tile size from the average query length; here the tile size is the handle's
 * mode).  With g = num_qo_heads / num_kv_heads fused rows per position: one position -> FI_MODE_DECODE; at most 16
 * fused rows per request -> FI_MODE_TILE64 (its four wavefronts walk a chunk side by side); more -> FI_MODE_APPEND
 * (the 256-row matrix kernel wins from there on although most of its rows are empty).  Measured on this part at
 * g = 4, page size 16; a rule of thumb, not a guarantee.  Returns the mode, or FI_ERR_INVALID_ARG (< 0). */
int32_t fi_suggest_mode(int32_t num_qo_heads, int32_t num_kv_heads, double mean_qo_len);

/* HOST helper for tests: FI_OK iff every indices[i] is in [0, num_pages). */
int32_t fi_check_indices(const int32_t* indices_host, int64_t n, int32_t num_pages);

/* Message for the last non-zero status returned on this thread (never NULL). */
const char* fi_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FI355_H_ */
