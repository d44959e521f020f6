// C ABI of the library (declared in include/fi355.h): argument checks, the plan/run
// split of Sec. 3.4, workspace sections at fixed offsets (App. D.1), kernel launches.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/fi355.h"
#include "kernels.h"
#include "plan.h"

using namespace fi355;

namespace {
thread_local std::string g_last_error;
thread_local const char* g_fixed_error = nullptr;  // a message that needed no allocation (set when one failed)

int32_t set_error(int32_t code, const std::string& msg) {
  g_fixed_error = nullptr;
  g_last_error = msg;
  return code;
}

// Every entry point runs inside this: the planner's vectors and the error strings allocate host memory, and
// no C++ exception may cross the C boundary.
template <class Body>
int32_t guarded(Body&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    g_fixed_error = "out of host memory inside the library";
    return FI_ERR_HOST_MEMORY;
  } catch (...) {
    g_fixed_error = "unexpected C++ exception inside the library";
    return FI_ERR_HOST_MEMORY;
  }
}
int32_t hip_error(const char* what, hipError_t e) {
  return set_error(FI_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
}  // namespace

// ---- scratch memory of fi_run_composed_static: the state rows of the two passes, for callers that cannot
//      allocate.  One copy per GPU, held until the process ends; every call on a GPU uses that GPU's copy. ----
constexpr int64_t kStaticRowsMax = 4096;  // (query row, query head) pairs per call
constexpr size_t kStaticOBytes = static_cast<size_t>(kStaticRowsMax) * kHeadDim * sizeof(float);
constexpr size_t kStaticLseBytes = static_cast<size_t>(kStaticRowsMax) * sizeof(float);
constexpr size_t kStaticScratchBytes = 2 * (kStaticOBytes + kStaticLseBytes);  // 4 227 072 bytes
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU (null: not asked yet)

// The address of this GPU's copy of `scratch`.  In host code the array's name is only a handle for the runtime:
// the address comes from hipGetSymbolAddress, asked once per device with that device current.
int32_t static_scratch(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_error("fi_run_composed_static: hipGetDevice", e);
  if (dev < 0 || dev >= kMaxDevices)
    return set_error(FI_ERR_UNSUPPORTED, "fi_run_composed_static: device ordinal " + std::to_string(dev) + " outside [0, 64)");
  unsigned char* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !sym) return hip_error("fi_run_composed_static: hipGetSymbolAddress", e);
    ptr = static_cast<unsigned char*>(sym);
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // (a concurrent first call stores the same address)
  }
  *out = ptr;
  return FI_OK;
}
}  // namespace

constexpr int32_t kMaxFormats = 8;  // formats one fi_plan_formats call composes

struct fi_handle {
  fi_config cfg;
  PlanParams pp;
  WorkspaceLayout layout;
  std::vector<int32_t> host_plan;  // last plan section (also the pageable staging buffer)
  bool planned_host = false;
  bool planned_dev = false;
  bool pp_causal_last = false;  // `causal` of the last successful fi_plan
  int32_t n_formats_last = 1;   // formats of the last successful plan (> 1: every state is partial, rows fold by list)
  int64_t nnz_qo_last = 0;      // query rows of the last successful fi_plan
  void* workspace_dev = nullptr;
  size_t workspace_bytes = 0;
  hipEvent_t ev_before = nullptr;
  hipEvent_t ev_after = nullptr;
};

namespace impl {


int32_t fi_create(const fi_config* cfg, fi_handle** out) {
  if (!cfg || !out) return set_error(FI_ERR_INVALID_ARG, "fi_create: null argument");
  *out = nullptr;
  if (cfg->dtype != FI_DTYPE_F16 && cfg->dtype != FI_DTYPE_BF16)
    return set_error(FI_ERR_INVALID_ARG, "fi_create: dtype must be FI_DTYPE_F16 or FI_DTYPE_BF16");
  if (cfg->mode != FI_MODE_DECODE && cfg->mode != FI_MODE_APPEND && cfg->mode != FI_MODE_TILE16 &&
      cfg->mode != FI_MODE_TILE64)
    return set_error(FI_ERR_INVALID_ARG, "fi_create: unknown mode");
  if (cfg->num_qo_heads <= 0 || cfg->num_kv_heads <= 0 || cfg->num_qo_heads % cfg->num_kv_heads != 0)
    return set_error(FI_ERR_INVALID_ARG, "fi_create: num_qo_heads must be a positive multiple of num_kv_heads");
  if (cfg->max_batch <= 0 || cfg->max_qo_tiles <= 0 || cfg->num_ctas < 0 || cfg->alpha < 0 || cfg->beta < 0 ||
      cfg->min_chunk < 0)
    return set_error(FI_ERR_INVALID_ARG, "fi_create: max_batch/max_qo_tiles must be > 0, the rest >= 0");
  if (cfg->balance < 0 || cfg->balance > 2)
    return set_error(FI_ERR_INVALID_ARG, "fi_create: balance must be 0 (default), 1 (as printed) or 2 (refined)");
  if (cfg->merge < 0 || cfg->merge > 2)
    return set_error(FI_ERR_INVALID_ARG, "fi_create: merge must be 0 (default), 1 (second launch) or 2 (in the attention launch)");
  if (cfg->merge == 2 && cfg->mode != FI_MODE_DECODE)
    return set_error(FI_ERR_UNSUPPORTED, "fi_create: the contraction inside the attention launch is built for decode mode");
  if (cfg->plan_window < 0) return set_error(FI_ERR_INVALID_ARG, "fi_create: plan_window must be >= 0");
  if (cfg->head_dim != kHeadDim) return set_error(FI_ERR_UNSUPPORTED, "fi_create: only head_dim = 128 is built");
  if (cfg->page_size < 1 || cfg->page_size > 64 || (cfg->page_size & (cfg->page_size - 1)) != 0)
    return set_error(FI_ERR_UNSUPPORTED, "fi_create: page_size must be a power of two between 1 and 64");
  const int g = cfg->num_qo_heads / cfg->num_kv_heads;
  if (cfg->mode == FI_MODE_DECODE && !(g == 1 || g == 2 || g == 4 || g == 8 || g == 16))
    return set_error(FI_ERR_UNSUPPORTED, "fi_create: decode mode is built for group size 1, 2, 4, 8, 16");
  if (cfg->mode == FI_MODE_DECODE && cfg->merge == 2 && g > 4)
    return set_error(FI_ERR_UNSUPPORTED, "fi_create: the contraction inside the attention launch is built for group size 1, 2, 4");
  if (cfg->mode == FI_MODE_APPEND && !(g == 1 || g == 2 || g == 4 || g == 8 || g == 16))
    return set_error(FI_ERR_UNSUPPORTED, "fi_create: append mode is built for group size 1, 2, 4, 8, 16");
  const bool small_tiles = cfg->mode == FI_MODE_TILE16 || cfg->mode == FI_MODE_TILE64;
  if (cfg->max_formats < 0) return set_error(FI_ERR_INVALID_ARG, "fi_create: max_formats must be >= 0");
  if (cfg->max_formats > 1 && !small_tiles)
    return set_error(FI_ERR_UNSUPPORTED, "fi_create: several formats in one plan are built for the 16-row and 64-row tile modes");
  if (small_tiles && (!(g == 1 || g == 2 || g == 4 || g == 8 || g == 16) || cfg->page_size != kPageSize || cfg->plan_window > 0))
    return set_error(FI_ERR_UNSUPPORTED, "fi_create: the 16-row and 64-row tile modes are built for group size 1, 2, 4, 8, 16, page_size 16, "
                                         "no planned window");

  int num_ctas = cfg->num_ctas;
  if (num_ctas == 0) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_error("fi_create: hipGetDevice (num_ctas = 0 needs a GPU)", e);
    int cus = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return hip_error("fi_create: hipDeviceGetAttribute", e);
    // decode: one wavefront per CTA, 8 resident per CU; append: one 8-wavefront CTA per CU
    // (64-row tiles: two CTAs of four wavefronts per CU)
    num_ctas = cfg->mode == FI_MODE_APPEND ? cus : cfg->mode == FI_MODE_TILE64 ? 2 * cus : 8 * cus;
  }
  fi_handle* h = new (std::nothrow) fi_handle();
  if (!h) return set_error(FI_ERR_HOST_MEMORY, "fi_create: out of host memory");
  h->cfg = *cfg;
  h->cfg.num_ctas = num_ctas;
  PlanParams& pp = h->pp;
  pp.page_size = cfg->page_size;
  pp.group = g;
  pp.t_pos = cfg->mode == FI_MODE_DECODE   ? 1
              : cfg->mode == FI_MODE_TILE16 ? 16 / g
              : cfg->mode == FI_MODE_TILE64 ? 64 / g
                                            : append_tile_rows() / g;
  pp.ctas_per_head = num_ctas / cfg->num_kv_heads > 0 ? num_ctas / cfg->num_kv_heads : 1;
  // Decode items are short and many: the greedy pass of Algorithm 1 balances them to about 1 %.  Append
  // items are few and long (C3: 4.8 per CTA): there the refined assignment is the default, with the cost
  // measured on this kernel: 19 800 cycles per item + 48 per token, 64 % of that per token for a tile of at most
  // 128 fused rows (at most one live wavefront per SIMD), i.e. alpha : beta = 8 : 5 with T_q = 256.
  pp.plan_window = cfg->plan_window;
  const bool tile64 = cfg->mode == FI_MODE_TILE64;
  pp.refine = cfg->balance == 2 || (cfg->balance == 0 && (cfg->mode == FI_MODE_APPEND || tile64));
  // decode: a work item costs a wavefront about as much as 64 more tokens before its first tile arrives
  pp.item_cost = (cfg->balance == 0 && cfg->mode != FI_MODE_APPEND && !tile64) ? 64 : 0;
  const bool default_cost = cfg->alpha == 0 && cfg->beta == 0;
  pp.alpha = default_cost ? (pp.refine && cfg->mode == FI_MODE_APPEND ? 8 : 1) : cfg->alpha;
  pp.beta = default_cost ? (pp.refine && cfg->mode == FI_MODE_APPEND ? 5 : 1) : cfg->beta;
  pp.light_rows = (pp.refine && cfg->mode == FI_MODE_APPEND) ? append_tile_rows() / 2 : 0;
  pp.light_pct = 64;
  pp.kv_quantum = (pp.refine && cfg->mode == FI_MODE_APPEND) ? 64 : 1;  // the append kernel's KV tile
  // 64-row tiles: a tile of at most 16 fused rows has its chunk walked by the CTA's four wavefronts side by side
  // (30 percent of a full tile's time per token, measured); its tokens count that much in the chunk length too
  if (pp.refine && tile64) {
    pp.light_rows = 16;
    pp.light_pct = 30;
    pp.kv_quantum = 32;  // the kernel's step
    pp.weighted_lkv = true;
  }
  // default smallest chunk: append 256 tokens; decode one 32-token step of the kernel: with fewer tokens than that per CTA the chip is not filled, and a
  // wavefront that walks 128 tokens alone takes longer than four that walk 32 each plus their merge
  pp.min_chunk = cfg->min_chunk > 0 ? cfg->min_chunk : (cfg->mode == FI_MODE_APPEND ? 256 : tile64 ? 128 : 32);
  pp.literal_lkv = cfg->literal_lkv != 0;
  pp.max_batch = cfg->max_batch;
  pp.max_qo_tiles = cfg->max_qo_tiles;
  h->layout.init(pp.ctas_per_head, cfg->max_qo_tiles, pp.t_pos, cfg->num_qo_heads, cfg->num_kv_heads, cfg->head_dim,
                 small_tiles && cfg->max_formats != 1, pp.weighted_lkv ? (100 + pp.light_pct - 1) / pp.light_pct : 1);
  h->host_plan.assign(h->layout.plan_ints, 0);
  *out = h;
  return FI_OK;
}

int32_t fi_destroy(fi_handle* h) {
  delete h;
  return FI_OK;
}

int32_t fi_workspace_bytes(const fi_handle* h, size_t* device_bytes, size_t* pinned_host_bytes) {
  if (!h) return set_error(FI_ERR_INVALID_ARG, "fi_workspace_bytes: null handle");
  if (device_bytes) *device_bytes = h->layout.total_bytes;
  if (pinned_host_bytes) *pinned_host_bytes = h->layout.plan_bytes;
  return FI_OK;
}

// fi_plan and fi_plan_formats: plan on the host, then one transfer into the plan section of the workspace
int32_t plan_and_upload(fi_handle* h, const FormatView* formats, int32_t n_formats, int32_t causal, void* workspace_dev,
                        size_t workspace_bytes, void* pinned_host, size_t pinned_bytes, fi_stream stream) {
  if (workspace_dev && workspace_bytes < h->layout.total_bytes)
    return set_error(FI_ERR_WORKSPACE_TOO_SMALL, "fi_plan: device workspace has " + std::to_string(workspace_bytes) +
                                                     " bytes, needs " + std::to_string(h->layout.total_bytes));
  if (pinned_host && pinned_bytes < h->layout.plan_bytes)
    return set_error(FI_ERR_WORKSPACE_TOO_SMALL, "fi_plan: pinned staging buffer has " + std::to_string(pinned_bytes) +
                                                     " bytes, needs " + std::to_string(h->layout.plan_bytes));
  h->planned_host = false;
  h->planned_dev = false;
  PlanParams pp = h->pp;
  pp.causal = causal != 0;
  std::string err;
  const int32_t rc = make_plan_formats(pp, h->layout, formats, n_formats, h->host_plan.data(), &err);
  if (rc != FI_OK) return set_error(rc, err);
  h->planned_host = true;
  h->pp_causal_last = causal != 0;
  h->n_formats_last = n_formats;
  h->nnz_qo_last = formats[0].batch > 0 ? formats[0].qo_indptr[formats[0].batch] : 0;
  if (!workspace_dev) return FI_OK;
  const size_t bytes = h->layout.plan_ints * sizeof(int32_t);
  hipStream_t s = static_cast<hipStream_t>(stream);
  bool uploaded = false;
  if (pinned_host) {
    std::memcpy(pinned_host, h->host_plan.data(), bytes);
    // page-locked memory that is mapped into the device address space is pulled by a copy kernel
    void* dev_view = nullptr;
    if (hipHostGetDevicePointer(&dev_view, pinned_host, 0) == hipSuccess && dev_view) {
      const hipError_t e = launch_plan_upload(static_cast<const int32_t*>(dev_view), static_cast<int32_t*>(workspace_dev),
                                              static_cast<int32_t>(h->layout.plan_ints), s);
      if (e != hipSuccess) return hip_error("fi_plan: plan upload launch", e);
      uploaded = true;
    } else {
      (void)hipGetLastError();  // not device-mapped: fall back to a copy-engine transfer
    }
  }
  if (!uploaded) {
    const void* src = pinned_host ? pinned_host : static_cast<const void*>(h->host_plan.data());
    const hipError_t e = hipMemcpyAsync(workspace_dev, src, bytes, hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return hip_error("fi_plan: hipMemcpyAsync", e);
  }
  h->workspace_dev = workspace_dev;
  h->workspace_bytes = workspace_bytes;
  h->planned_dev = true;
  return FI_OK;
}

int32_t fi_plan(fi_handle* h, const int32_t* qo_indptr, const int32_t* kv_indptr, const int32_t* last_page_len,
                int32_t batch, int32_t causal, void* workspace_dev, size_t workspace_bytes, void* pinned_host,
                size_t pinned_bytes, fi_stream stream) {
  if (!h) return set_error(FI_ERR_INVALID_ARG, "fi_plan: null handle");
  FormatView f;
  f.qo_indptr = qo_indptr;
  f.kv_indptr = kv_indptr;
  f.last_page_len = last_page_len;
  f.batch = batch;
  if (!qo_indptr || !kv_indptr) return set_error(FI_ERR_INVALID_ARG, "fi_plan: null array");
  return plan_and_upload(h, &f, 1, causal, workspace_dev, workspace_bytes, pinned_host, pinned_bytes, stream);
}

int32_t fi_plan_formats(fi_handle* h, int32_t n_formats, const int32_t* const* qo_indptr, const int32_t* const* kv_indptr,
                        const int32_t* const* last_page_len, const int32_t* batch, const int32_t* kv_indices_base,
                        void* workspace_dev, size_t workspace_bytes, void* pinned_host, size_t pinned_bytes,
                        fi_stream stream) {
  if (!h) return set_error(FI_ERR_INVALID_ARG, "fi_plan_formats: null handle");
  if (h->cfg.mode != FI_MODE_TILE16 && h->cfg.mode != FI_MODE_TILE64)
    return set_error(FI_ERR_UNSUPPORTED, "fi_plan_formats: needs a handle in FI_MODE_TILE16 or FI_MODE_TILE64 (one kernel runs the tiles of every format)");
  if (n_formats < 1 || n_formats > kMaxFormats)
    return set_error(FI_ERR_INVALID_ARG, "fi_plan_formats: n_formats must be between 1 and " + std::to_string(kMaxFormats));
  if (!qo_indptr || !kv_indptr || !last_page_len || !batch || !kv_indices_base)
    return set_error(FI_ERR_INVALID_ARG, "fi_plan_formats: null array");
  FormatView f[kMaxFormats];
  for (int32_t i = 0; i < n_formats; ++i) {
    if (!qo_indptr[i] || !kv_indptr[i]) return set_error(FI_ERR_INVALID_ARG, "fi_plan_formats: null array");
    f[i].qo_indptr = qo_indptr[i];
    f[i].kv_indptr = kv_indptr[i];
    f[i].last_page_len = last_page_len[i];
    f[i].batch = batch[i];
    f[i].kv_base = kv_indices_base[i];
  }
  return plan_and_upload(h, f, n_formats, 0, workspace_dev, workspace_bytes, pinned_host, pinned_bytes, stream);
}

int32_t fi_plan_view(const fi_handle* h, fi_plan_arrays* out) {
  if (!h || !out) return set_error(FI_ERR_INVALID_ARG, "fi_plan_view: null argument");
  if (!h->planned_host) return set_error(FI_ERR_NOT_PLANNED, "fi_plan_view: no successful fi_plan yet");
  const WorkspaceLayout& L = h->layout;
  const int32_t* base = h->host_plan.data();
  const int32_t* hdr = base + L.off_header;
  out->t_pos = h->pp.t_pos;
  out->group = h->pp.group;
  out->ctas_per_head = h->pp.ctas_per_head;
  out->l_kv_chunk = hdr[H_L_KV];
  out->n_work = hdr[H_N_WORK];
  out->n_merge = hdr[H_N_MERGE];
  out->n_slots = hdr[H_N_SLOTS];
  out->pad_ = 0;
  out->cta_indptr = base + L.off_cta_indptr;
  out->w_request = base + L.off_work[W_REQUEST];
  out->w_q_row0 = base + L.off_work[W_Q_ROW0];
  out->w_n_pos = base + L.off_work[W_N_POS];
  out->w_kv_page0 = base + L.off_work[W_KV_PAGE0];
  out->w_kv_start = base + L.off_work[W_KV_START];
  out->w_kv_len = base + L.off_work[W_KV_LEN];
  out->w_diag0 = base + L.off_work[W_DIAG0];
  out->w_out_slot = base + L.off_work[W_OUT_SLOT];
  out->w_merge = base + L.off_work[W_MERGE];
  out->m_q_row0 = base + L.off_merge[M_Q_ROW0];
  out->m_n_pos = base + L.off_merge[M_N_POS];
  out->m_slot_base = base + L.off_merge[M_SLOT_BASE];
  out->m_n_chunks = base + L.off_merge[M_N_CHUNKS];
  out->n_rows = hdr[H_N_ROWS];
  out->pad2_ = 0;
  out->row_indptr = hdr[H_N_ROWS] > 0 ? base + L.off_row_indptr : nullptr;
  out->row_entry = hdr[H_N_ROWS] > 0 ? base + L.off_row_entry : nullptr;
  return FI_OK;
}

}  // namespace impl

namespace {
// fi_run and fi_run_kv8: kv8 = the pools hold E4M3 codes whose values are code * k_scale (v_scale)
int32_t run_impl(fi_handle* h, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides,
                 const int32_t* kv_indices, float sm_scale, bool kv8, float k_scale, float v_scale, float* o,
                 float* lse, void* o_cast, fi_stream stream, const fi_variant* variant = nullptr,
                 const int32_t* kv_indptr_dev = nullptr, const int32_t* last_page_len_dev = nullptr,
                 MergeParams* deferred = nullptr) {
  // deferred != null: the contraction launch is left to the caller, who gets its parameters
  if (!h) return set_error(FI_ERR_INVALID_ARG, "fi_run: null handle");
  if (variant) {
    if (h->cfg.mode == FI_MODE_TILE16 || h->cfg.mode == FI_MODE_TILE64)
      return set_error(FI_ERR_UNSUPPORTED, "fi_run_variant: not built for the 16-row and 64-row tile modes");
    if (h->cfg.page_size != kPageSize && h->cfg.mode == FI_MODE_DECODE && variant->rope_theta > 0.f)
      return set_error(FI_ERR_UNSUPPORTED, "fi_run_variant: the rotary embedding in decode mode is built for page_size 16");
    if (h->cfg.mode != FI_MODE_DECODE && !h->pp_causal_last)
      return set_error(FI_ERR_UNSUPPORTED, "fi_run_variant: in append mode the batch must be planned with causal = 1");
    if (!kv_indptr_dev || !last_page_len_dev) return set_error(FI_ERR_INVALID_ARG, "fi_run_variant: null pointer");
    if (!(variant->logits_soft_cap >= 0.f) || variant->window_left < -1)
      return set_error(FI_ERR_INVALID_ARG, "fi_run_variant: logits_soft_cap must be >= 0 and window_left >= -1");
    if (!(variant->rope_theta >= 0.f) || !(variant->rope_scale >= 0.f) || std::isinf(variant->rope_theta) ||
        std::isinf(variant->rope_scale))
      return set_error(FI_ERR_INVALID_ARG, "fi_run_variant: rope_theta and rope_scale must be finite and >= 0");
  }
  if (h->pp.plan_window > 0 && !(variant && variant->window_left >= 0 && variant->window_left < h->pp.plan_window))
    return set_error(FI_ERR_INVALID_ARG, "fi_run: the handle plans a sliding window of " + std::to_string(h->pp.plan_window) +
                                             " keys: run it with fi_run_variant and 0 <= window_left <= plan_window - 1");
  if (kv8 && h->cfg.mode != FI_MODE_DECODE)
    return set_error(FI_ERR_UNSUPPORTED, "fi_run_kv8: the 8-bit KV cache is built for decode mode only");
  if (deferred && h->n_formats_last > 1)
    return set_error(FI_ERR_UNSUPPORTED, "fi_run_composed: a handle planned over several formats composes them by itself (fi_run)");
  if (kv8 && !(k_scale > 0.f && v_scale > 0.f))
    return set_error(FI_ERR_INVALID_ARG, "fi_run_kv8: k_scale and v_scale must be > 0");
  if (!h->planned_dev) return set_error(FI_ERR_NOT_PLANNED, "fi_run: call fi_plan with a device workspace first");
  if (!q || !k_pool || !v_pool || !kv_strides || !lse) return set_error(FI_ERR_INVALID_ARG, "fi_run: null pointer");
  if (!kv_indices && (kv8 || variant || h->cfg.mode == FI_MODE_TILE16 || h->cfg.mode == FI_MODE_TILE64 || deferred))
    return set_error(FI_ERR_UNSUPPORTED, "fi_run: contiguous KV (kv_indices = NULL) is built for fi_run in decode and append mode");
  if (!o && !o_cast) return set_error(FI_ERR_INVALID_ARG, "fi_run: o and o_cast are both null: nowhere to write the output");
  if (!(sm_scale > 0.f)) return set_error(FI_ERR_INVALID_ARG, "fi_run: sm_scale must be > 0");
  if (kv_strides[0] <= 0 || kv_strides[1] <= 0 || kv_strides[2] < kHeadDim || kv_strides[0] % 8 != 0 ||
      kv_strides[1] % 8 != 0 || kv_strides[2] % 8 != 0)
    return set_error(FI_ERR_INVALID_ARG,
                     "fi_run: kv strides must be positive multiples of 8 elements, slot stride >= head_dim");
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) |
       reinterpret_cast<uintptr_t>(o) | reinterpret_cast<uintptr_t>(o_cast)) & 15)
    return set_error(FI_ERR_INVALID_ARG, "fi_run: q, k_pool, v_pool, o, o_cast must be 16-byte aligned");

  const WorkspaceLayout& L = h->layout;
  const int32_t* plan = static_cast<const int32_t*>(h->workspace_dev);
  char* ws = static_cast<char*>(h->workspace_dev);
  RunParams p{};
  p.cta_indptr = plan + L.off_cta_indptr;
  p.w_q_row0 = plan + L.off_work[W_Q_ROW0];
  p.w_n_pos = plan + L.off_work[W_N_POS];
  p.w_kv_page0 = plan + L.off_work[W_KV_PAGE0];
  p.w_kv_start = plan + L.off_work[W_KV_START];
  p.w_kv_len = plan + L.off_work[W_KV_LEN];
  p.w_diag0 = plan + L.off_work[W_DIAG0];
  p.w_out_slot = plan + L.off_work[W_OUT_SLOT];
  const bool fused_merge = h->cfg.mode == FI_MODE_DECODE && h->cfg.merge == 2;
  p.w_merge = fused_merge ? plan + L.off_work[W_MERGE] : nullptr;
  p.m_slot_base = plan + L.off_merge[M_SLOT_BASE];
  p.m_n_chunks = plan + L.off_merge[M_N_CHUNKS];
  p.merge_counters = const_cast<int32_t*>(plan) + L.off_counters;
  p.kv_indices = kv_indices;
  p.q = q;
  p.k_pool = k_pool;
  p.v_pool = v_pool;
  p.stride_page = kv_strides[0];
  p.stride_head = kv_strides[1];
  p.stride_tok = kv_strides[2];
  p.o = o;
  p.lse = lse;
  p.o_cast = o_cast;
  p.part_lse = reinterpret_cast<float*>(ws + L.off_part_lse);
  p.part_o = reinterpret_cast<float*>(ws + L.off_part_o);
  p.scale_log2 = sm_scale * 1.4426950408889634f * (kv8 ? k_scale : 1.f);
  p.out_scale = kv8 ? v_scale : 1.f;
  p.num_qo_heads = h->cfg.num_qo_heads;
  p.num_kv_heads = h->cfg.num_kv_heads;
  p.group = h->pp.group;
  p.t_pos = h->pp.t_pos;
  p.ctas_per_head = h->pp.ctas_per_head;
  p.w_request = plan + L.off_work[W_REQUEST];
  p.kv_indptr = kv_indptr_dev;
  p.last_page_len = last_page_len_dev;
  p.alibi_slopes = variant ? variant->alibi_slopes : nullptr;
  p.soft_cap = variant ? variant->logits_soft_cap : 0.f;
  p.cap_k1 = p.soft_cap > 0.f ? 2.0f * p.scale_log2 / p.soft_cap : 0.f;
  p.cap_a = p.soft_cap * 1.4426950408889634f;
  p.window_left = variant ? variant->window_left : -1;
  p.page_log2 = 0;
  while ((1 << p.page_log2) < h->cfg.page_size) ++p.page_log2;
  const bool bf = h->cfg.dtype == FI_DTYPE_BF16;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (h->ev_before && (e = hipEventRecord(h->ev_before, s)) != hipSuccess) return hip_error("fi_run: hipEventRecord", e);
  RopeTable rope;
  const bool with_rope = variant && variant->rope_theta > 0.f;
  if (with_rope) {
    // revolutions per position of pair d, in double precision; the kernel reduces 256 * t1 + t0 positions with
    // the fraction of 256 times that
    const double scale = variant->rope_scale > 0.f ? static_cast<double>(variant->rope_scale) : 1.0;
    for (int d = 0; d < kHeadDim / 2; ++d) {
      const double rev = std::pow(static_cast<double>(variant->rope_theta), -2.0 * d / kHeadDim) /
                         (2.0 * 3.14159265358979323846) / scale;
      rope.rev[d] = static_cast<float>(rev);
      rope.rev256[d] = static_cast<float>(256.0 * rev - std::floor(256.0 * rev));
    }
  }
  e = h->cfg.mode == FI_MODE_DECODE   ? launch_decode(p, bf, kv8, variant != nullptr, with_rope ? &rope : nullptr, s)
      : h->cfg.mode == FI_MODE_TILE16 ? launch_tiles(p, bf, s)
      : h->cfg.mode == FI_MODE_TILE64 ? launch_tiles64(p, bf, s)
                                      : launch_append(p, bf, variant != nullptr, with_rope ? &rope : nullptr, s);
  if (e != hipSuccess) return hip_error("fi_run: attention launch", e);
  if (h->ev_after && (e = hipEventRecord(h->ev_after, s)) != hipSuccess) return hip_error("fi_run: hipEventRecord", e);

  if (fused_merge) return FI_OK;  // the attention launch has folded the partial states itself
  if (h->n_formats_last > 1) {  // several formats: every query row folds the partial states on its list
    RowMergeParams rp{};
    rp.header = plan + L.off_header;
    rp.row_indptr = plan + L.off_row_indptr;
    rp.row_entry = plan + L.off_row_entry;
    rp.part_o = p.part_o;
    rp.part_lse = p.part_lse;
    rp.o = o;
    rp.lse = lse;
    rp.o_cast = o_cast;
    rp.num_qo_heads = h->cfg.num_qo_heads;
    rp.is_bf16 = bf ? 1 : 0;
    e = launch_merge_rows(rp, kMergeGrid, s);
    if (e != hipSuccess) return hip_error("fi_run: row contraction launch", e);
    return FI_OK;
  }
  MergeParams mp{};
  mp.header = plan + L.off_header;
  mp.m_q_row0 = plan + L.off_merge[M_Q_ROW0];
  mp.m_n_pos = plan + L.off_merge[M_N_POS];
  mp.m_slot_base = plan + L.off_merge[M_SLOT_BASE];
  mp.m_n_chunks = plan + L.off_merge[M_N_CHUNKS];
  mp.part_o = p.part_o;
  mp.part_lse = p.part_lse;
  mp.o = o;
  mp.lse = lse;
  mp.o_cast = o_cast;
  mp.num_qo_heads = h->cfg.num_qo_heads;
  mp.t_pos = h->pp.t_pos;
  mp.is_bf16 = bf ? 1 : 0;
  mp.max_merge = L.max_merge;
  if (deferred) {
    *deferred = mp;
    return FI_OK;
  }
  e = launch_merge_planned(mp, kMergeGrid, s);
  if (e != hipSuccess) return hip_error("fi_run: merge launch", e);
  return FI_OK;
}
}  // namespace

namespace impl {

int32_t fi_run(fi_handle* h, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides,
               const int32_t* kv_indices, float sm_scale, float* o, float* lse, void* o_cast, fi_stream stream) {
  return run_impl(h, q, k_pool, v_pool, kv_strides, kv_indices, sm_scale, false, 1.f, 1.f, o, lse, o_cast, stream);
}

int32_t fi_run_variant(fi_handle* h, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides,
                       const int32_t* kv_indices, const int32_t* kv_indptr, const int32_t* last_page_len,
                       float sm_scale, const fi_variant* variant, float* o, float* lse, void* o_cast,
                       fi_stream stream) {
  if (!variant) return set_error(FI_ERR_INVALID_ARG, "fi_run_variant: null variant");
  return run_impl(h, q, k_pool, v_pool, kv_strides, kv_indices, sm_scale, false, 1.f, 1.f, o, lse, o_cast, stream,
                  variant, kv_indptr, last_page_len);
}

int32_t fi_run_kv8(fi_handle* h, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides,
                   const int32_t* kv_indices, float sm_scale, float k_scale, float v_scale, float* o, float* lse,
                   void* o_cast, fi_stream stream) {
  return run_impl(h, q, k_pool, v_pool, kv_strides, kv_indices, sm_scale, true, k_scale, v_scale, o, lse, o_cast,
                  stream);
}

int32_t fi_run_composed(fi_handle* h_a, fi_handle* h_b, const void* q, const void* k_pool, const void* v_pool,
                        const int64_t* kv_strides, const int32_t* kv_indices_a, const int32_t* kv_indices_b,
                        float sm_scale, float* o_a, float* lse_a, float* o_b, float* lse_b, int64_t nnz_qo, float* o,
                        float* lse, void* o_cast, fi_stream stream) {
  if (!h_a || !h_b) return set_error(FI_ERR_INVALID_ARG, "fi_run_composed: null handle");
  if (h_a == h_b) return set_error(FI_ERR_INVALID_ARG, "fi_run_composed: the two passes need a handle (and workspace) each");
  if (h_a->cfg.dtype != h_b->cfg.dtype || h_a->cfg.num_qo_heads != h_b->cfg.num_qo_heads ||
      h_a->cfg.num_kv_heads != h_b->cfg.num_kv_heads)
    return set_error(FI_ERR_INVALID_ARG, "fi_run_composed: the two handles differ in dtype or head counts");
  if (h_a->cfg.merge == 2 || h_b->cfg.merge == 2)
    return set_error(FI_ERR_UNSUPPORTED, "fi_run_composed: handles with the contraction inside the attention launch (merge = 2)");
  if (h_a->cfg.plan_window > 0 || h_b->cfg.plan_window > 0)
    return set_error(FI_ERR_UNSUPPORTED, "fi_run_composed: handles that plan a sliding window");
  if (!h_a->planned_dev || !h_b->planned_dev)
    return set_error(FI_ERR_NOT_PLANNED, "fi_run_composed: call fi_plan with a device workspace on both handles first");
  if (h_a->workspace_dev == h_b->workspace_dev)
    return set_error(FI_ERR_INVALID_ARG, "fi_run_composed: the two passes share one workspace");
  if (nnz_qo != h_a->nnz_qo_last || nnz_qo != h_b->nnz_qo_last)
    return set_error(FI_ERR_INVALID_ARG, "fi_run_composed: both plans must cover the same nnz_qo query rows (" +
                                             std::to_string(h_a->nnz_qo_last) + ", " + std::to_string(h_b->nnz_qo_last) +
                                             " planned, " + std::to_string(nnz_qo) + " given)");
  if (!o_a || !lse_a || !o_b || !lse_b || !lse || (!o && !o_cast))
    return set_error(FI_ERR_INVALID_ARG, "fi_run_composed: null pointer");
  if (o_a == o_b || lse_a == lse_b) return set_error(FI_ERR_INVALID_ARG, "fi_run_composed: the passes need state rows of their own");
  if ((reinterpret_cast<uintptr_t>(o) | reinterpret_cast<uintptr_t>(o_cast)) & 15)
    return set_error(FI_ERR_INVALID_ARG, "fi_run_composed: o, o_cast must be 16-byte aligned");
  ComposeParams cp{};
  int32_t rc = run_impl(h_a, q, k_pool, v_pool, kv_strides, kv_indices_a, sm_scale, false, 1.f, 1.f, o_a, lse_a, nullptr,
                        stream, nullptr, nullptr, nullptr, &cp.a);
  if (rc != FI_OK) return rc;
  rc = run_impl(h_b, q, k_pool, v_pool, kv_strides, kv_indices_b, sm_scale, false, 1.f, 1.f, o_b, lse_b, nullptr, stream,
                nullptr, nullptr, nullptr, &cp.b);
  if (rc != FI_OK) return rc;
  cp.o = o;
  cp.lse = lse;
  cp.o_cast = o_cast;
  cp.nnz_qo = nnz_qo;
  const hipError_t e = launch_compose(cp, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_error("fi_run_composed: contraction launch", e);
  return FI_OK;
}

int32_t fi_run_composed_static(fi_handle* h_a, fi_handle* h_b, const void* q, const void* k_pool, const void* v_pool,
                               const int64_t* kv_strides, const int32_t* kv_indices_a, const int32_t* kv_indices_b,
                               float sm_scale, int64_t nnz_qo, float* o, float* lse, void* o_cast, fi_stream stream) {
  if (!h_a || !h_b) return set_error(FI_ERR_INVALID_ARG, "fi_run_composed_static: null handle");
  if (nnz_qo < 0 || nnz_qo * h_a->cfg.num_qo_heads > kStaticRowsMax)
    return set_error(FI_ERR_WORKSPACE_TOO_SMALL,
                     "fi_run_composed_static: " + std::to_string(nnz_qo) + " query rows x " +
                         std::to_string(h_a->cfg.num_qo_heads) + " heads exceed the " + std::to_string(kStaticRowsMax) +
                         " state rows of the library's static scratch memory; use fi_run_composed with buffers of your own");
  unsigned char* base = nullptr;
  const int32_t rc = static_scratch(&base);
  if (rc != FI_OK) return rc;
  // fixed offsets, whatever nnz_qo is: the same four pointers on every call.  Nothing has to start at zero: the
  // attention kernels write every state row the contraction reads (rows of split tiles are read from the handles'
  // workspaces instead).
  float* o_a = reinterpret_cast<float*>(base);
  float* o_b = reinterpret_cast<float*>(base + kStaticOBytes);
  float* lse_a = reinterpret_cast<float*>(base + 2 * kStaticOBytes);
  float* lse_b = reinterpret_cast<float*>(base + 2 * kStaticOBytes + kStaticLseBytes);
  return impl::fi_run_composed(h_a, h_b, q, k_pool, v_pool, kv_strides, kv_indices_a, kv_indices_b, sm_scale, o_a, lse_a,
                               o_b, lse_b, nnz_qo, o, lse, o_cast, stream);
}

int32_t fi_set_timing_events(fi_handle* h, void* before, void* after) {
  if (!h) return set_error(FI_ERR_INVALID_ARG, "fi_set_timing_events: null handle");
  if ((before == nullptr) != (after == nullptr))
    return set_error(FI_ERR_INVALID_ARG, "fi_set_timing_events: set both events or neither");
  h->ev_before = static_cast<hipEvent_t>(before);
  h->ev_after = static_cast<hipEvent_t>(after);
  return FI_OK;
}

int32_t fi_merge_states(const float* o_parts, const float* lse_parts, int64_t n_rows, int32_t n_states,
                        int32_t head_dim, float* o, float* lse, fi_stream stream) {
  if (head_dim != kHeadDim) return set_error(FI_ERR_UNSUPPORTED, "fi_merge_states: only head_dim = 128 is built");
  if (n_rows < 0 || n_states < 0) return set_error(FI_ERR_INVALID_ARG, "fi_merge_states: negative size");
  if (n_rows > 0 && (!o || !lse || (n_states > 0 && (!o_parts || !lse_parts))))
    return set_error(FI_ERR_INVALID_ARG, "fi_merge_states: null pointer");
  const hipError_t e = launch_merge_states(o_parts, lse_parts, n_rows, n_states, o, lse, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_error("fi_merge_states: launch", e);
  return FI_OK;
}

int32_t fi_merge_state_pair(const float* o_a, const float* lse_a, const float* o_b, const float* lse_b, int64_t n_rows,
                            int32_t head_dim, float* o, float* lse, fi_stream stream) {
  if (head_dim != kHeadDim) return set_error(FI_ERR_UNSUPPORTED, "fi_merge_state_pair: only head_dim = 128 is built");
  if (n_rows < 0) return set_error(FI_ERR_INVALID_ARG, "fi_merge_state_pair: negative size");
  if (n_rows > 0 && (!o_a || !lse_a || !o_b || !lse_b || !o || !lse))
    return set_error(FI_ERR_INVALID_ARG, "fi_merge_state_pair: null pointer");
  const hipError_t e = launch_merge_pair(o_a, lse_a, o_b, lse_b, n_rows, o, lse, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_error("fi_merge_state_pair: launch", e);
  return FI_OK;
}

int32_t fi_suggest_mode(int32_t num_qo_heads, int32_t num_kv_heads, double mean_qo_len) {
  if (num_qo_heads <= 0 || num_kv_heads <= 0 || num_qo_heads % num_kv_heads != 0 || !(mean_qo_len >= 0))
    return set_error(FI_ERR_INVALID_ARG, "fi_suggest_mode: heads must be positive, num_qo_heads a multiple of num_kv_heads, mean_qo_len >= 0");
  const double rows = mean_qo_len * (num_qo_heads / num_kv_heads);  // fused rows per request and kv head
  if (mean_qo_len <= 1.0) return FI_MODE_DECODE;
  if (rows <= 16.0) return FI_MODE_TILE64;
  return FI_MODE_APPEND;
}

int32_t fi_check_indices(const int32_t* indices_host, int64_t n, int32_t num_pages) {
  if (n < 0 || (n > 0 && !indices_host)) return set_error(FI_ERR_INVALID_ARG, "fi_check_indices: bad arguments");
  for (int64_t i = 0; i < n; ++i)
    if (indices_host[i] < 0 || indices_host[i] >= num_pages)
      return set_error(FI_ERR_INVALID_ARG, "fi_check_indices: indices[" + std::to_string(i) + "] = " +
                                               std::to_string(indices_host[i]) + " outside [0, " +
                                               std::to_string(num_pages) + ")");
  return FI_OK;
}

}  // namespace impl

// ---- the exported C symbols: the functions above, with every C++ exception turned into a status ----
extern "C" {

const char* fi_last_error(void) { return g_fixed_error ? g_fixed_error : g_last_error.c_str(); }

int32_t fi_create(const fi_config* cfg, fi_handle** out) {
  return guarded([&]() -> int32_t { return impl::fi_create(cfg, out); });
}

int32_t fi_destroy(fi_handle* h) {
  return guarded([&]() -> int32_t { return impl::fi_destroy(h); });
}

int32_t fi_workspace_bytes(const fi_handle* h, size_t* device_bytes, size_t* pinned_host_bytes) {
  return guarded([&]() -> int32_t { return impl::fi_workspace_bytes(h, device_bytes, pinned_host_bytes); });
}

int32_t fi_plan(fi_handle* h, const int32_t* qo_indptr, const int32_t* kv_indptr, const int32_t* last_page_len, int32_t batch, int32_t causal, void* workspace_dev, size_t workspace_bytes, void* pinned_host, size_t pinned_bytes, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_plan(h, qo_indptr, kv_indptr, last_page_len, batch, causal, workspace_dev, workspace_bytes, pinned_host, pinned_bytes, stream); });
}

int32_t fi_plan_formats(fi_handle* h, int32_t n_formats, const int32_t* const* qo_indptr, const int32_t* const* kv_indptr, const int32_t* const* last_page_len, const int32_t* batch, const int32_t* kv_indices_base, void* workspace_dev, size_t workspace_bytes, void* pinned_host, size_t pinned_bytes, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_plan_formats(h, n_formats, qo_indptr, kv_indptr, last_page_len, batch, kv_indices_base, workspace_dev, workspace_bytes, pinned_host, pinned_bytes, stream); });
}

int32_t fi_plan_view(const fi_handle* h, fi_plan_arrays* out) {
  return guarded([&]() -> int32_t { return impl::fi_plan_view(h, out); });
}

int32_t fi_run(fi_handle* h, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides, const int32_t* kv_indices, float sm_scale, float* o, float* lse, void* o_cast, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_run(h, q, k_pool, v_pool, kv_strides, kv_indices, sm_scale, o, lse, o_cast, stream); });
}

int32_t fi_run_variant(fi_handle* h, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides, const int32_t* kv_indices, const int32_t* kv_indptr, const int32_t* last_page_len, float sm_scale, const fi_variant* variant, float* o, float* lse, void* o_cast, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_run_variant(h, q, k_pool, v_pool, kv_strides, kv_indices, kv_indptr, last_page_len, sm_scale, variant, o, lse, o_cast, stream); });
}

int32_t fi_run_kv8(fi_handle* h, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides, const int32_t* kv_indices, float sm_scale, float k_scale, float v_scale, float* o, float* lse, void* o_cast, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_run_kv8(h, q, k_pool, v_pool, kv_strides, kv_indices, sm_scale, k_scale, v_scale, o, lse, o_cast, stream); });
}

int32_t fi_run_composed(fi_handle* h_a, fi_handle* h_b, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides, const int32_t* kv_indices_a, const int32_t* kv_indices_b, float sm_scale, float* o_a, float* lse_a, float* o_b, float* lse_b, int64_t nnz_qo, float* o, float* lse, void* o_cast, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_run_composed(h_a, h_b, q, k_pool, v_pool, kv_strides, kv_indices_a, kv_indices_b, sm_scale, o_a, lse_a, o_b, lse_b, nnz_qo, o, lse, o_cast, stream); });
}

int32_t fi_run_composed_static(fi_handle* h_a, fi_handle* h_b, const void* q, const void* k_pool, const void* v_pool, const int64_t* kv_strides, const int32_t* kv_indices_a, const int32_t* kv_indices_b, float sm_scale, int64_t nnz_qo, float* o, float* lse, void* o_cast, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_run_composed_static(h_a, h_b, q, k_pool, v_pool, kv_strides, kv_indices_a, kv_indices_b, sm_scale, nnz_qo, o, lse, o_cast, stream); });
}

int32_t fi_set_timing_events(fi_handle* h, void* before, void* after) {
  return guarded([&]() -> int32_t { return impl::fi_set_timing_events(h, before, after); });
}

int32_t fi_merge_states(const float* o_parts, const float* lse_parts, int64_t n_rows, int32_t n_states, int32_t head_dim, float* o, float* lse, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_merge_states(o_parts, lse_parts, n_rows, n_states, head_dim, o, lse, stream); });
}

int32_t fi_merge_state_pair(const float* o_a, const float* lse_a, const float* o_b, const float* lse_b, int64_t n_rows, int32_t head_dim, float* o, float* lse, fi_stream stream) {
  return guarded([&]() -> int32_t { return impl::fi_merge_state_pair(o_a, lse_a, o_b, lse_b, n_rows, head_dim, o, lse, stream); });
}

int32_t fi_suggest_mode(int32_t num_qo_heads, int32_t num_kv_heads, double mean_qo_len) {
  return guarded([&]() -> int32_t { return impl::fi_suggest_mode(num_qo_heads, num_kv_heads, mean_qo_len); });
}

int32_t fi_check_indices(const int32_t* indices_host, int64_t n, int32_t num_pages) {
  return guarded([&]() -> int32_t { return impl::fi_check_indices(indices_host, n, num_pages); });
}


}  // extern "C"
