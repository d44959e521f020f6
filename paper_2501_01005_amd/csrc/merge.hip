// Merge operator on attention states (Sec. 2.2): variable-length contraction of the
// partial states of split query tiles (Sec. 3.3.1), n-ary merge of caller-provided states,
// and the two-state merge that composes a shared-prefix pass with a per-request pass
// (Sec. 3.1.2).  A lane owns two of the 128 columns of a row.  The summation order is a
// function of the number of states only, so results are deterministic.
#include "kernels.h"
#include "plan.h"

namespace fi355 {
namespace {

typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;

constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLog2e = 1.4426950408889634f;

constexpr int kMergeWaves = 8;  // wavefronts that share one output row

// Folds n states of one row with the kMergeWaves wavefronts of a CTA.  State s has its lse at
// lse_ptr[s * lse_stride] and its 128-wide output at o_ptr + s * o_stride.  Wavefront w folds
// the contiguous range of states [w * per, (w + 1) * per) in ascending order, then wavefront 0
// adds the per-wavefront sums in ascending w: the summation order depends on n only.
// Returns (on wavefront 0) the merged pair for this lane's two columns.  Contains CTA barriers:
// every wavefront of the CTA must call it with the same arguments.
__device__ __forceinline__ void fold_row(const float* lse_ptr, int64_t lse_stride, const float* o_ptr,
                                         int64_t o_stride, int n, int wave, int lane, float* red_acc,
                                         float* red_den, f32x2_t* o_out, float* lse_out) {
  const float NEG_INF = -__builtin_inff();
  // pass 1 (every wavefront, redundantly): maximum lse
  float mx = NEG_INF;
  for (int s = lane; s < n; s += 64) mx = fmaxf(mx, lse_ptr[s * lse_stride]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  const float mx_safe = (mx == NEG_INF) ? 0.f : mx;
  // pass 2: weights exp(lse_s - max)
  const int per = (n + kMergeWaves - 1) / kMergeWaves;
  const int s_begin = min(wave * per, n);
  const int s_end = min(s_begin + per, n);
  f32x2_t acc = {0.f, 0.f};
  float den = 0.f;
  for (int s0 = s_begin; s0 < s_end; s0 += 64) {
    const int s_mine = s0 + lane;
    const float w_mine =
        (s_mine < s_end) ? __builtin_amdgcn_exp2f((lse_ptr[s_mine * lse_stride] - mx_safe) * kLog2e) : 0.f;
    const int cnt = min(64, s_end - s0);
    for (int j0 = 0; j0 < cnt; j0 += 8) {
      f32x2_t v[8];
      float w[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int j = j0 + u;
        w[u] = (j < cnt) ? __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w_mine), j & 63))
                         : 0.f;
        v[u] = (j < cnt) ? *reinterpret_cast<const f32x2_t*>(o_ptr + (s0 + j) * o_stride + 2 * lane)
                         : f32x2_t{0.f, 0.f};
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (w[u] != 0.f) {  // an empty state contributes nothing, whatever rides on it
          acc += w[u] * v[u];
          den += w[u];
        }
      }
    }
  }
  __syncthreads();  // red_* free again
  *reinterpret_cast<f32x2_t*>(red_acc + wave * kHeadDim + 2 * lane) = acc;
  if (lane == 0) red_den[wave] = den;
  __syncthreads();
  if (wave == 0) {
    f32x2_t tot = {0.f, 0.f};
    float dtot = 0.f;
#pragma unroll
    for (int w2 = 0; w2 < kMergeWaves; ++w2) {
      tot += *reinterpret_cast<const f32x2_t*>(red_acc + w2 * kHeadDim + 2 * lane);
      dtot += red_den[w2];
    }
    if (dtot > 0.f) {
      const float inv = 1.0f / dtot;
      *o_out = tot * inv;
      *lse_out = mx_safe + __builtin_amdgcn_logf(dtot) * kLn2;
    } else {
      *o_out = f32x2_t{0.f, 0.f};
      *lse_out = NEG_INF;
    }
  }
}

// ---- fold_row by a single wavefront.  The same sums in the same order (eight contiguous ranges of states, each
// folded in ascending order, the range sums added in ascending order: a running sum per range that is added to
// the total when the next range starts), so the result is bit-identical to fold_row's; no LDS, no barriers, and
// all loads of the row's states go out at once.

// The loads of up to T states of a row (n >= 1; indices past n - 1 re-read the last state), issued back to back.
template <int T>
struct RowStates {
  float l_raw;  // lse of state min(lane, n - 1)
  f32x2_t v[T];
};
template <int T>
__device__ __forceinline__ void load_states(RowStates<T>* rs, const float* lse_ptr, int64_t lse_stride, const float* o_ptr,
                                            int64_t o_stride, int n, int lane) {
  rs->l_raw = lse_ptr[min(lane, n - 1) * lse_stride];
#pragma unroll
  for (int u = 0; u < T; ++u)
    rs->v[u] = *reinterpret_cast<const f32x2_t*>(o_ptr + min(u, n - 1) * o_stride + 2 * lane);
}
template <int T>
__device__ __forceinline__ void reduce_states(const RowStates<T>& rs, int n, int lane, f32x2_t* o_out, float* lse_out) {
  const float NEG_INF = -__builtin_inff();
  const float l_mine = lane < n ? rs.l_raw : NEG_INF;
  float mx = l_mine;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  const float mx_safe = (mx == NEG_INF) ? 0.f : mx;
  const float w_mine = lane < n ? __builtin_amdgcn_exp2f((l_mine - mx_safe) * kLog2e) : 0.f;
  const int per = (n + kMergeWaves - 1) / kMergeWaves;
  int next = per;  // first state of the next range
  f32x2_t tot = {0.f, 0.f}, cur = {0.f, 0.f};
  float dtot = 0.f, dcur = 0.f;
#pragma unroll
  for (int u = 0; u < T; ++u) {
    if (u < n) {  // wavefront-uniform
      if (u == next) {
        tot += cur;
        dtot += dcur;
        cur = f32x2_t{0.f, 0.f};
        dcur = 0.f;
        next += per;
      }
      const float w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w_mine), u));
      if (w != 0.f) {  // an empty state contributes nothing, whatever rides on it
        cur += w * rs.v[u];
        dcur += w;
      }
    }
  }
  tot += cur;
  dtot += dcur;
  if (dtot > 0.f) {
    const float inv = 1.0f / dtot;
    *o_out = tot * inv;
    *lse_out = mx_safe + __builtin_amdgcn_logf(dtot) * kLn2;
  } else {
    *o_out = f32x2_t{0.f, 0.f};
    *lse_out = NEG_INF;
  }
}

// Any number of states, T loads in flight at a time (the sums and their order do not depend on T).
template <int T = 32>
__device__ __forceinline__ void fold_row_wave(const float* lse_ptr, int64_t lse_stride, const float* o_ptr,
                                              int64_t o_stride, int n, int lane, f32x2_t* o_out, float* lse_out) {
  const float NEG_INF = -__builtin_inff();
  float mx = NEG_INF;
  for (int s = lane; s < n; s += 64) mx = fmaxf(mx, lse_ptr[s * lse_stride]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  const float mx_safe = (mx == NEG_INF) ? 0.f : mx;
  const int per = (n + kMergeWaves - 1) / kMergeWaves;
  int next = per;
  f32x2_t tot = {0.f, 0.f}, cur = {0.f, 0.f};
  float dtot = 0.f, dcur = 0.f;
  for (int s0 = 0; s0 < n; s0 += 64) {
    const float w_mine =
        (s0 + lane < n) ? __builtin_amdgcn_exp2f((lse_ptr[(s0 + lane) * lse_stride] - mx_safe) * kLog2e) : 0.f;
    const int cnt = min(64, n - s0);
    for (int j0 = 0; j0 < cnt; j0 += T) {
      f32x2_t v[T];
#pragma unroll
      for (int u = 0; u < T; ++u)
        v[u] = *reinterpret_cast<const f32x2_t*>(o_ptr + min(s0 + j0 + u, n - 1) * o_stride + 2 * lane);
#pragma unroll
      for (int u = 0; u < T; ++u) {
        const int st = s0 + j0 + u;
        if (st < n) {
          if (st == next) {
            tot += cur;
            dtot += dcur;
            cur = f32x2_t{0.f, 0.f};
            dcur = 0.f;
            next += per;
          }
          const float w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w_mine), (j0 + u) & 63));
          if (w != 0.f) {
            cur += w * v[u];
            dcur += w;
          }
        }
      }
    }
  }
  tot += cur;
  dtot += dcur;
  if (dtot > 0.f) {
    const float inv = 1.0f / dtot;
    *o_out = tot * inv;
    *lse_out = mx_safe + __builtin_amdgcn_logf(dtot) * kLn2;
  } else {
    *o_out = f32x2_t{0.f, 0.f};
    *lse_out = NEG_INF;
  }
}

__device__ __forceinline__ void store_cast(void* o_cast, int64_t row, int lane, f32x2_t v, int is_bf16) {
  uint32_t* dst = static_cast<uint32_t*>(o_cast) + row * (kHeadDim / 2) + lane;
  if (is_bf16) {
    bf16x2_t h = {static_cast<__bf16>(v[0]), static_cast<__bf16>(v[1])};
    *dst = __builtin_bit_cast(uint32_t, h);
  } else {
    f16x2_t h = {static_cast<_Float16>(v[0]), static_cast<_Float16>(v[1])};
    *dst = __builtin_bit_cast(uint32_t, h);
  }
}

__device__ __forceinline__ void planned_store(const MergeParams& p, int64_t out_row, int lane, f32x2_t o2, float l) {
  if (p.o != nullptr) *reinterpret_cast<f32x2_t*>(p.o + out_row * kHeadDim + 2 * lane) = o2;
  if (lane == 0) p.lse[out_row] = l;
  if (p.o_cast != nullptr) store_cast(p.o_cast, out_row, lane, o2, p.is_bf16);
}

// Fixed grid; the number of split tiles is read from the plan header on the device.
// One CTA (kMergeWaves wavefronts) per output row, grid-stride over rows.  (One row per wavefront with all of
// its loads in flight at once is not faster here, neither with eight consecutive rows per CTA nor with the
// rows dealt out over the CTAs: measured 2-4 us slower on batches of 16 requests, 1-2 us on the large ones.)
__global__ void __launch_bounds__(64 * kMergeWaves) merge_planned_kernel(const MergeParams p) {
  __shared__ float red_acc[kMergeWaves * kHeadDim];
  __shared__ float red_den[kMergeWaves];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n_merge = p.header[H_N_MERGE];
  const int H = p.num_qo_heads;
  // rows (position, head) of every split tile, up to the largest number of positions a split tile has (a query
  // tile of a short request holds fewer positions than t_pos: one, for a decode step in a tile mode)
  const int rows_per_tile = p.header[H_MERGE_POS] * H;
  const int64_t total = static_cast<int64_t>(n_merge) * rows_per_tile;
  // Many rows (query tiles of several positions: tens of thousands of rows of a few states each): a wavefront per
  // row, the row's loads all in flight at once, no LDS, no barriers; the same sums in the same order as fold_row,
  // hence the same bits whichever way a plan's rows are walked.
  if (total > 4 * static_cast<int64_t>(gridDim.x)) {
    for (int64_t r = static_cast<int64_t>(blockIdx.x) * kMergeWaves + wave; r < total;
         r += static_cast<int64_t>(gridDim.x) * kMergeWaves) {
      const int mt = static_cast<int>(r / rows_per_tile);
      const int rr = static_cast<int>(r % rows_per_tile);
      const int pos = rr / H;
      const int head = rr % H;
      if (pos >= p.m_n_pos[mt]) continue;  // wavefront-uniform
      const int n = p.m_n_chunks[mt];
      const int64_t slot_row0 = (static_cast<int64_t>(p.m_slot_base[mt]) * p.t_pos + pos) * H + head;
      const int64_t slot_stride = static_cast<int64_t>(p.t_pos) * H;
      f32x2_t o2;
      float l;
      if (n <= 8) {  // (a split tile has at least two chunks)
        RowStates<8> rs;
        load_states<8>(&rs, p.part_lse + slot_row0, slot_stride, p.part_o + slot_row0 * kHeadDim, slot_stride * kHeadDim, n, lane);
        reduce_states<8>(rs, n, lane, &o2, &l);
      } else {
        // (eight loads in flight: the kernel stays within 128 registers, two CTAs per CU, for the other way too)
        fold_row_wave<8>(p.part_lse + slot_row0, slot_stride, p.part_o + slot_row0 * kHeadDim, slot_stride * kHeadDim, n,
                         lane, &o2, &l);
      }
      planned_store(p, (static_cast<int64_t>(p.m_q_row0[mt]) + pos) * H + head, lane, o2, l);
    }
    return;
  }
  for (int64_t r = blockIdx.x; r < total; r += gridDim.x) {
    const int mt = static_cast<int>(r / rows_per_tile);
    const int rr = static_cast<int>(r % rows_per_tile);
    const int pos = rr / H;
    const int head = rr % H;
    if (pos >= p.m_n_pos[mt]) continue;  // CTA-uniform
    const int n = p.m_n_chunks[mt];
    const int64_t slot_row0 = (static_cast<int64_t>(p.m_slot_base[mt]) * p.t_pos + pos) * H + head;
    const int64_t slot_stride = static_cast<int64_t>(p.t_pos) * H;  // rows between consecutive slots
    f32x2_t o2;
    float l;
    fold_row(p.part_lse + slot_row0, slot_stride, p.part_o + slot_row0 * kHeadDim, slot_stride * kHeadDim, n, wave,
             lane, red_acc, red_den, &o2, &l);
    if (wave == 0) planned_store(p, (static_cast<int64_t>(p.m_q_row0[mt]) + pos) * H + head, lane, o2, l);
  }
}

__global__ void __launch_bounds__(64 * kMergeWaves) merge_states_kernel(const float* o_parts, const float* lse_parts,
                                                                        int64_t n_rows, int n_states, float* o,
                                                                        float* lse) {
  __shared__ float red_acc[kMergeWaves * kHeadDim];
  __shared__ float red_den[kMergeWaves];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  for (int64_t r = blockIdx.x; r < n_rows; r += gridDim.x) {
    f32x2_t o2;
    float l;
    fold_row(lse_parts + r * n_states, 1, o_parts + r * n_states * kHeadDim, kHeadDim, n_states, wave, lane, red_acc,
             red_den, &o2, &l);
    if (wave == 0) {
      *reinterpret_cast<f32x2_t*>(o + r * kHeadDim + 2 * lane) = o2;
      if (lane == 0) lse[r] = l;
    }
  }
}

// Merge of two states (Sec. 2.2) for this lane's two columns.
__device__ __forceinline__ void merge_two(float la, f32x2_t va, float lb, f32x2_t vb, f32x2_t* res_out, float* l_out) {
  const float NEG_INF = -__builtin_inff();
  const float mx = fmaxf(la, lb);
  f32x2_t res = {0.f, 0.f};
  float l = NEG_INF;
  if (mx != NEG_INF) {
    const float wa = __builtin_amdgcn_exp2f((la - mx) * kLog2e);
    const float wb = __builtin_amdgcn_exp2f((lb - mx) * kLog2e);
    const float den = wa + wb;
    const float inv = 1.0f / den;
    if (wa != 0.f) res += (wa * inv) * va;
    if (wb != 0.f) res += (wb * inv) * vb;
    l = mx + __builtin_amdgcn_logf(den) * kLn2;
  }
  *res_out = res;
  *l_out = l;
}

// Where the states of one pass for output row (pos, head) are: the partial states of the split tile of that
// pass's plan that holds the position, else the one row the attention kernel wrote (a single state, which folds
// to itself).  The first 64 entries of the merge list are read one per lane together with the header.
struct StateRun {
  const float* lse_ptr;
  const float* o_ptr;
  int64_t lse_stride, o_stride;
  int n;
};
__device__ __forceinline__ StateRun find_states(const MergeParams& m, int pos, int head, int lane) {
  const int n_merge = m.header[H_N_MERGE];
  const int mine = min(lane, m.max_merge - 1);
  int q0 = m.m_q_row0[mine], np = m.m_n_pos[mine], nc = m.m_n_chunks[mine], sb = m.m_slot_base[mine];
  int found_lane = -1;
  uint64_t mask = __ballot(lane < n_merge && pos >= q0 && pos < q0 + np);
  if (mask != 0) {
    found_lane = __builtin_ctzll(mask);
  } else {
    for (int base = 64; base < n_merge && found_lane < 0; base += 64) {
      const int mt = min(base + lane, m.max_merge - 1);
      q0 = m.m_q_row0[mt], np = m.m_n_pos[mt], nc = m.m_n_chunks[mt], sb = m.m_slot_base[mt];
      mask = __ballot(base + lane < n_merge && pos >= q0 && pos < q0 + np);
      if (mask != 0) found_lane = __builtin_ctzll(mask);
    }
  }
  const int H = m.num_qo_heads;
  StateRun run;
  if (found_lane >= 0) {
    const int f_q0 = __builtin_amdgcn_readlane(q0, found_lane);
    const int f_sb = __builtin_amdgcn_readlane(sb, found_lane);
    run.n = __builtin_amdgcn_readlane(nc, found_lane);
    const int64_t slot_row0 = (static_cast<int64_t>(f_sb) * m.t_pos + (pos - f_q0)) * H + head;
    run.lse_stride = static_cast<int64_t>(m.t_pos) * H;
    run.o_stride = run.lse_stride * kHeadDim;
    run.lse_ptr = m.part_lse + slot_row0;
    run.o_ptr = m.part_o + slot_row0 * kHeadDim;
  } else {
    const int64_t r = static_cast<int64_t>(pos) * H + head;
    run.n = 1;
    run.lse_stride = 0;
    run.o_stride = 0;
    run.lse_ptr = m.lse + r;
    run.o_ptr = m.o + r * kHeadDim;
  }
  return run;
}

template <int T>
__device__ __forceinline__ void compose_row_alone(const StateRun& a, const StateRun& b, int lane, f32x2_t* oa, float* la,
                                                  f32x2_t* ob, float* lb) {
  RowStates<T> ra, rb;  // the loads of both passes go out before either is reduced
  load_states<T>(&ra, a.lse_ptr, a.lse_stride, a.o_ptr, a.o_stride, a.n, lane);
  load_states<T>(&rb, b.lse_ptr, b.lse_stride, b.o_ptr, b.o_stride, b.n, lane);
  reduce_states<T>(ra, a.n, lane, oa, la);
  reduce_states<T>(rb, b.n, lane, ob, lb);
}

__device__ __forceinline__ void compose_store(const ComposeParams& p, int64_t r, int lane, float la, f32x2_t oa, float lb,
                                              f32x2_t ob) {
  f32x2_t res;
  float l;
  merge_two(la, oa, lb, ob, &res, &l);
  if (p.o != nullptr) *reinterpret_cast<f32x2_t*>(p.o + r * kHeadDim + 2 * lane) = res;
  if (lane == 0) p.lse[r] = l;
  if (p.o_cast != nullptr) store_cast(p.o_cast, r, lane, res, p.a.is_bf16);
}

// Composition of two passes over the same query rows (Sec. 3.1.2) in one launch: per output row the state of
// pass a and the state of pass b, each folded from its partial states where its tile was split, then merged.
// The arithmetic is that of the two contraction launches followed by the two-state merge.  One row per
// wavefront (eight consecutive rows per CTA), no barriers; the loads of both passes' states go out together.
__global__ void __launch_bounds__(64 * kMergeWaves) compose_kernel(const ComposeParams p) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int H = p.a.num_qo_heads;
  const int64_t total = p.nnz_qo * H;
  for (int64_t r = static_cast<int64_t>(blockIdx.x) * kMergeWaves + wave; r < total;
       r += static_cast<int64_t>(gridDim.x) * kMergeWaves) {
    const int pos = static_cast<int>(r / H);
    const int head = static_cast<int>(r % H);
    const StateRun a = find_states(p.a, pos, head, lane);
    const StateRun b = find_states(p.b, pos, head, lane);
    f32x2_t oa, ob;
    float la, lb;
    const int n = max(a.n, b.n);
    if (n <= 4) {
      compose_row_alone<4>(a, b, lane, &oa, &la, &ob, &lb);
    } else if (n <= 8) {
      compose_row_alone<8>(a, b, lane, &oa, &la, &ob, &lb);
    } else if (n <= 16) {
      compose_row_alone<16>(a, b, lane, &oa, &la, &ob, &lb);
    } else if (n <= 32) {
      compose_row_alone<32>(a, b, lane, &oa, &la, &ob, &lb);
    } else {
      fold_row_wave(a.lse_ptr, a.lse_stride, a.o_ptr, a.o_stride, a.n, lane, &oa, &la);
      fold_row_wave(b.lse_ptr, b.lse_stride, b.o_ptr, b.o_stride, b.n, lane, &ob, &lb);
    }
    compose_store(p, r, lane, la, oa, lb, ob);
  }
}

// Contraction of a plan over several formats (Sec. 3.1.2; Sec. 2.2): one wavefront per (query row, head) folds the
// row's partial states in list order (a left fold with a common reference, the maximum lse: every state weighs
// exp(lse_s - max)).  Fixed grid; the number of rows is read from the plan header.  Loads go out 16 states at a time.
__global__ void __launch_bounds__(64 * kMergeWaves) merge_rows_kernel(const RowMergeParams p) {
  const float NEG_INF = -__builtin_inff();
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int H = p.num_qo_heads;
  const int64_t total = static_cast<int64_t>(p.header[H_N_ROWS]) * H;
  for (int64_t r = static_cast<int64_t>(blockIdx.x) * kMergeWaves + wave; r < total;
       r += static_cast<int64_t>(gridDim.x) * kMergeWaves) {
    const int row = static_cast<int>(r / H);
    const int head = static_cast<int>(r % H);
    const int e0 = p.row_indptr[row];
    const int n = p.row_indptr[row + 1] - e0;
    float mx = NEG_INF;
    for (int s0 = 0; s0 < n; s0 += 64)
      if (s0 + lane < n) mx = fmaxf(mx, p.part_lse[static_cast<int64_t>(p.row_entry[e0 + s0 + lane]) * H + head]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    f32x2_t acc = {0.f, 0.f};
    float den = 0.f;
    if (mx != NEG_INF) {
      for (int s0 = 0; s0 < n; s0 += 16) {
        float l[16];
        f32x2_t v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          const int64_t prow = static_cast<int64_t>(p.row_entry[e0 + min(s0 + u, n - 1)]) * H + head;
          l[u] = p.part_lse[prow];
          v[u] = *reinterpret_cast<const f32x2_t*>(p.part_o + prow * kHeadDim + 2 * lane);
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          const float w = s0 + u < n ? __builtin_amdgcn_exp2f((l[u] - mx) * kLog2e) : 0.f;
          if (w != 0.f) {  // an empty state contributes nothing, whatever rides on it
            acc += w * v[u];
            den += w;
          }
        }
      }
    }
    f32x2_t res = {0.f, 0.f};
    float lse = NEG_INF;
    if (den > 0.f) {
      res = acc * (1.0f / den);
      lse = mx + __builtin_amdgcn_logf(den) * kLn2;
    }
    if (p.o != nullptr) *reinterpret_cast<f32x2_t*>(p.o + r * kHeadDim + 2 * lane) = res;
    if (lane == 0) p.lse[r] = lse;
    if (p.o_cast != nullptr) store_cast(p.o_cast, r, lane, res, p.is_bf16);
  }
}

__global__ void __launch_bounds__(256) merge_pair_kernel(const float* o_a, const float* lse_a, const float* o_b,
                                                         const float* lse_b, int64_t n_rows, float* o, float* lse) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t n_waves = static_cast<int64_t>(gridDim.x) * 4;
  for (int64_t r = wave; r < n_rows; r += n_waves) {
    const float la = lse_a[r], lb = lse_b[r];
    const f32x2_t va = *reinterpret_cast<const f32x2_t*>(o_a + r * kHeadDim + 2 * lane);
    const f32x2_t vb = *reinterpret_cast<const f32x2_t*>(o_b + r * kHeadDim + 2 * lane);
    f32x2_t res;
    float l;
    merge_two(la, va, lb, vb, &res, &l);
    *reinterpret_cast<f32x2_t*>(o + r * kHeadDim + 2 * lane) = res;
    if (lane == 0) lse[r] = l;
  }
}

int grid_for_rows(int64_t n_rows) {
  int64_t blocks = (n_rows + 3) / 4;
  if (blocks < 1) blocks = 1;
  if (blocks > 4096) blocks = 4096;
  return static_cast<int>(blocks);
}

}  // namespace

hipError_t launch_merge_planned(const MergeParams& p, int32_t grid, hipStream_t stream) {
  hipLaunchKernelGGL(merge_planned_kernel, dim3(grid), dim3(64 * kMergeWaves), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_merge_rows(const RowMergeParams& p, int32_t grid, hipStream_t stream) {
  hipLaunchKernelGGL(merge_rows_kernel, dim3(grid), dim3(64 * kMergeWaves), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_compose(const ComposeParams& p, hipStream_t stream) {
  const int64_t rows = p.nnz_qo * p.a.num_qo_heads;
  if (rows == 0) return hipSuccess;
  int64_t blocks = (rows + kMergeWaves - 1) / kMergeWaves;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(compose_kernel, dim3(static_cast<unsigned>(blocks)), dim3(64 * kMergeWaves), 0, stream, p);
  return hipGetLastError();
}

hipError_t launch_merge_states(const float* o_parts, const float* lse_parts, int64_t n_rows, int32_t n_states,
                               float* o, float* lse, hipStream_t stream) {
  if (n_rows == 0) return hipSuccess;
  const int64_t blocks = n_rows < 8192 ? n_rows : 8192;
  hipLaunchKernelGGL(merge_states_kernel, dim3(static_cast<unsigned>(blocks)), dim3(64 * kMergeWaves), 0, stream,
                     o_parts, lse_parts, n_rows, n_states, o, lse);
  return hipGetLastError();
}

hipError_t launch_merge_pair(const float* o_a, const float* lse_a, const float* o_b, const float* lse_b,
                             int64_t n_rows, float* o, float* lse, hipStream_t stream) {
  if (n_rows == 0) return hipSuccess;
  hipLaunchKernelGGL(merge_pair_kernel, dim3(grid_for_rows(n_rows)), dim3(256), 0, stream, o_a, lse_a, o_b, lse_b,
                     n_rows, o, lse);
  return hipGetLastError();
}

}  // namespace fi355
