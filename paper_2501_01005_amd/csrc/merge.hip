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

// Fixed grid; the number of split tiles is read from the plan header on the device.
// One CTA (kMergeWaves wavefronts) per output row, grid-stride over rows.
__global__ void __launch_bounds__(64 * kMergeWaves) merge_planned_kernel(const MergeParams p) {
  __shared__ float red_acc[kMergeWaves * kHeadDim];
  __shared__ float red_den[kMergeWaves];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n_merge = p.header[H_N_MERGE];
  const int H = p.num_qo_heads;
  const int rows_per_tile = p.t_pos * H;
  const int64_t total = static_cast<int64_t>(n_merge) * rows_per_tile;
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
    if (wave == 0) {
      const int64_t out_row = (static_cast<int64_t>(p.m_q_row0[mt]) + pos) * H + head;
      if (p.o != nullptr) *reinterpret_cast<f32x2_t*>(p.o + out_row * kHeadDim + 2 * lane) = o2;
      if (lane == 0) p.lse[out_row] = l;
      if (p.o_cast != nullptr) store_cast(p.o_cast, out_row, lane, o2, p.is_bf16);
    }
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

__global__ void __launch_bounds__(256) merge_pair_kernel(const float* o_a, const float* lse_a, const float* o_b,
                                                         const float* lse_b, int64_t n_rows, float* o, float* lse) {
  const float NEG_INF = -__builtin_inff();
  const int lane = threadIdx.x & 63;
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int64_t n_waves = static_cast<int64_t>(gridDim.x) * 4;
  for (int64_t r = wave; r < n_rows; r += n_waves) {
    const float la = lse_a[r], lb = lse_b[r];
    const f32x2_t va = *reinterpret_cast<const f32x2_t*>(o_a + r * kHeadDim + 2 * lane);
    const f32x2_t vb = *reinterpret_cast<const f32x2_t*>(o_b + r * kHeadDim + 2 * lane);
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
