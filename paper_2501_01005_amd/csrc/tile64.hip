// Query tiles of up to 64 fused rows (row R = position * g + head, App. A) for gfx950, CTAs of four wavefronts
// (Sec. 3.2.2: the tile size follows the query lengths).  Work items of one launch are of two kinds:
//
//   wide  (more than 16 live rows: a block of queries over a shared prefix, Sec. 3.1.2; a short append): wavefront w
//         owns rows 16 w .. 16 w + 15, and the four stage every 32-token step of K and V through LDS, a quarter of
//         the rows each, so that the CTA reads a K/V row once whatever the number of rows (the 16-row tile kernel
//         re-reads it per 16 rows: on the shared-prefix workload 451 MB of L2 requests for 92 MB of K/V; cutting
//         them fourfold gains 10 % there, the steps being chains of dependent phases rather than waits for data);
//   light (at most 16 live rows: a decode step): all four wavefronts hold the same rows, wavefront w walks steps
//         w, w + 4, ... of the chunk on its own (K through a private LDS area, V in registers, streaming loads),
//         and wavefront 0 merges the four states (Sec. 2.2) through LDS before the epilogue.  Four wavefronts side
//         by side keep as many bytes in flight per CU as the one-wavefront CTAs of the decode kernel.
//
// The products and the softmax of a step are those of the 16-row tile kernel (tile.hip):
//   S^T[token][row] = K . Q^T      v_mfma_f32_16x16x32, A = K rows (through LDS), B = Q^T
//   O^T[d][row]    += V^T . P^T    A = V^T built in-lane from row-major V rows, B = P^T from the S^T accumulators
// bf16: P enters the second product as head + remainder.  Causal items mask per row.  A row that has seen no key
// keeps the empty state (m = -inf, l = 0).
//
// The grid is one-dimensional with the kv head as the fast index (see tile.hip).
#include <type_traits>

#include "kernels.h"

namespace fi355 {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

constexpr int kWaves = 4;
constexpr int kStepTokens = 32;
// LDS, in 16-byte entries.  Wide items: two step buffers of 1024 entries (K: page pg, token t, 16-byte block x at
// pg * 256 + t * 16 + ((x ^ t) & 15); V: 512 + (pg * 4 + i) * 64 + lane).  Light items: a private K area of 512
// entries per wavefront in the same layout; afterwards the states of wavefronts 1..3 (8 x 64 entries each) and,
// from entry 1536, their (m, l) pairs.
constexpr int kLdsEntries = 2048;
constexpr int kBufEntries = 1024;
constexpr int kVOffset = 512;
constexpr int kStateEntries = 512;
constexpr int kMlOffset = 1536;

template <bool BF>
__device__ __forceinline__ f32x4_t mfma(u32x4_t a, u32x4_t b, f32x4_t c) {
  if constexpr (BF) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
}

template <bool BF>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  if constexpr (BF) {
    bf16x2_t v = {static_cast<__bf16>(lo), static_cast<__bf16>(hi)};
    return __builtin_bit_cast(uint32_t, v);
  } else {
    f16x2_t v = {static_cast<_Float16>(lo), static_cast<_Float16>(hi)};
    return __builtin_bit_cast(uint32_t, v);
  }
}

__device__ __forceinline__ float bf16_round(float x) { return static_cast<float>(static_cast<__bf16>(x)); }
// (a.lo16, b.lo16) and (a.hi16, b.hi16) packed as (first, second) halves of one dword
__device__ __forceinline__ uint32_t lo_halves(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t hi_halves(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// max / sum over the four 16-lane groups (lanes l, l ^ 16, l ^ 32, l ^ 48), the result in all of them: two register
// swaps between lane halves (a's lanes 32..63 <-> b's lanes 0..31) and between rows of 16 lanes (a's odd rows <-> b's
// even rows) instead of two round trips through the LDS crossbar.  Inline assembly, with the wait states the swaps
// need after a vector write of their operands: the compiler's builtin folds away when both operands are one value.
__device__ __forceinline__ float max_over_lane_groups(float x) {
  float a = x, b = x;
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_max_f32 %0, %0, %1\n\tv_mov_b32 %1, %0\n\t"
      "s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\tv_max_f32 %0, %0, %1"
      : "+v"(a), "+v"(b));
  return a;
}
__device__ __forceinline__ float sum_over_lane_groups(float x) {
  float a = x, b = x;
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_add_f32 %0, %0, %1\n\tv_mov_b32 %1, %0\n\t"
      "s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\tv_add_f32 %0, %0, %1"
      : "+v"(a), "+v"(b));
  return a;
}

struct KvStep {       // a whole 32-token step in one wavefront's registers (light items)
  u32x4_t k[2][4];    // [page][j]: K[token 4 j + c][d = 8 m .. +8]
  u32x4_t v[2][4];    // [page][i]: V[token 4 c + i][d = 8 m .. +8]
};
struct KvQuarter {    // this wavefront's share of a step (wide items): page w / 2, j and i = 2 (w % 2) + {0, 1}
  u32x4_t k[2];
  u32x4_t v[2];
};

template <bool BF>
__global__ void __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu(2, 2)))
tile64_kernel(const RunParams p) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) >> 6);
  const int m = lane & 15;  // K: token in page; V: 16-byte column block; S/O: row within the wavefront's 16 fused rows
  const int c = lane >> 4;  // lane group
  const int cta = static_cast<int>(blockIdx.x) / p.num_kv_heads;
  const int kvh = static_cast<int>(blockIdx.x) % p.num_kv_heads;
  const int g = p.group;
  const int g_log2 = 31 - __builtin_clz(g);
  const int H = p.num_qo_heads;
  const float NEG_INF = -__builtin_inff();

  const uint8_t* kbase = static_cast<const uint8_t*>(p.k_pool) + (kvh * p.stride_head + c * p.stride_tok + m * 8) * 2;
  const uint8_t* vbase = static_cast<const uint8_t*>(p.v_pool) + (kvh * p.stride_head + (4 * c) * p.stride_tok + m * 8) * 2;
  const int64_t stride_tok = p.stride_tok * 2;  // bytes
  const int64_t stride_page = p.stride_page * 2;
  __shared__ __attribute__((aligned(16))) u32x4_t lds[kLdsEntries];

  // plan arrays and page ids through the constant address space: wavefront-uniform scalar loads
  using ConstInts = const __attribute__((address_space(4))) int32_t*;
  auto as_const = [](const int32_t* ptr) { return (ConstInts)(reinterpret_cast<uintptr_t>(ptr)); };
  ConstInts cta_indptr = as_const(p.cta_indptr), page_ids = as_const(p.kv_indices);
  const int w_begin = cta_indptr[cta];
  const int w_end = cta_indptr[cta + 1];

  // Two passes over the CTA's queue, the wide items first: each pass holds one kind's loop only, so that the
  // registers of the other kind's tiles in flight are not live across it.
  auto work_item = [&](auto wide_tag, int w) {
    constexpr bool wide = decltype(wide_tag)::value;  // (a property of the item: the same for the whole CTA)
    const int q_row0 = as_const(p.w_q_row0)[w];
    const int kv_page0 = as_const(p.w_kv_page0)[w];
    const int kv_len = as_const(p.w_kv_len)[w];
    const int out_slot = as_const(p.w_out_slot)[w];
    const int diag0 = as_const(p.w_diag0)[w];
    const int rows = as_const(p.w_n_pos)[w] * g;  // live fused rows of the tile
    // causal items: chunk-local index of the last token the tile's first position sees (all tokens otherwise)
    const int lim_first = diag0 != kNoDiagMarker ? diag0 - as_const(p.w_kv_start)[w] : 0x3FFFFFFF;
    const int n_pages = (kv_len + 15) >> 4;
    const int n_steps = (kv_len + kStepTokens - 1) / kStepTokens;

    // this lane's row R -> (position, head); Q^T as the B operand of the first product: lane (m, c) holds row R,
    // d = 32 s + 8 c .. +8
    const int row_base = wide ? 16 * wave : 0;
    const bool live_wave = row_base < rows;  // wide items: a wavefront past the tile's rows only helps with the staging
    const int R = row_base + m;
    const int pos = R >> g_log2;
    const int lim = lim_first == 0x3FFFFFFF ? lim_first : lim_first + pos;
    u32x4_t qreg[4];
    f32x4_t acc[8];  // acc[e][i] = O^T[d = 32 c + 8 i + e][row R]
    float m_run = NEG_INF;  // running max of the scaled logits, log2 units (same in all 4 lane groups)
    float l_run = 0.f;      // this lane's share of the running sum
    if (R < rows) {
      const uint16_t* qp = static_cast<const uint16_t*>(p.q) +
                           (static_cast<int64_t>(q_row0 + pos) * H + kvh * g + (R & (g - 1))) * kHeadDim + c * 8;
#pragma unroll
      for (int s = 0; s < 4; ++s) qreg[s] = *reinterpret_cast<const u32x4_t*>(qp + 32 * s);
    } else {
#pragma unroll
      for (int s = 0; s < 4; ++s) qreg[s] = u32x4_t{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // one 32-token step of this wavefront's 16 rows: K operands from the LDS tile at `kt`, V rows in `v`
    auto compute_step = [&](const u32x4_t* kt, u32x4_t (&v)[2][4], int t) {
      f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const u32x4_t ka0 = kt[m * 16 + (((4 * s + c) ^ m) & 15)];
        const u32x4_t ka1 = kt[256 + m * 16 + (((4 * s + c) ^ m) & 15)];
        s0 = mfma<BF>(ka0, qreg[s], s0);
        s1 = mfma<BF>(ka1, qreg[s], s1);
      }
      // lane (m, c) now holds S^T[token 16 pg + 4 c + i][row R]
      const int tok0 = kStepTokens * t + 4 * c;
      const bool tail = kStepTokens * t + kStepTokens > kv_len;  // ragged end of the chunk
      if (tail) {  // V rows past the chunk must not reach the second product (0 x garbage need not be 0)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (tok0 + i >= kv_len) v[0][i] = u32x4_t{0u, 0u, 0u, 0u};
          if (tok0 + 16 + i >= kv_len) v[1][i] = u32x4_t{0u, 0u, 0u, 0u};
        }
      }
      // vt[e][pg * 2 + pr] = column e of tokens (2 pr, 2 pr + 1) of page pg, as a pair of 16-bit values
      u32x4_t vt[8];
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        const uint32_t a0 = v[0][0][wd], a1 = v[0][1][wd], a2 = v[0][2][wd], a3 = v[0][3][wd];
        const uint32_t b0 = v[1][0][wd], b1 = v[1][1][wd], b2 = v[1][2][wd], b3 = v[1][3][wd];
        vt[2 * wd] = u32x4_t{lo_halves(a0, a1), lo_halves(a2, a3), lo_halves(b0, b1), lo_halves(b2, b3)};
        vt[2 * wd + 1] = u32x4_t{hi_halves(a0, a1), hi_halves(a2, a3), hi_halves(b0, b1), hi_halves(b2, b3)};
      }
      float sv[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        sv[i] = s0[i] * p.scale_log2;
        sv[4 + i] = s1[i] * p.scale_log2;
      }
      if (kStepTokens * t + kStepTokens - 1 > lim_first || tail) {  // the causal diagonal or the end of the chunk cuts this step
        const int last = min(lim, kv_len - 1);
#pragma unroll
        for (int j = 0; j < 8; ++j) sv[j] = (tok0 + 16 * (j >> 2) + (j & 3) <= last) ? sv[j] : NEG_INF;
      }
      // ---- online softmax (Sec. 2.1) ----
      float tmax = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
      tmax = max_over_lane_groups(tmax);
      const float m_new = fmaxf(m_run, tmax);
      const bool none_yet = m_new == NEG_INF;  // the row has not seen a key so far
      const float alpha = none_yet ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      float pv[8];
      float psum = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        pv[j] = none_yet ? 0.f : __builtin_amdgcn_exp2f(sv[j] - m_new);
        psum += pv[j];
      }
      l_run = l_run * alpha + psum;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= alpha;
      }
      // ---- P^T as B operand: register j <-> (page j / 4, token 4 c + j % 4) ----
      const u32x4_t pb = {pack2<BF>(pv[0], pv[1]), pack2<BF>(pv[2], pv[3]), pack2<BF>(pv[4], pv[5]), pack2<BF>(pv[6], pv[7])};
      u32x4_t pb_lo = {0u, 0u, 0u, 0u};
      if constexpr (BF) {
        float r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = pv[j] - bf16_round(pv[j]);
        pb_lo = u32x4_t{pack2<BF>(r[0], r[1]), pack2<BF>(r[2], r[3]), pack2<BF>(r[4], r[5]), pack2<BF>(r[6], r[7])};
      }
      // ---- O^T += V^T . P^T, one product per column e of the lane's 8-wide block ----
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc[e] = mfma<BF>(vt[e], pb, acc[e]);
        if constexpr (BF) acc[e] = mfma<BF>(vt[e], pb_lo, acc[e]);
      }
    };

    if constexpr (wide) {
      // ---- the four wavefronts stage each step through LDS, three steps of loads in flight ----
      const int my_page = wave >> 1;        // which of the step's two pages this wavefront loads from
      const int my_first = 2 * (wave & 1);  // its two row groups j (K: tokens 4 j + c) and rows i (V: tokens 4 c + i)
      auto load_quarter = [&](KvQuarter& T, int t) {
        // (the step's first page always lies inside the chunk; a second page past its end is replaced by the first)
        const int pi = kv_page0 + 2 * t;
        const int pg = page_ids[(2 * t + my_page < n_pages) ? pi + my_page : pi];
        const uint8_t* k = kbase + pg * stride_page;
        const uint8_t* v = vbase + pg * stride_page;
        // plain loads: other CTAs of this kv head read the same rows and should find them in the XCD's L2
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          T.k[x] = *reinterpret_cast<const u32x4_t*>(k + 4 * (my_first + x) * stride_tok);
          T.v[x] = *reinterpret_cast<const u32x4_t*>(v + (my_first + x) * stride_tok);
        }
      };
      auto stage_and_compute = [&](KvQuarter& T, int t) {
        u32x4_t* buf = lds + (t & 1) * kBufEntries;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const int tk = 4 * (my_first + x) + c;
          buf[my_page * 256 + tk * 16 + ((m ^ tk) & 15)] = T.k[x];
          buf[kVOffset + (my_page * 4 + my_first + x) * 64 + lane] = T.v[x];
        }
        if (t + 3 < n_steps) load_quarter(T, t + 3);
        // One barrier per step: a wavefront that writes buffer t % 2 here has passed the barrier of step t - 1,
        // which every wavefront reaches only after its reads of step t - 2, the buffer's previous contents.
        __syncthreads();
        if (live_wave) {
          u32x4_t v[2][4];
#pragma unroll
          for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int i = 0; i < 4; ++i) v[pg][i] = buf[kVOffset + (pg * 4 + i) * 64 + lane];
          compute_step(buf, v, t);
        }
      };
      KvQuarter T0, T1, T2;
      if (n_steps > 0) load_quarter(T0, 0);
      if (n_steps > 1) load_quarter(T1, 1);
      if (n_steps > 2) load_quarter(T2, 2);
      for (int t = 0; t < n_steps; t += 3) {
        stage_and_compute(T0, t);
        if (t + 1 < n_steps) stage_and_compute(T1, t + 1);
        if (t + 2 < n_steps) stage_and_compute(T2, t + 2);
      }
    } else {
      // ---- every wavefront walks its own steps w, w + 4, ...; two of them in flight ----
      u32x4_t* mine = lds + wave * 512;
      auto load_step = [&](KvStep& T, int t) {
        const int pi = kv_page0 + 2 * t;
        const int pg0 = page_ids[pi];
        const int pg1 = (2 * t + 1 < n_pages) ? page_ids[pi + 1] : pg0;
        const uint8_t* k0 = kbase + pg0 * stride_page;
        const uint8_t* k1 = kbase + pg1 * stride_page;
        const uint8_t* v0 = vbase + pg0 * stride_page;
        const uint8_t* v1 = vbase + pg1 * stride_page;
        // read once: streams past the caches
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          T.k[0][s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(k0 + 4 * s * stride_tok));
          T.k[1][s] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(k1 + 4 * s * stride_tok));
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          T.v[0][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(v0 + i * stride_tok));
          T.v[1][i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(v1 + i * stride_tok));
        }
      };
      auto relayout_and_compute = [&](KvStep& T, int t) {
        // K rows -> this wavefront's LDS area (token 4 j + c, block m), back as A operands (token m, block 4 s + c)
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int tk = 4 * j + c;
            mine[pg * 256 + tk * 16 + ((m ^ tk) & 15)] = T.k[pg][j];
          }
        compute_step(mine, T.v, t);
      };
      const int n_mine = wave < n_steps ? (n_steps - wave + kWaves - 1) / kWaves : 0;
      {
        KvStep TA, TB;
        if (n_mine > 0) load_step(TA, wave);
        if (n_mine > 1) load_step(TB, wave + kWaves);
        for (int k = 0; k < n_mine; k += 2) {
          relayout_and_compute(TA, wave + kWaves * k);
          if (k + 2 < n_mine) load_step(TA, wave + kWaves * (k + 2));
          if (k + 1 < n_mine) {
            relayout_and_compute(TB, wave + kWaves * (k + 1));
            if (k + 3 < n_mine) load_step(TB, wave + kWaves * (k + 3));
          }
        }
      }
      // ---- wavefront 0 merges the four states (Sec. 2.2), in wavefront order ----
      l_run = sum_over_lane_groups(l_run);
      __syncthreads();  // the private K areas are free: the states go over them
      float* ml = reinterpret_cast<float*>(lds + kMlOffset);
      if (wave > 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) lds[(wave - 1) * kStateEntries + e * 64 + lane] = __builtin_bit_cast(u32x4_t, acc[e]);
        if (c == 0) {
          ml[(wave - 1) * 32 + 2 * m] = m_run;
          ml[(wave - 1) * 32 + 2 * m + 1] = l_run;
        }
      }
      __syncthreads();
      if (wave == 0) {
#pragma unroll
        for (int o = 0; o < kWaves - 1; ++o) {
          const float m_o = ml[o * 32 + 2 * m];
          const float l_o = ml[o * 32 + 2 * m + 1];
          const float m_new = fmaxf(m_run, m_o);
          const float m_ref = m_new == NEG_INF ? 0.f : m_new;  // both states empty: exp2(-inf) = 0, no NaN
          const float a = __builtin_amdgcn_exp2f(m_run - m_ref);
          const float b = __builtin_amdgcn_exp2f(m_o - m_ref);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const f32x4_t other = __builtin_bit_cast(f32x4_t, lds[o * kStateEntries + e * 64 + lane]);
            acc[e] = acc[e] * a + other * b;
          }
          l_run = l_run * a + l_o * b;
          m_run = m_new;
        }
      }
    }

    // ---- epilogue: o = O / l, lse = ln(sum exp) (Sec. 2.2); final rows (write-through, App. D.2) or the item's
    //      partial slot: partial row (slot * T_pos + position) * H + head ----
    if (wide ? live_wave : wave == 0) {
      float l = l_run;
      if (wide) {  // (light items: already summed over the lane groups, before the merge)
        l = sum_over_lane_groups(l);
      }
      const bool live = l > 0.f;
      const float inv = live ? 1.0f / l : 0.f;
      const float lse_val = live ? (m_run + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : NEG_INF;
      if (R < rows) {
        const int head = kvh * g + (R & (g - 1));
        const int64_t final_row = static_cast<int64_t>(q_row0 + pos) * H + head;
        const int64_t row = out_slot < 0 ? final_row : (static_cast<int64_t>(out_slot) * p.t_pos + pos) * H + head;
        float* dst_o = (out_slot < 0 ? p.o : p.part_o) + row * kHeadDim;
        float* dst_lse = (out_slot < 0 ? p.lse : p.part_lse) + row;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const f32x4_t lo = {acc[0][i] * inv, acc[1][i] * inv, acc[2][i] * inv, acc[3][i] * inv};
          const f32x4_t hi = {acc[4][i] * inv, acc[5][i] * inv, acc[6][i] * inv, acc[7][i] * inv};
          if (out_slot >= 0 || p.o != nullptr) {  // final rows may be wanted in the input type only
            *reinterpret_cast<f32x4_t*>(dst_o + 32 * c + 8 * i) = lo;
            *reinterpret_cast<f32x4_t*>(dst_o + 32 * c + 8 * i + 4) = hi;
          }
          if (out_slot < 0 && p.o_cast != nullptr) {
            uint16_t* dc = static_cast<uint16_t*>(p.o_cast) + final_row * kHeadDim + 32 * c + 8 * i;
            const u32x4_t pk = {pack2<BF>(lo[0], lo[1]), pack2<BF>(lo[2], lo[3]), pack2<BF>(hi[0], hi[1]), pack2<BF>(hi[2], hi[3])};
            *reinterpret_cast<u32x4_t*>(dc) = pk;
          }
        }
        if (c == 0) *dst_lse = lse_val;
      }
    }
    __syncthreads();  // the next work item reuses the LDS areas
  };
  for (int w = w_begin; w < w_end; ++w)
    if (as_const(p.w_n_pos)[w] * g > 16) work_item(std::true_type{}, w);
  for (int w = w_begin; w < w_end; ++w)
    if (as_const(p.w_n_pos)[w] * g <= 16) work_item(std::false_type{}, w);
}

}  // namespace

hipError_t launch_tiles64(const RunParams& p, bool is_bf16, hipStream_t stream) {
  const dim3 grid(static_cast<unsigned>(p.ctas_per_head) * static_cast<unsigned>(p.num_kv_heads), 1, 1);
  const dim3 block(64 * kWaves, 1, 1);
  if (is_bf16)
    hipLaunchKernelGGL((tile64_kernel<true>), grid, block, 0, stream, p);
  else
    hipLaunchKernelGGL((tile64_kernel<false>), grid, block, 0, stream, p);
  return hipGetLastError();
}

}  // namespace fi355
