// Small query tiles (Sec. 3.2.2) for gfx950: a query tile holds up to NB x 16 fused rows (row R = position * g +
// head, App. A) of one request, one wavefront per CTA.  Short appends (causal or not, e.g. the draft tokens of
// speculative decoding), decode steps, and the row blocks of a shared prefix in composed formats (Sec. 3.1.2) run
// as work items of ONE launch: a decode item is a tile of one position, a shared-prefix item a tile of NB x 16 / g.
//
// The products are those of the decode kernel (decode.hip): per 32-token step of a work item
//   S^T[token][row] = K . Q^T      v_mfma_f32_16x16x32, A = K rows (through a wavefront-private LDS buffer), B = Q^T
//   O^T[d][row]    += V^T . P^T    A = V^T built in-lane from row-major V rows, B = P^T from the S^T accumulators
// once per block of 16 rows, with every column of the matrix tile live when the tile is full.  The K/V rows of a
// step are loaded once per wavefront whatever NB is.  Only NB = 1 is instantiated: measured on the shared-prefix
// workload (64 queries x 4 096 keys + 64 suffixes), NB = 1 at two wavefronts per SIMD takes 32 us, NB = 2 at one
// wavefront per SIMD 35 us, NB = 4 (which needs more than the 512 registers of a lone wavefront and spills) 71 us:
// the re-reads of the prefix hit in the XCD's L2 and are not what bounds the launch (the 64-row tile kernel cuts
// them fourfold and gains 10 %).  Neither is the count of vector instructions (about 255 per 32-token step): a build
// with the K/V address arithmetic moved to scalar registers (buffer loads off per-page descriptors) ran 2.8 us
// slower, one with the softmax scale folded into the exponent's multiply-add 0.7 us slower.  A step is a chain of
// dependent phases (K through LDS, product, softmax, product) of one in-order wavefront, and with 239 registers
// only two wavefronts share a SIMD to overlap it.
// bf16: P enters the second product as head + remainder (see decode.hip).
//
// Causal items mask per row: row R sees chunk tokens <= diag0 - kv_start + position(R).  A row that has seen no
// key yet keeps the empty state (m = -inf, l = 0).
//
// The grid is one-dimensional with the kv head as the fast index: workgroups go to the eight XCDs round-robin, so
// the CTAs of a kv head, which re-read a shared prefix once per query tile, share one XCD's L2.
#include "kernels.h"

namespace fi355 {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

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

struct KvStep {
  u32x4_t k[2][4];  // [page][j]: K[token 4 j + c][d = 8 m .. +8]   (as loaded: a lane group loads whole 256-byte rows)
  u32x4_t v[2][4];  // [page][i]: V[token 4 c + i][d = 8 m .. +8]
};

template <bool BF, int NB>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(NB > 1 ? 1 : 2, NB > 1 ? 1 : 2)))
tile_kernel(const RunParams p) {
  const int lane = threadIdx.x;
  const int m = lane & 15;  // K: token in page; V: 16-byte column block; S/O: row within a block of 16 fused rows
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
  // K relayout buffer: block (page pg, token t, 16-byte block x) lives at pg*4096 + t*256 + ((x ^ t) & 15)*16
  __shared__ __attribute__((aligned(16))) u32x4_t k_lds[2 * 16 * 16];

  // plan arrays and page ids through the constant address space: wavefront-uniform scalar loads
  using ConstInts = const __attribute__((address_space(4))) int32_t*;
  auto as_const = [](const int32_t* ptr) { return (ConstInts)(reinterpret_cast<uintptr_t>(ptr)); };
  ConstInts cta_indptr = as_const(p.cta_indptr), page_ids = as_const(p.kv_indices);
  const int w_begin = cta_indptr[cta];
  const int w_end = cta_indptr[cta + 1];

  for (int w = w_begin; w < w_end; ++w) {
    const int q_row0 = as_const(p.w_q_row0)[w];
    const int kv_page0 = as_const(p.w_kv_page0)[w];
    const int kv_len = as_const(p.w_kv_len)[w];
    const int out_slot = as_const(p.w_out_slot)[w];
    const int diag0 = as_const(p.w_diag0)[w];
    const int rows = as_const(p.w_n_pos)[w] * g;  // live fused rows of the tile
    const int nb_live = (rows + 15) >> 4;        // blocks of 16 rows with a live row
    const bool shared_kv = rows > g;             // other query tiles of the request read the same K/V
    // causal items: chunk-local index of the last token the tile's first position sees (all tokens otherwise)
    const int lim_first = diag0 != kNoDiagMarker ? diag0 - as_const(p.w_kv_start)[w] : 0x3FFFFFFF;
    const int n_pages = (kv_len + 15) >> 4;
    const int n_steps = (kv_len + 31) >> 5;

    // per block of 16 rows: this lane's row R = 16 b + m -> (position, head); Q^T as the B operand of the first
    // product: lane (m, c) holds row R, d = 32 s + 8 c .. +8
    int pos[NB], lim[NB];
    u32x4_t qreg[NB][4];
    f32x4_t acc[NB][8];  // acc[b][e][i] = O^T[d = 32 c + 8 i + e][row 16 b + m]
    float m_run[NB];     // running max of the scaled logits, log2 units (same in all 4 lane groups)
    float l_run[NB];     // this lane's share of the running sum
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int R = 16 * b + m;
      pos[b] = R >> g_log2;
      lim[b] = lim_first == 0x3FFFFFFF ? lim_first : lim_first + pos[b];
      if (R < rows) {
        const uint16_t* qp = static_cast<const uint16_t*>(p.q) +
                             (static_cast<int64_t>(q_row0 + pos[b]) * H + kvh * g + (R & (g - 1))) * kHeadDim + c * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) qreg[b][s] = *reinterpret_cast<const u32x4_t*>(qp + 32 * s);
      } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) qreg[b][s] = u32x4_t{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[b][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      m_run[b] = NEG_INF;
      l_run[b] = 0.f;
    }

    auto load_step = [&](KvStep& T, int t) {
      const int pi = kv_page0 + 2 * t;
      const int pg0 = page_ids[pi];
      const int pg1 = (2 * t + 1 < n_pages) ? page_ids[pi + 1] : pg0;
      const uint8_t* k0 = kbase + pg0 * stride_page;
      const uint8_t* k1 = kbase + pg1 * stride_page;
      const uint8_t* v0 = vbase + pg0 * stride_page;
      const uint8_t* v1 = vbase + pg1 * stride_page;
      // K/V that other query tiles read again (a shared prefix) should stay in the XCD's L2: plain loads; K/V read
      // once (a decode item) streams past the caches
      if (shared_kv) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          T.k[0][s] = *reinterpret_cast<const u32x4_t*>(k0 + 4 * s * stride_tok);
          T.k[1][s] = *reinterpret_cast<const u32x4_t*>(k1 + 4 * s * stride_tok);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          T.v[0][i] = *reinterpret_cast<const u32x4_t*>(v0 + i * stride_tok);
          T.v[1][i] = *reinterpret_cast<const u32x4_t*>(v1 + i * stride_tok);
        }
      } else {
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
      }
    };

    auto compute_step = [&](KvStep& T, int t) {
      // ---- S^T = K . Q^T: K rows -> LDS (token 4 j + c, block m), back as A operands (token m, block 4 s + c) ----
#pragma unroll
      for (int pg = 0; pg < 2; ++pg)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int tk = 4 * j + c;
          k_lds[pg * 256 + tk * 16 + ((m ^ tk) & 15)] = T.k[pg][j];
        }
      f32x4_t s0[NB], s1[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b) s0[b] = s1[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const u32x4_t ka0 = k_lds[m * 16 + (((4 * s + c) ^ m) & 15)];
        const u32x4_t ka1 = k_lds[256 + m * 16 + (((4 * s + c) ^ m) & 15)];
#pragma unroll
        for (int b = 0; b < NB; ++b)
          if (b < nb_live) {
            s0[b] = mfma<BF>(ka0, qreg[b][s], s0[b]);
            s1[b] = mfma<BF>(ka1, qreg[b][s], s1[b]);
          }
      }
      // lane (m, c) now holds S^T[token 16 pg + 4 c + i][row 16 b + m]
      const int tok0 = 32 * t + 4 * c;
      const bool tail = 32 * t + 32 > kv_len;  // ragged end of the chunk
      if (tail) {  // V rows past the chunk must not reach the second product (0 x garbage need not be 0)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (tok0 + i >= kv_len) T.v[0][i] = u32x4_t{0u, 0u, 0u, 0u};
          if (tok0 + 16 + i >= kv_len) T.v[1][i] = u32x4_t{0u, 0u, 0u, 0u};
        }
      }
      // vt[e][pg * 2 + pr] = column e of tokens (2 pr, 2 pr + 1) of page pg, as a pair of 16-bit values
      u32x4_t vt[8];
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        const uint32_t a0 = T.v[0][0][wd], a1 = T.v[0][1][wd], a2 = T.v[0][2][wd], a3 = T.v[0][3][wd];
        const uint32_t b0 = T.v[1][0][wd], b1 = T.v[1][1][wd], b2 = T.v[1][2][wd], b3 = T.v[1][3][wd];
        vt[2 * wd] = u32x4_t{lo_halves(a0, a1), lo_halves(a2, a3), lo_halves(b0, b1), lo_halves(b2, b3)};
        vt[2 * wd + 1] = u32x4_t{hi_halves(a0, a1), hi_halves(a2, a3), hi_halves(b0, b1), hi_halves(b2, b3)};
      }
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        if (b >= nb_live) continue;  // wavefront-uniform
        float sv[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          sv[i] = s0[b][i] * p.scale_log2;
          sv[4 + i] = s1[b][i] * p.scale_log2;
        }
        if (32 * t + 31 > lim_first || tail) {  // the causal diagonal or the end of the chunk cuts this step
          const int last = min(lim[b], kv_len - 1);
#pragma unroll
          for (int j = 0; j < 8; ++j) sv[j] = (tok0 + 16 * (j >> 2) + (j & 3) <= last) ? sv[j] : NEG_INF;
        }
        // ---- online softmax (Sec. 2.1) ----
        float tmax = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run[b], tmax);
        const bool none_yet = m_new == NEG_INF;  // the row has not seen a key so far
        const float alpha = none_yet ? 1.0f : __builtin_amdgcn_exp2f(m_run[b] - m_new);
        m_run[b] = m_new;
        float pv[8];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          pv[j] = none_yet ? 0.f : __builtin_amdgcn_exp2f(sv[j] - m_new);
          psum += pv[j];
        }
        l_run[b] = l_run[b] * alpha + psum;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[b][e] *= alpha;
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
          acc[b][e] = mfma<BF>(vt[e], pb, acc[b][e]);
          if constexpr (BF) acc[b][e] = mfma<BF>(vt[e], pb_lo, acc[b][e]);
        }
        // one block after the other: interleaving the softmax of several blocks would multiply the temporaries
        if constexpr (NB > 1) __builtin_amdgcn_sched_barrier(0);
      }
    };

    {
      KvStep TA, TB;  // two steps in flight
      if (n_steps > 0) load_step(TA, 0);
      if (n_steps > 1) load_step(TB, 1);
      for (int t = 0; t < n_steps; t += 2) {
        compute_step(TA, t);
        if (t + 2 < n_steps) load_step(TA, t + 2);
        if (t + 1 < n_steps) {
          compute_step(TB, t + 1);
          if (t + 3 < n_steps) load_step(TB, t + 3);
        }
      }
    }

    // ---- epilogue: o = O / l, lse = ln(sum exp) (Sec. 2.2); final rows (write-through, App. D.2) or the item's
    //      partial slot: partial row (slot * T_pos + position) * H + head ----
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      if (b >= nb_live) continue;
      float l = l_run[b];
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
      const bool live = l > 0.f;
      const float inv = live ? 1.0f / l : 0.f;
      const float lse_val = live ? (m_run[b] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : NEG_INF;
      const int R = 16 * b + m;
      if (R < rows) {
        const int head = kvh * g + (R & (g - 1));
        const int64_t final_row = static_cast<int64_t>(q_row0 + pos[b]) * H + head;
        const int64_t row = out_slot < 0 ? final_row : (static_cast<int64_t>(out_slot) * p.t_pos + pos[b]) * H + head;
        float* dst_o = (out_slot < 0 ? p.o : p.part_o) + row * kHeadDim;
        float* dst_lse = (out_slot < 0 ? p.lse : p.part_lse) + row;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const f32x4_t lo = {acc[b][0][i] * inv, acc[b][1][i] * inv, acc[b][2][i] * inv, acc[b][3][i] * inv};
          const f32x4_t hi = {acc[b][4][i] * inv, acc[b][5][i] * inv, acc[b][6][i] * inv, acc[b][7][i] * inv};
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
  }
}

}  // namespace

hipError_t launch_tiles(const RunParams& p, bool is_bf16, hipStream_t stream) {
  const dim3 grid(static_cast<unsigned>(p.ctas_per_head) * static_cast<unsigned>(p.num_kv_heads), 1, 1);
  const dim3 block(64, 1, 1);
  if (is_bf16)
    hipLaunchKernelGGL((tile_kernel<true, 1>), grid, block, 0, stream, p);
  else
    hipLaunchKernelGGL((tile_kernel<false, 1>), grid, block, 0, stream, p);
  return hipGetLastError();
}

}  // namespace fi355
