// Paged append / prefill attention for gfx950 (causal or not): query tile = 128 fused rows
// (128/g consecutive positions x g query heads of one kv head, App. A), four wavefronts per
// CTA, each owning 32 rows.  K/V tiles of 64 tokens (four 16-token pages, gathered through
// kv_indices, Sec. 3.2.1) are staged in LDS and shared by the four wavefronts; both products
// run on the matrix cores:
//   S^T[token][row] = K . Q^T      v_mfma_f32_16x16x32   A = K rows from LDS, B = Q^T in registers
//   O^T[d][row]    += V^T . P^T    v_mfma_f32_16x16x32   A = V^T built by in-lane 16-bit permutes
//                                                        of row-major V rows read from LDS,
//                                                        B = P^T straight from the S^T accumulators
// Computing the transposed products puts one query row per lane column, so the online-softmax
// row maximum is an in-lane reduction plus two cross-lane exchanges, and P never moves
// between lanes.  The contraction index of the second product is (page, lane group,
// register) on both operands, so its order inside the instruction does not matter.
//
// P is rounded to fp16 (11 significant bits).  For bf16 inputs V is converted to fp16 while it
// is staged into LDS (exact for 2^-14 <= |v| <= 65504, saturating above, absolute error
// < 2^-24 below), because a bf16 P (8 bits) would miss the 2e-3 output tolerance on rows that
// see few keys; Q.K^T stays in the input type.
#include "kernels.h"

namespace fi355 {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

constexpr int kTileKv = 64;        // tokens per LDS tile
constexpr int kRowElems = 136;     // LDS row pitch in 16-bit elements: 128 + 8 pad (272 B) -> conflict-free b128 reads
constexpr int kCtaThreads = 256;

template <bool BF>
__device__ __forceinline__ f32x4_t mfma_qk(u32x4_t a, u32x4_t b, f32x4_t c) {
  if constexpr (BF) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                   c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c,
                                                  0, 0, 0);
  }
}
__device__ __forceinline__ f32x4_t mfma_pv(u32x4_t a, u32x4_t b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0,
                                                0, 0);
}

__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
  f16x2_t v = {static_cast<_Float16>(lo), static_cast<_Float16>(hi)};
  return __builtin_bit_cast(uint32_t, v);
}
template <bool BF>
__device__ __forceinline__ uint32_t pack_out(float lo, float hi) {
  if constexpr (BF) {
    bf16x2_t v = {static_cast<__bf16>(lo), static_cast<__bf16>(hi)};
    return __builtin_bit_cast(uint32_t, v);
  } else {
    return pack_f16(lo, hi);
  }
}
// two bf16 in one dword -> two fp16 in one dword (toward zero: a finite value never becomes inf)
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) {
  const float lo = __builtin_bit_cast(float, w << 16);
  const float hi = __builtin_bit_cast(float, w & 0xFFFF0000u);
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

__device__ __forceinline__ uint32_t lo_halves(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t hi_halves(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

template <bool BF>
__global__ void __launch_bounds__(kCtaThreads) append_kernel(const RunParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[kTileKv * kRowElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[kTileKv * kRowElems];

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int m = lane & 15;  // K: token in page; V: 16-byte column block; S/O: query row in block
  const int c = lane >> 4;  // lane group
  const int cta = blockIdx.x;
  const int kvh = blockIdx.y;
  const int g = p.group;
  const int g_log2 = 31 - __builtin_clz(g);
  const int H = p.num_qo_heads;
  const float NEG_INF = -__builtin_inff();

  // staging role: this thread moves the 16-byte block `st_chunk` of token slot `st_slot` of each of the 4 pages
  const int st_slot = tid >> 4;
  const int st_chunk = tid & 15;
  const int64_t st_off = kvh * p.stride_head + st_slot * p.stride_tok + st_chunk * 8;
  const uint16_t* kpool = static_cast<const uint16_t*>(p.k_pool);
  const uint16_t* vpool = static_cast<const uint16_t*>(p.v_pool);

  const int w_begin = __builtin_amdgcn_readfirstlane(p.cta_indptr[cta]);
  const int w_end = __builtin_amdgcn_readfirstlane(p.cta_indptr[cta + 1]);

  for (int w = w_begin; w < w_end; ++w) {
    const int q_row0 = __builtin_amdgcn_readfirstlane(p.w_q_row0[w]);
    const int n_pos = __builtin_amdgcn_readfirstlane(p.w_n_pos[w]);
    const int kv_page0 = __builtin_amdgcn_readfirstlane(p.w_kv_page0[w]);
    const int kv_start = __builtin_amdgcn_readfirstlane(p.w_kv_start[w]);
    const int kv_len = __builtin_amdgcn_readfirstlane(p.w_kv_len[w]);
    const int diag0 = __builtin_amdgcn_readfirstlane(p.w_diag0[w]);
    const int out_slot = __builtin_amdgcn_readfirstlane(p.w_out_slot[w]);
    const int n_pages = (kv_len + kPageSize - 1) / kPageSize;
    const int n_tiles = (kv_len + kTileKv - 1) / kTileKv;

    // ---- this lane's two query rows (one per 16-row block) ----
    int pos[2], hh[2], lim[2];
    bool row_ok[2];
    u32x4_t qreg[2][4];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int R = 32 * wave + 16 * nb + m;
      pos[nb] = R >> g_log2;
      hh[nb] = R & (g - 1);
      row_ok[nb] = pos[nb] < n_pos;
      // row sees request tokens <= diag0 + pos; in chunk-local terms: local index <= lim
      lim[nb] = (diag0 == kNoDiagMarker) ? 0x3FFFFFFF : diag0 + pos[nb] - kv_start;
      if (row_ok[nb]) {
        const uint16_t* qp = static_cast<const uint16_t*>(p.q) +
                             (static_cast<int64_t>(q_row0 + pos[nb]) * H + kvh * g + hh[nb]) * kHeadDim + c * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) qreg[nb][s] = *reinterpret_cast<const u32x4_t*>(qp + 32 * s);
      } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) qreg[nb][s] = u32x4_t{0u, 0u, 0u, 0u};
      }
    }
    // wave-uniform bounds of lim over the wave's 32 rows (rows are position-major)
    const int wave_pos_lo = (32 * wave) >> g_log2;
    const int wave_pos_hi = (32 * wave + 31) >> g_log2;
    const int wave_lim_lo = (diag0 == kNoDiagMarker) ? 0x3FFFFFFF : diag0 + wave_pos_lo - kv_start;
    const int wave_lim_hi = (diag0 == kNoDiagMarker) ? 0x3FFFFFFF : diag0 + wave_pos_hi - kv_start;

    f32x4_t acc[2][8];  // acc[nb][e][i] = O^T[d = 32 c + 8 i + e][row m of block nb]
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[nb][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run[2] = {NEG_INF, NEG_INF};
    float l_run[2] = {0.f, 0.f};

    u32x4_t stage_k[4], stage_v[4];
    auto fetch_tile = [&](int t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        int pi = 4 * t + r;
        pi = pi < n_pages ? pi : n_pages - 1;  // never index past the chunk's pages
        const int pg = __builtin_amdgcn_readfirstlane(p.kv_indices[kv_page0 + pi]);
        const int64_t off = pg * p.stride_page + st_off;
        stage_k[r] = *reinterpret_cast<const u32x4_t*>(kpool + off);
        stage_v[r] = *reinterpret_cast<const u32x4_t*>(vpool + off);
      }
    };
    auto store_tile = [&](int t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int tok = 16 * r + st_slot;
        u32x4_t v = stage_v[r];
        if constexpr (BF) {
          v = u32x4_t{bf16x2_to_f16x2(v[0]), bf16x2_to_f16x2(v[1]), bf16x2_to_f16x2(v[2]), bf16x2_to_f16x2(v[3])};
        }
        if (kTileKv * t + tok >= kv_len) v = u32x4_t{0u, 0u, 0u, 0u};  // rows past the chunk must not reach P.V
        *reinterpret_cast<u32x4_t*>(&lds_k[tok * kRowElems + st_chunk * 8]) = stage_k[r];
        *reinterpret_cast<u32x4_t*>(&lds_v[tok * kRowElems + st_chunk * 8]) = v;
      }
    };

    if (n_tiles > 0) fetch_tile(0);
    for (int t = 0; t < n_tiles; ++t) {
      __syncthreads();  // everyone is done reading the previous tile
      store_tile(t);
      __syncthreads();
      if (t + 1 < n_tiles) fetch_tile(t + 1);  // in flight while this tile is consumed

#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int tok_base = kTileKv * t + 32 * u;  // chunk-local index of this 32-token step
        if (tok_base >= kv_len || tok_base > wave_lim_hi) continue;  // nothing visible to this wavefront
        // ---- S^T = K . Q^T ----
        f32x4_t sacc[2][2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int pg = 0; pg < 2; ++pg) sacc[nb][pg] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
          const uint16_t* krow = &lds_k[(32 * u + 16 * pg + m) * kRowElems + c * 8];
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const u32x4_t ka = *reinterpret_cast<const u32x4_t*>(krow + 32 * s);
            sacc[0][pg] = mfma_qk<BF>(ka, qreg[0][s], sacc[0][pg]);
            sacc[1][pg] = mfma_qk<BF>(ka, qreg[1][s], sacc[1][pg]);
          }
        }
        // ---- online softmax, one row per (lane column, block) ----
        const bool need_mask = (tok_base + 32 > kv_len) || (tok_base + 31 > wave_lim_lo);
        u32x4_t pb[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          float sv[8];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            sv[i] = sacc[nb][0][i] * p.scale_log2;
            sv[4 + i] = sacc[nb][1][i] * p.scale_log2;
          }
          if (need_mask) {
            const int cap = min(lim[nb], kv_len - 1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int t0 = tok_base + 4 * c + i;
              sv[i] = (t0 <= cap) ? sv[i] : NEG_INF;
              sv[4 + i] = (t0 + 16 <= cap) ? sv[4 + i] : NEG_INF;
            }
          }
          float tmax =
              fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
          tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
          tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
          const float m_new = fmaxf(m_run[nb], tmax);
          const float m_use = (m_new == NEG_INF) ? 0.f : m_new;  // row has seen nothing yet
          const float alpha = __builtin_amdgcn_exp2f(m_run[nb] - m_use);
          m_run[nb] = m_new;
          float pv[8];
          float psum = 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            pv[j] = __builtin_amdgcn_exp2f(sv[j] - m_use);
            psum += pv[j];
          }
          l_run[nb] = l_run[nb] * alpha + psum;
          if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[nb][e] *= alpha;
          }
          pb[nb] = u32x4_t{pack_f16(pv[0], pv[1]), pack_f16(pv[2], pv[3]), pack_f16(pv[4], pv[5]),
                           pack_f16(pv[6], pv[7])};
        }
        // ---- O^T += V^T . P^T ----
        u32x4_t vr[2][4];
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            vr[pg][i] =
                *reinterpret_cast<const u32x4_t*>(&lds_v[(32 * u + 16 * pg + 4 * c + i) * kRowElems + m * 8]);
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
          const uint32_t a0 = vr[0][0][wd], a1 = vr[0][1][wd], a2 = vr[0][2][wd], a3 = vr[0][3][wd];
          const uint32_t b0 = vr[1][0][wd], b1 = vr[1][1][wd], b2 = vr[1][2][wd], b3 = vr[1][3][wd];
          const u32x4_t vt_even = {lo_halves(a0, a1), lo_halves(a2, a3), lo_halves(b0, b1), lo_halves(b2, b3)};
          const u32x4_t vt_odd = {hi_halves(a0, a1), hi_halves(a2, a3), hi_halves(b0, b1), hi_halves(b2, b3)};
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            acc[nb][2 * wd] = mfma_pv(vt_even, pb[nb], acc[nb][2 * wd]);
            acc[nb][2 * wd + 1] = mfma_pv(vt_odd, pb[nb], acc[nb][2 * wd + 1]);
          }
        }
      }
    }

    // ---- epilogue: o = O / l, lse = ln(sum exp) (Sec. 2.2) ----
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      float l = l_run[nb];
      l += __shfl_xor(l, 16);
      l += __shfl_xor(l, 32);
      const bool live = l > 0.f;
      const float inv = live ? 1.0f / l : 0.f;
      const float lse_val = live ? (m_run[nb] + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : NEG_INF;
      if (row_ok[nb]) {
        const int head = kvh * g + hh[nb];
        const int64_t final_row = static_cast<int64_t>(q_row0 + pos[nb]) * H + head;
        float* dst_o;
        float* dst_lse;
        if (out_slot < 0) {  // write-through (App. D.2)
          dst_o = p.o + final_row * kHeadDim;
          dst_lse = p.lse + final_row;
        } else {
          const int64_t row = (static_cast<int64_t>(out_slot) * p.t_pos + pos[nb]) * H + head;
          dst_o = p.part_o + row * kHeadDim;
          dst_lse = p.part_lse + row;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float* d = dst_o + 32 * c + 8 * i;
          const f32x4_t lo = {acc[nb][0][i] * inv, acc[nb][1][i] * inv, acc[nb][2][i] * inv, acc[nb][3][i] * inv};
          const f32x4_t hi = {acc[nb][4][i] * inv, acc[nb][5][i] * inv, acc[nb][6][i] * inv, acc[nb][7][i] * inv};
          *reinterpret_cast<f32x4_t*>(d) = lo;
          *reinterpret_cast<f32x4_t*>(d + 4) = hi;
          if (out_slot < 0 && p.o_cast != nullptr) {
            uint16_t* dc = static_cast<uint16_t*>(p.o_cast) + final_row * kHeadDim + 32 * c + 8 * i;
            const u32x4_t pk = {pack_out<BF>(lo[0], lo[1]), pack_out<BF>(lo[2], lo[3]), pack_out<BF>(hi[0], hi[1]),
                                pack_out<BF>(hi[2], hi[3])};
            *reinterpret_cast<u32x4_t*>(dc) = pk;
          }
        }
        if (c == 0) *dst_lse = lse_val;
      }
    }
  }
}

}  // namespace

hipError_t launch_append(const RunParams& p, bool is_bf16, hipStream_t stream) {
  const dim3 grid(static_cast<unsigned>(p.ctas_per_head), static_cast<unsigned>(p.num_kv_heads), 1);
  const dim3 block(kCtaThreads, 1, 1);
  if (is_bf16)
    hipLaunchKernelGGL(append_kernel<true>, grid, block, 0, stream, p);
  else
    hipLaunchKernelGGL(append_kernel<false>, grid, block, 0, stream, p);
  return hipGetLastError();
}

}  // namespace fi355
