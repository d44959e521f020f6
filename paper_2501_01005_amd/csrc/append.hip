// Paged append / prefill attention for gfx950 (causal or not): query tile = 128 fused rows
// (128/g consecutive positions x g query heads of one kv head, App. A), four wavefronts per
// CTA, each owning 32 rows.  K/V tiles of 64 tokens (four 16-token pages, gathered through
// kv_indices, Sec. 3.2.1) are staged in LDS and shared by the four wavefronts; both products
// run on the matrix cores:
//   S^T[token][row] = K . Q^T      v_mfma_f32_16x16x32   A = K rows from LDS, B = Q^T in registers
//   O^T[d][row]    += V^T . P^T    v_mfma_f32_16x16x32   A = V^T read from the row-major V tile with
//                                                        the LDS transpose read ds_read_b64_tr_b16,
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
constexpr int kRowElems = 136;     // K tile row pitch in 16-bit elements (272 B): rows 4 banks apart, conflict-free b128 reads
constexpr int kRowElemsV = 144;    // V tile row pitch (288 B): rows 8 banks apart, conflict-free transpose reads
constexpr int kCtaThreads = 256;
constexpr float kLazyLog2 = 8.0f;  // P may exceed 1 by at most 2^8 before the running reference is raised

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

typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
// ds_read_b64_tr_b16: within each group of 16 lanes, lane 4 k + q supplies the address of 4
// consecutive 16-bit elements; lane l of the group receives, in slot k = 0..3, element l % 4 of
// the row supplied by lane 4 k + l / 4.  With lane 4 k + q pointing at row k, columns
// c0 + 4 q .. + 3, lane l ends up with column c0 + l of rows 0..3: a 4 x 16 block transposed.
__device__ __forceinline__ u32x2_t lds_read_tr16(const uint16_t* p) {
  const s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4_t*)(const_cast<uint16_t*>(p)));
  return __builtin_bit_cast(u32x2_t, v);
}

// Exchanges between the four 16-lane rows of a wavefront without going through LDS:
// v_permlane32_swap swaps the upper half of its first operand with the lower half of its
// second, v_permlane16_swap swaps the odd rows of the first with the even rows of the second.
// With both operands holding x, the pair afterwards holds (x of lane l, x of lane l ^ 32)
// resp. (x of lane l, x of lane l ^ 16) in some order, which is all a max or a sum needs.
__device__ __forceinline__ void swap32(float x, float* a, float* b) {
  uint32_t u = __builtin_bit_cast(uint32_t, x), v = u;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32_e32 %0, %1" : "+v"(u), "+v"(v));
  *a = __builtin_bit_cast(float, u);
  *b = __builtin_bit_cast(float, v);
}
__device__ __forceinline__ void swap16(float x, float* a, float* b) {
  uint32_t u = __builtin_bit_cast(uint32_t, x), v = u;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32_e32 %0, %1" : "+v"(u), "+v"(v));
  *a = __builtin_bit_cast(float, u);
  *b = __builtin_bit_cast(float, v);
}
__device__ __forceinline__ float rows_max(float x) {
  float a, b;
  swap32(x, &a, &b);
  x = fmaxf(a, b);
  swap16(x, &a, &b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float rows_sum(float x) {
  float a, b;
  swap32(x, &a, &b);
  x = a + b;
  swap16(x, &a, &b);
  return a + b;
}

template <bool BF>
__global__ void __launch_bounds__(kCtaThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
append_kernel(const RunParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[kTileKv * kRowElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[kTileKv * kRowElemsV];

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
  const float lazy_raw = kLazyLog2 / p.scale_log2;  // kLazyLog2 binary orders of magnitude in raw-logit units

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

    f32x4_t acc[2][8];  // acc[nb][e][i] = O^T[d = 16 e + 4 c + i][row m of block nb]
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[nb][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run[2] = {NEG_INF, NEG_INF};  // reference for the exponentials: raw-logit units, >= row max - lazy_raw
    float l_run[2] = {0.f, 0.f};

    u32x4_t stage_k[4], stage_v[4];
    // Page ids are fetched one tile ahead of the data they address (lane r holds page r of the
    // tile), so that the data loads never wait behind an index load.
    auto fetch_page_ids = [&](int t) -> int {
      int pi = 4 * t + (lane & 3);
      pi = pi < n_pages ? pi : n_pages - 1;  // never index past the chunk's pages
      return p.kv_indices[kv_page0 + pi];
    };
    auto fetch_tile = [&](int ids) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int pg = __builtin_amdgcn_readlane(ids, r);
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
        *reinterpret_cast<u32x4_t*>(&lds_v[tok * kRowElemsV + st_chunk * 8]) = v;
      }
    };

    int ids_next = 0;
    if (n_tiles > 0) {
      fetch_tile(fetch_page_ids(0));
      if (n_tiles > 1) ids_next = fetch_page_ids(1);
    }
    for (int t = 0; t < n_tiles; ++t) {
      __syncthreads();  // everyone is done reading the previous tile
      store_tile(t);
      __syncthreads();
      if (t + 1 < n_tiles) {
        fetch_tile(ids_next);  // in flight while this tile is consumed
        if (t + 2 < n_tiles) ids_next = fetch_page_ids(t + 2);
      }

#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int tok_base = kTileKv * t + 32 * u;  // chunk-local index of this 32-token step
        if (tok_base >= kv_len || tok_base > wave_lim_hi) continue;  // nothing visible to this wavefront
        // ---- S^T = K . Q^T: all eight A operands are requested before the first product ----
        u32x4_t ka[2][4];
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
          const uint16_t* krow = &lds_k[(32 * u + 16 * pg + m) * kRowElems + c * 8];
#pragma unroll
          for (int s = 0; s < 4; ++s) ka[pg][s] = *reinterpret_cast<const u32x4_t*>(krow + 32 * s);
        }
        f32x4_t sacc[2][2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int pg = 0; pg < 2; ++pg) sacc[nb][pg] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int pg = 0; pg < 2; ++pg) {
            sacc[0][pg] = mfma_qk<BF>(ka[pg][s], qreg[0][s], sacc[0][pg]);
            sacc[1][pg] = mfma_qk<BF>(ka[pg][s], qreg[1][s], sacc[1][pg]);
          }
        // ---- V^T operands (16 columns d = 16 e + m of tokens (page, 4 c + k)): requested now,
        //      they arrive while the softmax below runs on the vector ALU ----
        u32x4_t vt[8];
        {
          const int k4 = m >> 2, q4 = m & 3;  // this lane's role as address supplier in its 16-lane group
          const uint16_t* vsrc = &lds_v[(32 * u + 4 * c + k4) * kRowElemsV + 4 * q4];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const u32x2_t lo = lds_read_tr16(vsrc + 16 * e);                    // page 0 of the step
            const u32x2_t hi = lds_read_tr16(vsrc + 16 * kRowElemsV + 16 * e);  // page 1
            vt[e] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
          }
        }
        // ---- online softmax, one row per (lane column, block) ----
        const bool need_mask = (tok_base + 32 > kv_len) || (tok_base + 31 > wave_lim_lo);
        u32x4_t pb[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          float sv[8];  // raw logits q.k; the softmax scale is folded into the exponent below
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            sv[i] = sacc[nb][0][i];
            sv[4 + i] = sacc[nb][1][i];
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
          float tmax = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
          tmax = rows_max(tmax);
          // Lazy reference update: the reference m_run only has to bound the logits from above
          // up to 2^kLazyLog2 (P then stays <= 2^kLazyLog2, well inside fp16 and fp32 range); the
          // result o = O / l does not depend on it.  Rescaling the 32 accumulator registers is
          // thus needed only when the row maximum jumps, not on every small increase.
          if (__builtin_amdgcn_ballot_w64(tmax > m_run[nb] + lazy_raw) != 0) {
            const float m_new = fmaxf(m_run[nb], tmax);
            const float m_use = (m_new == NEG_INF) ? 0.f : m_new;  // row has seen nothing yet
            const float alpha = __builtin_amdgcn_exp2f((m_run[nb] - m_use) * p.scale_log2);
            m_run[nb] = m_new;
            l_run[nb] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[nb][e] *= alpha;
          }
          const float neg_ms = (m_run[nb] == NEG_INF) ? 0.f : -m_run[nb] * p.scale_log2;
          float pv[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) pv[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[j], p.scale_log2, neg_ms));
          const f16x2_t h0 = {static_cast<_Float16>(pv[0]), static_cast<_Float16>(pv[1])};
          const f16x2_t h1 = {static_cast<_Float16>(pv[2]), static_cast<_Float16>(pv[3])};
          const f16x2_t h2 = {static_cast<_Float16>(pv[4]), static_cast<_Float16>(pv[5])};
          const f16x2_t h3 = {static_cast<_Float16>(pv[6]), static_cast<_Float16>(pv[7])};
          pb[nb] = u32x4_t{__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1),
                           __builtin_bit_cast(uint32_t, h2), __builtin_bit_cast(uint32_t, h3)};
          // The row sum is taken over the fp16-rounded P that the second product consumes
          // (v_dot2_f32_f16 with a vector of ones, fp32 accumulation): o = O / l is then an exact
          // convex combination of V rows whatever the reference, and a single dominant key
          // returns its V row exactly.
          const f16x2_t ones = {static_cast<_Float16>(1.0f), static_cast<_Float16>(1.0f)};
          float l = l_run[nb];
          l = __builtin_amdgcn_fdot2(h0, ones, l, false);
          l = __builtin_amdgcn_fdot2(h1, ones, l, false);
          l = __builtin_amdgcn_fdot2(h2, ones, l, false);
          l = __builtin_amdgcn_fdot2(h3, ones, l, false);
          l_run[nb] = l;
        }
        // ---- O^T += V^T . P^T ----
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          acc[0][e] = mfma_pv(vt[e], pb[0], acc[0][e]);
          acc[1][e] = mfma_pv(vt[e], pb[1], acc[1][e]);
        }
      }
    }

    // ---- epilogue: o = O / l, lse = ln(sum exp) (Sec. 2.2) ----
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const float l = rows_sum(l_run[nb]);
      const bool live = l > 0.f;
      const float inv = live ? 1.0f / l : 0.f;
      const float lse_val =
          live ? (m_run[nb] * p.scale_log2 + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : NEG_INF;
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
        for (int e = 0; e < 8; ++e) {
          const f32x4_t v = acc[nb][e] * inv;
          *reinterpret_cast<f32x4_t*>(dst_o + 16 * e + 4 * c) = v;
          if (out_slot < 0 && p.o_cast != nullptr) {
            uint16_t* dc = static_cast<uint16_t*>(p.o_cast) + final_row * kHeadDim + 16 * e + 4 * c;
            *reinterpret_cast<u32x2_t*>(dc) = u32x2_t{pack_out<BF>(v[0], v[1]), pack_out<BF>(v[2], v[3])};
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
