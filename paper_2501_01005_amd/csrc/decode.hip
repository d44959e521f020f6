// Paged decode attention for gfx950: query tile = one position x g fused query heads
// (head-group fusion, App. A), one wavefront per CTA, K/V streamed from HBM with whole-row
// coalesced non-temporal loads.  HBM-bandwidth bound: every K/V byte of a chunk is read once.
// V rows are consumed from registers as loaded; K rows pass through a wavefront-private 8 KB
// LDS buffer (XOR-swizzled 16-byte blocks, conflict-free both ways) to reach the A-operand
// layout of the first product, because loading that layout directly (16 rows x 64 B per
// instruction) halves the request size and loses the benefit of streaming loads.
//
// Per 32-token step (two 16-token pages) of a work item:
//   S^T[token][head] = K . Q^T         v_mfma_f32_16x16x32 (A = K page, B = Q^T padded to 16 heads)
//   online softmax (Sec. 2.1) on the 4 x 2 logits a lane owns, row max across the
//   four 16-lane groups by two cross-lane exchanges
//   O^T[d][head]    += V^T . P^T       v_mfma_f32_16x16x32 (A = V^T built by in-lane 16-bit
//                                      permutes of row-major V rows, B = P^T straight from
//                                      the S^T accumulator layout -- no cross-lane traffic)
// The contraction index of the second product is (page, lane group, register), which both
// operands enumerate identically, so its order inside the instruction never matters.
//
// bf16 inputs: P is split into a bf16 head and a bf16 remainder and the second product is
// issued twice; the matrix pipe has an order of magnitude of slack on this path and it keeps
// P to ~16 significant bits without restricting the range of V.
//
// 8-bit KV cache (App. F: fp8 K/V, 16-bit queries, wider arithmetic): the pools hold OCP E4M3
// codes; a lane loads the same (token, 8 columns) piece as above in 8 bytes instead of 16 and
// widens it to the query type (exact: E4M3 is a subset of both) when the tile is consumed, so
// everything after the load is shared; for V the codes of a token pair are interleaved
// byte-wise first, so that the conversion instruction delivers the pair the V^T operand needs.
// Four tiles are in flight instead of two, which keeps the bytes in flight per wavefront.  The
// K and V scales are folded into the softmax scale and into the final normalisation.
#include <type_traits>

#include "kernels.h"

namespace fi355 {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

template <bool BF>
__device__ __forceinline__ f32x4_t mfma_16x16x32(u32x4_t a, u32x4_t b, f32x4_t c) {
  if constexpr (BF) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                   c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c,
                                                  0, 0, 0);
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

__device__ __forceinline__ u32x4_t ld16(const uint16_t* p) { return *reinterpret_cast<const u32x4_t*>(p); }
// K/V bytes are used exactly once: streaming (non-temporal) loads keep them from displacing
// each other in the caches and measure ~13 % faster than plain loads on a pure read stream.
__device__ __forceinline__ u32x4_t ld16_stream(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
}

__device__ __forceinline__ u32x2_t ld8_stream(const uint8_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
}

// eight E4M3 codes (byte i = column i) -> eight values of the query type, column i in 16-bit slot i
// (one conversion instruction per pair: the scaled fp8 conversions of gfx950 with scale 1)
template <bool BF>
__device__ __forceinline__ u32x4_t widen8(u32x2_t w) {
  if constexpr (BF) {
    return u32x4_t{__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[0], 1.0f, false)),
                   __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[0], 1.0f, true)),
                   __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[1], 1.0f, false)),
                   __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[1], 1.0f, true))};
  } else {
    return u32x4_t{__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[0], 1.0f, false)),
                   __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[0], 1.0f, true)),
                   __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[1], 1.0f, false)),
                   __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w[1], 1.0f, true))};
  }
}

template <bool KV8>
struct KvTile {
  using Piece = typename std::conditional<KV8, u32x2_t, u32x4_t>::type;  // 8 columns as stored
  Piece k[2][4];  // [page][j]:        K[token 4 j + c][d = 8 m .. +8]   (as loaded, row-coalesced)
  Piece v[2][4];  // [page][i]:        V[token 4 c + i][d = 8 m .. +8]
};

// ANYPS: the page size is a run-time power of two instead of 16 (Sec. 3.1.1: the block size B_c of the
// BSR cache is a free parameter); every lane then looks up the page of each token row it loads.
// VAR: attention variants (Sec. 3.2.3, logits transform and logits mask) on the scaled logits, in this order:
// soft cap c * tanh(s / c), ALiBi bias slope[head] * (t - pos), sliding window (tokens t < pos - window hidden);
// pos = l_kv - 1 is the absolute position of the request's query.  A step may then hold no visible token; steps
// wholly before the window are skipped without being read.
// ROPE (with VAR): rotary position embedding as query and key transform (Sec. 3.2.3; the fused-RoPE kernels of
// Sec. 4.3): key t of a request is rotated by its position t, the query by pos, pairing components (d, d + 64).
// The rotated values are formed in fp32 from the K operands as they come back from LDS (a lane holds both
// components of a pair there).  They enter the first product as a head and a remainder in the input type, as P
// does in the second (three instructions per operand pair: head x head, remainder x head, head x remainder): a
// rotated value rounded once costs 2^-9 (bf16) or 2^-12 (fp16) of relative accuracy per operand, which on peaked
// distributions over large values reaches the comparison bound (measured 2.2e-3 on o with fp16 operands, V ~ 2 N(0,1),
// ALiBi and a soft cap; 3e-6 with the remainder).
struct NoRope {};
template <bool ROPE>
using RopeArg = typename std::conditional<ROPE, RopeTable, NoRope>::type;

template <bool BF>
__device__ __forceinline__ float elem16(uint32_t word, int odd) {
  if constexpr (BF) {
    return __builtin_bit_cast(float, odd ? (word & 0xffff0000u) : (word << 16));
  } else {
    const f16x2_t h = __builtin_bit_cast(f16x2_t, word);
    return static_cast<float>(odd ? h[1] : h[0]);
  }
}

// (x, y) = the lane's eight components of the blocks d and d + 64 of one row; cs / sn = cosine / sine of the
// row's angle for each of the eight pairs.  Rotated values -> MFMA operands: head and remainder.
template <bool BF>
__device__ __forceinline__ void rotate_blocks(const u32x4_t x, const u32x4_t y, const float* cs, const float* sn,
                                              u32x4_t* xh, u32x4_t* yh, u32x4_t* xl, u32x4_t* yl) {
  float xr[8], yr[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float xe = elem16<BF>(x[e >> 1], e & 1), ye = elem16<BF>(y[e >> 1], e & 1);
    xr[e] = xe * cs[e] - ye * sn[e];
    yr[e] = ye * cs[e] + xe * sn[e];
  }
  *xh = u32x4_t{pack2<BF>(xr[0], xr[1]), pack2<BF>(xr[2], xr[3]), pack2<BF>(xr[4], xr[5]), pack2<BF>(xr[6], xr[7])};
  *yh = u32x4_t{pack2<BF>(yr[0], yr[1]), pack2<BF>(yr[2], yr[3]), pack2<BF>(yr[4], yr[5]), pack2<BF>(yr[6], yr[7])};
  // remainder = value - head (the head's value read back from its 16 bits)
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    xr[e] -= elem16<BF>((*xh)[e >> 1], e & 1);
    yr[e] -= elem16<BF>((*yh)[e >> 1], e & 1);
  }
  *xl = u32x4_t{pack2<BF>(xr[0], xr[1]), pack2<BF>(xr[2], xr[3]), pack2<BF>(xr[4], xr[5]), pack2<BF>(xr[6], xr[7])};
  *yl = u32x4_t{pack2<BF>(yr[0], yr[1]), pack2<BF>(yr[2], yr[3]), pack2<BF>(yr[4], yr[5]), pack2<BF>(yr[6], yr[7])};
}

// (The rotary variant and the any-page-size variants run one wavefront per SIMD with up to 512 registers: at two
// they spill 70-180 registers into scratch memory inside the tile loop; the rotary kernel then takes 1.7 times as
// long, the any-page-size kernels 3-7 % longer.)
// CONTIG: contiguous KV (App. B's dense baseline; Sec. 3.1.1 with the identity as page table): page j of a request is
// page kv_page0 + j of the pool, so that rows are addressed affinely and no page id is ever loaded.  With page size
// 1 and the [pages, slots, heads, D] layout the pool is the ragged tensor [tokens, H_kv, D].
template <bool BF, bool KV8, bool ANYPS, bool VAR = false, bool ROPE = false, bool CONTIG = false>
__global__ void __launch_bounds__(64)
    __attribute__((amdgpu_waves_per_eu((ROPE || ANYPS) ? 1 : 2, (ROPE || ANYPS) ? 1 : 2)))
decode_kernel(const RunParams p, const RopeArg<ROPE> rope) {
  static_assert(!ROPE || (VAR && !KV8 && !ANYPS), "the rotary transform is built into the 16-bit variant kernel");
  static_assert(!CONTIG || (!VAR && !KV8), "affine addressing is built for the plain 16-bit kernel");
  const int lane = threadIdx.x;
  const int m = lane & 15;  // K: token in page; V: 16-byte column block; S/O: query head
  const int c = lane >> 4;  // lane group
  const int cta = blockIdx.x;
  const int kvh = blockIdx.y;
  const int g = p.group;
  const int H = p.num_qo_heads;
  const float NEG_INF = -__builtin_inff();

  constexpr int kElem = KV8 ? 1 : 2;  // bytes per stored K/V element
  using Tile = KvTile<KV8>;
  const uint8_t* kbase =
      static_cast<const uint8_t*>(p.k_pool) + (kvh * p.stride_head + c * p.stride_tok + m * 8) * kElem;
  // K relayout buffer: block (page pg, token t, 16-byte block x) lives at pg*4096 + t*256 + ((x ^ t) & 15)*16
  __shared__ __attribute__((aligned(16))) u32x4_t k_lds[2 * 16 * 16];
  const uint8_t* vbase =
      static_cast<const uint8_t*>(p.v_pool) + (kvh * p.stride_head + (4 * c) * p.stride_tok + m * 8) * kElem;
  const int64_t stride_tok = p.stride_tok * kElem;    // bytes from here on
  const int64_t stride_page = p.stride_page * kElem;
  // this lane's 8 columns of slot 0 of page 0 of the kv head (ANYPS adds page and slot per row)
  const uint8_t* khead = static_cast<const uint8_t*>(p.k_pool) + (kvh * p.stride_head + m * 8) * kElem;
  const uint8_t* vhead = static_cast<const uint8_t*>(p.v_pool) + (kvh * p.stride_head + m * 8) * kElem;
  auto ld_piece = [](const uint8_t* ptr) {
    if constexpr (KV8) {
      return ld8_stream(ptr);
    } else {
      return ld16_stream(reinterpret_cast<const uint16_t*>(ptr));
    }
  };

  // The plan arrays and the page table are only read while the kernel runs: viewed through the
  // constant address space their (wavefront-uniform) loads become scalar loads, which do not
  // share a counter with the K/V loads in flight; a vector load of a page id waits for every
  // K/V load issued before it.  Measured on the two decode workloads: with 8-bit K/V scalar
  // page ids are 8 % faster (half the bytes per tile leave less to hide that wait behind), with
  // 16-bit K/V the vector loads are 1 % faster, and issuing the tile loads unconditionally, so
  // that every wait is counted with the later tiles still in flight, is 4-7 % slower for both.
  using ConstInts = const __attribute__((address_space(4))) int32_t*;
  auto as_const = [](const int32_t* ptr) { return (ConstInts)(reinterpret_cast<uintptr_t>(ptr)); };
  ConstInts cta_indptr = as_const(p.cta_indptr), w_q_row0 = as_const(p.w_q_row0), w_kv_page0 = as_const(p.w_kv_page0),
            w_kv_len = as_const(p.w_kv_len), w_out_slot = as_const(p.w_out_slot), page_ids = as_const(p.kv_indices);
  const int w_begin = cta_indptr[cta];
  const int w_end = cta_indptr[cta + 1];

  // the frequency tables, one entry per lane, in LDS: a lane later reads the eight entries of each of its blocks
  // (the CTA is one wavefront: its LDS operations execute in program order)
  __shared__ __attribute__((aligned(16))) float rope_lds[ROPE ? 128 : 4];
  if constexpr (ROPE) {
    rope_lds[lane] = rope.rev[lane];
    rope_lds[64 + lane] = rope.rev256[lane];
  }
  // cosines and sines of the lane's eight pairs of block pair sp (components 32 sp + 8 c + e and + 64) at position t
  auto angles = [&](int t, int sp, float* cs, float* sn) {
    const float t1 = static_cast<float>(t >> 8), t0 = static_cast<float>(t & 255);
    const f32x4_t* fr = reinterpret_cast<const f32x4_t*>(&rope_lds[32 * sp + 8 * c]);
    const f32x4_t* gr = reinterpret_cast<const f32x4_t*>(&rope_lds[64 + 32 * sp + 8 * c]);
    const f32x4_t f0 = fr[0], f1 = fr[1], g0 = gr[0], g1 = gr[1];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float f = e < 4 ? f0[e & 3] : f1[e & 3], g = e < 4 ? g0[e & 3] : g1[e & 3];
      const float rev = __builtin_amdgcn_fractf(t1 * g + t0 * f);
      cs[e] = __builtin_amdgcn_cosf(rev);
      sn[e] = __builtin_amdgcn_sinf(rev);
    }
  };

  for (int w = w_begin; w < w_end; ++w) {
    const int q_row0 = w_q_row0[w];
    const int kv_page0 = w_kv_page0[w];
    const int kv_len = w_kv_len[w];
    const int out_slot = w_out_slot[w];
    const int ps_log2 = ANYPS ? p.page_log2 : 4;
    // variants: chunk-local token index -> distance to the query
    int tok_minus_pos = 0;  // (absolute index of the chunk's first token) - pos
    int tok_abs0 = 0;       // absolute index of the chunk's first token
    int pos = 0;
    float slope_log2 = 0.f;
    if constexpr (VAR) {
      const int req = as_const(p.w_request)[w];
      ConstInts indptr = as_const(p.kv_indptr);
      const int n_pg = indptr[req + 1] - indptr[req];
      const int l_kv = n_pg > 0 ? ((n_pg - 1) << p.page_log2) + as_const(p.last_page_len)[req] : 0;
      tok_abs0 = as_const(p.w_kv_start)[w];
      pos = l_kv - 1;
      tok_minus_pos = tok_abs0 - pos;
      if (p.alibi_slopes != nullptr && m < g) slope_log2 = p.alibi_slopes[kvh * g + m] * 1.4426950408889634f;
    }
    const int n_pages = (kv_len + (1 << ps_log2) - 1) >> ps_log2;
    const int n_tiles = (kv_len + 31) / 32;

    // Q^T as the B operand of the first product: lane (m, c) holds head m, d = 32 s + 8 c .. +8
    u32x4_t qreg[4];
    if (m < g) {
      const uint16_t* qp =
          static_cast<const uint16_t*>(p.q) + (static_cast<int64_t>(q_row0) * H + kvh * g + m) * kHeadDim + c * 8;
#pragma unroll
      for (int s = 0; s < 4; ++s) qreg[s] = ld16(qp + 32 * s);
    } else {
#pragma unroll
      for (int s = 0; s < 4; ++s) qreg[s] = u32x4_t{0u, 0u, 0u, 0u};
    }

    u32x4_t qlo[ROPE ? 4 : 1];  // remainder of the rotated query
    if constexpr (ROPE) {
#pragma unroll
      for (int sp = 0; sp < 2; ++sp) {
        float cs[8], sn[8];
        angles(pos, sp, cs, sn);
        u32x4_t xh, yh, xl, yl;
        rotate_blocks<BF>(qreg[sp], qreg[sp + 2], cs, sn, &xh, &yh, &xl, &yl);
        qreg[sp] = xh;
        qreg[sp + 2] = yh;
        qlo[sp] = xl;
        qlo[sp + 2] = yl;
      }
    }

    f32x4_t acc[8];  // acc[e][i] = O^T[d = 32 c + 8 i + e][head m]
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m_run = NEG_INF;  // running max of the scaled logits in log2 units (same in all 4 lane groups)
    float l_run = 0.f;      // this lane's share of the running sum

    // ANYPS: the page ids of a 32-token step (at most 32 pages), one per lane, fetched with one load two (8-bit
    // K/V: four) steps before the step's rows are requested; a lane then takes the id of each of its rows from the
    // lane that holds it.  (An index load per row would put a memory round trip in front of every row's load.)
    auto step_ids = [&](int t) {
      if constexpr (CONTIG) return 0;  // a page's id is its index: nothing to fetch
      const int first = (32 * t) >> ps_log2;
      return n_pages > 0 ? p.kv_indices[kv_page0 + min(first + (lane & 31), n_pages - 1)] : 0;
    };
    auto load_tile = [&](Tile& T, int& idv, int t) {
      if constexpr (ANYPS) {
        // row of chunk-local token tok: page tok >> ps_log2 (clamped to the chunk's last page: rows past the
        // end are masked later), slot tok % page_size
        const int first = (32 * t) >> ps_log2;
        auto row = [&](const uint8_t* base, int tok) {
          const int pg = min(tok >> ps_log2, n_pages - 1);
          const int64_t id = CONTIG ? kv_page0 + pg : __builtin_amdgcn_ds_bpermute((pg - first) << 2, idv);
          return base + id * stride_page + (tok & ((1 << ps_log2) - 1)) * stride_tok;
        };
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
          for (int s = 0; s < 4; ++s) T.k[pg][s] = ld_piece(row(khead, 32 * t + 16 * pg + 4 * s + c));
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
          for (int i = 0; i < 4; ++i) T.v[pg][i] = ld_piece(row(vhead, 32 * t + 16 * pg + 4 * c + i));
        idv = step_ids(t + (KV8 ? 4 : 2));  // for the step that reuses this tile's registers
        return;
      }
      const int pi = kv_page0 + 2 * t;
      int pg0, pg1;
      if constexpr (CONTIG) {
        pg0 = pi;
        pg1 = (2 * t + 1 < n_pages) ? pi + 1 : pi;
      } else if constexpr (KV8) {
        pg0 = page_ids[pi];
        pg1 = (2 * t + 1 < n_pages) ? page_ids[pi + 1] : pg0;
      } else {
        pg0 = __builtin_amdgcn_readfirstlane(p.kv_indices[pi]);
        pg1 = (2 * t + 1 < n_pages) ? __builtin_amdgcn_readfirstlane(p.kv_indices[pi + 1]) : pg0;
      }
      const uint8_t* k0 = kbase + pg0 * stride_page;
      const uint8_t* k1 = kbase + pg1 * stride_page;
      const uint8_t* v0 = vbase + pg0 * stride_page;
      const uint8_t* v1 = vbase + pg1 * stride_page;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        T.k[0][s] = ld_piece(k0 + 4 * s * stride_tok);
        T.k[1][s] = ld_piece(k1 + 4 * s * stride_tok);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        T.v[0][i] = ld_piece(v0 + i * stride_tok);
        T.v[1][i] = ld_piece(v1 + i * stride_tok);
      }
    };

    auto compute_tile = [&](Tile& T, int t) {
      // ---- S^T = K . Q^T ----
      // K rows -> LDS (token 4 j + c, block m), then back as A operands (token m, block 4 s + c)
#pragma unroll
      for (int pg = 0; pg < 2; ++pg)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int tk = 4 * j + c;
          if constexpr (KV8) {
            k_lds[pg * 256 + tk * 16 + ((m ^ tk) & 15)] = widen8<BF>(T.k[pg][j]);
          } else {
            k_lds[pg * 256 + tk * 16 + ((m ^ tk) & 15)] = T.k[pg][j];
          }
        }
      f32x4_t s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
      if constexpr (ROPE) {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
          f32x4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int sp = 0; sp < 2; ++sp) {
            float cs[8], sn[8];
            angles(tok_abs0 + 32 * t + 16 * pg + m, sp, cs, sn);  // this lane's K row is token m of the page
            const u32x4_t x = k_lds[pg * 256 + m * 16 + (((4 * sp + c) ^ m) & 15)];
            const u32x4_t y = k_lds[pg * 256 + m * 16 + (((4 * (sp + 2) + c) ^ m) & 15)];
            u32x4_t xh, yh, xl, yl;
            rotate_blocks<BF>(x, y, cs, sn, &xh, &yh, &xl, &yl);
            sacc = mfma_16x16x32<BF>(xh, qreg[sp], sacc);
            sacc = mfma_16x16x32<BF>(yh, qreg[sp + 2], sacc);
            sacc = mfma_16x16x32<BF>(xl, qreg[sp], sacc);
            sacc = mfma_16x16x32<BF>(yl, qreg[sp + 2], sacc);
            sacc = mfma_16x16x32<BF>(xh, qlo[sp], sacc);
            sacc = mfma_16x16x32<BF>(yh, qlo[sp + 2], sacc);
          }
          if (pg == 0) s0 = sacc; else s1 = sacc;
        }
      } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const u32x4_t ka0 = k_lds[m * 16 + (((4 * s + c) ^ m) & 15)];
          const u32x4_t ka1 = k_lds[256 + m * 16 + (((4 * s + c) ^ m) & 15)];
          s0 = mfma_16x16x32<BF>(ka0, qreg[s], s0);
          s1 = mfma_16x16x32<BF>(ka1, qreg[s], s1);
        }
      }
      // lane (m, c) now holds S^T[token 16 pg + 4 c + i][head m]
      const int tok0 = 32 * t + 4 * c;
      float sv[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        sv[i] = s0[i] * p.scale_log2;
        sv[4 + i] = s1[i] * p.scale_log2;
      }
      if constexpr (VAR) {
        const float cap = p.soft_cap;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int dist = tok_minus_pos + tok0 + 16 * (j >> 2) + (j & 3);  // t - pos, <= 0
          float s = sv[j];
          if (cap > 0.f) {  // cap * tanh(s / cap), s in log2 units: tanh(x) = 1 - 2 / (1 + exp(2 x))
            const float e2x = __builtin_amdgcn_exp2f(s * (2.0f / cap));
            s = cap * 1.4426950408889634f * (1.0f - 2.0f / (1.0f + e2x));
          }
          s += slope_log2 * static_cast<float>(dist);
          if (p.window_left >= 0 && dist < -p.window_left) s = NEG_INF;
          sv[j] = s;
        }
      }
      if (32 * t + 32 > kv_len) {  // ragged tail: hide tokens past the chunk, and zero their V rows
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool ok0 = tok0 + i < kv_len;
          const bool ok1 = tok0 + 16 + i < kv_len;
          sv[i] = ok0 ? sv[i] : NEG_INF;
          sv[4 + i] = ok1 ? sv[4 + i] : NEG_INF;
          if (!ok0) T.v[0][i] = typename Tile::Piece(0u);  // all-zero bits are 0.0 in every stored type
          if (!ok1) T.v[1][i] = typename Tile::Piece(0u);
        }
      }
      // ---- online softmax ----
      float tmax = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float m_new = fmaxf(m_run, tmax);  // finite: a tile always holds at least one valid token (VAR: may not)
      const bool none_yet = VAR && m_new == NEG_INF;
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
      u32x4_t pb, pb_lo;
      pb = u32x4_t{pack2<BF>(pv[0], pv[1]), pack2<BF>(pv[2], pv[3]), pack2<BF>(pv[4], pv[5]), pack2<BF>(pv[6], pv[7])};
      if constexpr (BF) {
        float r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = pv[j] - bf16_round(pv[j]);
        pb_lo = u32x4_t{pack2<BF>(r[0], r[1]), pack2<BF>(r[2], r[3]), pack2<BF>(r[4], r[5]), pack2<BF>(r[6], r[7])};
      }
      // ---- O^T += V^T . P^T, one product per column e of the lane's 8-wide block ----
      // vt[e][pg * 2 + pr] = column e of tokens (2 pr, 2 pr + 1) of page pg, as a pair of 16-bit values
      u32x4_t vt[8];
      if constexpr (KV8) {
        // the codes of a token pair are interleaved byte-wise first, so that one conversion yields the pair
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
          for (int pr = 0; pr < 2; ++pr)
#pragma unroll
            for (int w2 = 0; w2 < 2; ++w2) {
              const uint32_t x = T.v[pg][2 * pr][w2], y = T.v[pg][2 * pr + 1][w2];  // columns 4 w2 .. 4 w2 + 3
              const uint32_t z01 = __builtin_amdgcn_perm(y, x, 0x05010400u);        // x.b0 y.b0 x.b1 y.b1
              const uint32_t z23 = __builtin_amdgcn_perm(y, x, 0x07030602u);        // x.b2 y.b2 x.b3 y.b3
              const u32x4_t four = widen8<BF>(u32x2_t{z01, z23});
#pragma unroll
              for (int e = 0; e < 4; ++e) vt[4 * w2 + e][pg * 2 + pr] = four[e];
            }
      } else {
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
          const uint32_t a0 = T.v[0][0][wd], a1 = T.v[0][1][wd], a2 = T.v[0][2][wd], a3 = T.v[0][3][wd];
          const uint32_t b0 = T.v[1][0][wd], b1 = T.v[1][1][wd], b2 = T.v[1][2][wd], b3 = T.v[1][3][wd];
          vt[2 * wd] = u32x4_t{lo_halves(a0, a1), lo_halves(a2, a3), lo_halves(b0, b1), lo_halves(b2, b3)};
          vt[2 * wd + 1] = u32x4_t{hi_halves(a0, a1), hi_halves(a2, a3), hi_halves(b0, b1), hi_halves(b2, b3)};
        }
      }
#pragma unroll
      for (int wd = 0; wd < 4; ++wd) {
        acc[2 * wd] = mfma_16x16x32<BF>(vt[2 * wd], pb, acc[2 * wd]);
        acc[2 * wd + 1] = mfma_16x16x32<BF>(vt[2 * wd + 1], pb, acc[2 * wd + 1]);
        if constexpr (BF) {
          acc[2 * wd] = mfma_16x16x32<BF>(vt[2 * wd], pb_lo, acc[2 * wd]);
          acc[2 * wd + 1] = mfma_16x16x32<BF>(vt[2 * wd + 1], pb_lo, acc[2 * wd + 1]);
        }
      }
    };

    if constexpr (!KV8) {
      Tile TA, TB;
      // a sliding window hides the chunk's tokens before local index -window_left - tok_minus_pos: the steps that
      // lie wholly before it are not even loaded (a chunk wholly outside the window yields the empty state)
      int t_first = 0;
      if constexpr (VAR) {
        if (p.window_left >= 0) t_first = min(max(0, -p.window_left - tok_minus_pos) >> 5, n_tiles) & ~1;
      }
      int idA = 0, idB = 0;
      if constexpr (ANYPS) {
        idA = step_ids(t_first);
        idB = step_ids(t_first + 1);
      }
      if (n_tiles > t_first) load_tile(TA, idA, t_first);
      if (n_tiles > t_first + 1) load_tile(TB, idB, t_first + 1);
      for (int t = t_first; t < n_tiles; t += 2) {
        compute_tile(TA, t);
        if (t + 2 < n_tiles) load_tile(TA, idA, t + 2);
        if (t + 1 < n_tiles) {
          compute_tile(TB, t + 1);
          if (t + 3 < n_tiles) load_tile(TB, idB, t + 3);
        }
      }
    } else {  // half the bytes per tile: twice the tiles in flight
      Tile TA, TB, TC, TD;
      int idA = 0, idB = 0, idC = 0, idD = 0;
      if constexpr (ANYPS) {
        idA = step_ids(0);
        idB = step_ids(1);
        idC = step_ids(2);
        idD = step_ids(3);
      }
      if (n_tiles > 0) load_tile(TA, idA, 0);
      if (n_tiles > 1) load_tile(TB, idB, 1);
      if (n_tiles > 2) load_tile(TC, idC, 2);
      if (n_tiles > 3) load_tile(TD, idD, 3);
      for (int t = 0; t < n_tiles; t += 4) {
        compute_tile(TA, t);
        if (t + 4 < n_tiles) load_tile(TA, idA, t + 4);
        if (t + 1 < n_tiles) {
          compute_tile(TB, t + 1);
          if (t + 5 < n_tiles) load_tile(TB, idB, t + 5);
        }
        if (t + 2 < n_tiles) {
          compute_tile(TC, t + 2);
          if (t + 6 < n_tiles) load_tile(TC, idC, t + 6);
        }
        if (t + 3 < n_tiles) {
          compute_tile(TD, t + 3);
          if (t + 7 < n_tiles) load_tile(TD, idD, t + 7);
        }
      }
    }

    // ---- epilogue: o = O / l, lse = ln(sum exp) (Sec. 2.2) ----
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    const bool live = l_run > 0.f;
    float inv = live ? 1.0f / l_run : 0.f;
    if constexpr (KV8) inv *= p.out_scale;  // the V scale
    const float lse_val = live ? (m_run + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f : NEG_INF;
    if (m < g) {
      const int head = kvh * g + m;
      float* dst_o;
      float* dst_lse;
      if (out_slot < 0) {  // write-through (App. D.2)
        const int64_t row = static_cast<int64_t>(q_row0) * H + head;
        dst_o = p.o + row * kHeadDim;
        dst_lse = p.lse + row;
      } else {
        const int64_t row = static_cast<int64_t>(out_slot) * H + head;
        dst_o = p.part_o + row * kHeadDim;
        dst_lse = p.part_lse + row;
      }
      // a partial state that another CU's wavefront will fold inside this launch goes through the L2 to memory
      const bool through = p.w_merge != nullptr && out_slot >= 0;
      auto dev_store = [](float* ptr, float v) { __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float* d = dst_o + 32 * c + 8 * i;
        const f32x4_t lo = {acc[0][i] * inv, acc[1][i] * inv, acc[2][i] * inv, acc[3][i] * inv};
        const f32x4_t hi = {acc[4][i] * inv, acc[5][i] * inv, acc[6][i] * inv, acc[7][i] * inv};
        if (through) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            dev_store(d + e, lo[e]);
            dev_store(d + 4 + e, hi[e]);
          }
          continue;
        }
        if (out_slot >= 0 || p.o != nullptr) {  // final rows may be wanted in the input type only
          *reinterpret_cast<f32x4_t*>(d) = lo;
          *reinterpret_cast<f32x4_t*>(d + 4) = hi;
        }
        if (out_slot < 0 && p.o_cast != nullptr) {
          uint16_t* dc = static_cast<uint16_t*>(p.o_cast) +
                         (static_cast<int64_t>(q_row0) * H + head) * kHeadDim + 32 * c + 8 * i;
          const u32x4_t pk = {pack2<BF>(lo[0], lo[1]), pack2<BF>(lo[2], lo[3]), pack2<BF>(hi[0], hi[1]),
                              pack2<BF>(hi[2], hi[3])};
          *reinterpret_cast<u32x4_t*>(dc) = pk;
        }
      }
      if (c == 0) {
        if (through)
          dev_store(dst_lse, lse_val);
        else
          *dst_lse = lse_val;
      }
    }

    // ---- contraction inside the launch (Sec. 3.3.1): the wavefront that delivers a split tile's last partial
    //      state folds all of them, in chunk order, whichever wavefront that is: the result does not depend on
    //      the order of arrival.  The partial states come from other CUs, possibly behind another L2.  They were
    //      written with device-scope stores (through the L2, see above), the arrival is counted after those stores
    //      have completed, and they are read with device-scope loads: no cache is written back or invalidated as a
    //      whole, which a release / acquire fence pair would do for every split work item. ----
    if (p.w_merge != nullptr && out_slot >= 0) {
      const int mi = as_const(p.w_merge)[w];
      const int n_chunks = as_const(p.m_n_chunks)[mi];
      const int slot_base = as_const(p.m_slot_base)[mi];
      int32_t* counter = p.merge_counters + mi * p.num_kv_heads + kvh;
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wavefront's partial state has reached memory
      int arrived = 0;
      if (lane == 0) arrived = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      arrived = __builtin_amdgcn_readfirstlane(arrived);
      if (arrived == n_chunks - 1) {
        // lanes: head hd = lane / lanes_per_head, floats [fl * sub, fl * (sub + 1)) of its 128, fl = 2 g
        const int lanes_per_head = 64 / g;
        const int hd = lane / lanes_per_head, sub = lane % lanes_per_head;
        const int head = kvh * g + hd;
        const int fl = 2 * g;
        auto dev_load = [](const float* ptr) { return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
        auto lse_of = [&](int ch) { return dev_load(p.part_lse + static_cast<int64_t>(slot_base + ch) * H + head); };
        float mx = NEG_INF;
        for (int ch = sub; ch < n_chunks; ch += lanes_per_head) mx = fmaxf(mx, lse_of(ch));
        for (int off = lanes_per_head >> 1; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        float den = 0.f;
        if (mx != NEG_INF)
          for (int ch = sub; ch < n_chunks; ch += lanes_per_head)
            den += __builtin_amdgcn_exp2f((lse_of(ch) - mx) * 1.4426950408889634f);
        for (int off = lanes_per_head >> 1; off >= 1; off >>= 1) den += __shfl_xor(den, off);
        float acc_o[8];  // fl <= 8 values
#pragma unroll
        for (int e = 0; e < 8; ++e) acc_o[e] = 0.f;
        if (mx != NEG_INF) {
          const float inv_den = 1.0f / den;
          // chunks in order, four at a time so that their loads are in flight together
          for (int ch0 = 0; ch0 < n_chunks; ch0 += 4) {
            float wgt[4], val[4][8];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int ch = min(ch0 + u, n_chunks - 1);
              const float* src = p.part_o + (static_cast<int64_t>(slot_base + ch) * H + head) * kHeadDim + fl * sub;
              wgt[u] = lse_of(ch);
#pragma unroll
              for (int e = 0; e < 8; ++e) val[u][e] = e < fl ? dev_load(src + e) : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const float wu = ch0 + u < n_chunks ? __builtin_amdgcn_exp2f((wgt[u] - mx) * 1.4426950408889634f) * inv_den : 0.f;
              if (wu != 0.f) {  // a state with lse = -inf is the identity, whatever its o holds
#pragma unroll
                for (int e = 0; e < 8; ++e) acc_o[e] += wu * val[u][e];
              }
            }
          }
        }
        const int64_t out_row = static_cast<int64_t>(q_row0) * H + head;
        float* dst = p.o + out_row * kHeadDim + fl * sub;
#pragma unroll
        for (int e = 0; e < 8; e += 2)
          if (e < fl && p.o != nullptr) *reinterpret_cast<f32x2_t*>(dst + e) = f32x2_t{acc_o[e], acc_o[e + 1]};
        if (sub == 0) p.lse[out_row] = mx != NEG_INF ? mx + __builtin_amdgcn_logf(den) * 0.6931471805599453f : NEG_INF;
        if (p.o_cast != nullptr) {
          uint32_t* dc = static_cast<uint32_t*>(p.o_cast) + (out_row * kHeadDim + fl * sub) / 2;
#pragma unroll
          for (int e = 0; e < 8; e += 2)
            if (e < fl) dc[e / 2] = pack2<BF>(acc_o[e], acc_o[e + 1]);
        }
        // ready for the next launch with this plan (a new plan brings zeros anyway)
        if (lane == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
}

}  // namespace

namespace {
template <bool ANYPS>
void launch_decode_ps(const RunParams& p, bool is_bf16, bool kv8, hipStream_t stream) {
  const dim3 grid(static_cast<unsigned>(p.ctas_per_head), static_cast<unsigned>(p.num_kv_heads), 1);
  const dim3 block(64, 1, 1);
  if (kv8) {
    if (is_bf16)
      hipLaunchKernelGGL((decode_kernel<true, true, ANYPS>), grid, block, 0, stream, p, NoRope{});
    else
      hipLaunchKernelGGL((decode_kernel<false, true, ANYPS>), grid, block, 0, stream, p, NoRope{});
  } else {
    if (is_bf16)
      hipLaunchKernelGGL((decode_kernel<true, false, ANYPS>), grid, block, 0, stream, p, NoRope{});
    else
      hipLaunchKernelGGL((decode_kernel<false, false, ANYPS>), grid, block, 0, stream, p, NoRope{});
  }
}
}  // namespace

hipError_t launch_decode(const RunParams& p, bool is_bf16, bool kv8, bool variant, const RopeTable* rope,
                         hipStream_t stream) {
  if (variant) {
    const dim3 grid(static_cast<unsigned>(p.ctas_per_head), static_cast<unsigned>(p.num_kv_heads), 1);
    if (rope) {
      if (is_bf16)
        hipLaunchKernelGGL((decode_kernel<true, false, false, true, true>), grid, dim3(64, 1, 1), 0, stream, p, *rope);
      else
        hipLaunchKernelGGL((decode_kernel<false, false, false, true, true>), grid, dim3(64, 1, 1), 0, stream, p, *rope);
    } else if (p.page_log2 != 4) {  // the logits hooks on the general path (any page size)
      if (is_bf16)
        hipLaunchKernelGGL((decode_kernel<true, false, true, true>), grid, dim3(64, 1, 1), 0, stream, p, NoRope{});
      else
        hipLaunchKernelGGL((decode_kernel<false, false, true, true>), grid, dim3(64, 1, 1), 0, stream, p, NoRope{});
    } else if (is_bf16) {
      hipLaunchKernelGGL((decode_kernel<true, false, false, true>), grid, dim3(64, 1, 1), 0, stream, p, NoRope{});
    } else {
      hipLaunchKernelGGL((decode_kernel<false, false, false, true>), grid, dim3(64, 1, 1), 0, stream, p, NoRope{});
    }
    return hipGetLastError();
  }
  if (p.kv_indices == nullptr) {  // contiguous KV: affine addressing (the caller has refused kv8 and variants)
    const dim3 grid(static_cast<unsigned>(p.ctas_per_head), static_cast<unsigned>(p.num_kv_heads), 1);
    if (p.page_log2 == 4) {
      if (is_bf16)
        hipLaunchKernelGGL((decode_kernel<true, false, false, false, false, true>), grid, dim3(64, 1, 1), 0, stream, p, NoRope{});
      else
        hipLaunchKernelGGL((decode_kernel<false, false, false, false, false, true>), grid, dim3(64, 1, 1), 0, stream, p, NoRope{});
    } else {
      if (is_bf16)
        hipLaunchKernelGGL((decode_kernel<true, false, true, false, false, true>), grid, dim3(64, 1, 1), 0, stream, p, NoRope{});
      else
        hipLaunchKernelGGL((decode_kernel<false, false, true, false, false, true>), grid, dim3(64, 1, 1), 0, stream, p, NoRope{});
    }
    return hipGetLastError();
  }
  if (p.page_log2 == 4)
    launch_decode_ps<false>(p, is_bf16, kv8, stream);
  else
    launch_decode_ps<true>(p, is_bf16, kv8, stream);
  return hipGetLastError();
}

}  // namespace fi355
