// Paged append / prefill attention for gfx950 (causal or not): query tile = 256 fused rows
// (256/g consecutive positions x g query heads of one kv head, App. A), one CTA of eight
// wavefronts per CU, each wavefront owning 32 rows.  K/V tiles of 64 tokens (four 16-token
// pages, gathered through kv_indices, Sec. 3.2.1) are staged in LDS and shared by the eight
// wavefronts; both products run on the matrix cores:
//   S^T[token][row] = K . Q^T      v_mfma_f32_32x32x16   A = K rows from LDS, B = Q^T in registers
//   O^T[d][row]    += V^T . P^T    v_mfma_f32_32x32x16   A = V^T read from the row-major V tile with
//                                                        the LDS transpose read ds_read_b64_tr_b16,
//                                                        B = P^T straight from the S^T accumulators
// Computing the transposed products puts one query row per lane column (lane % 32), with 16
// of the step's 32 tokens in each half of the wavefront: the row maximum (needed only when the
// reference is raised) is an in-lane reduction plus one cross-lane exchange, and P never
// moves between lanes.  The contraction index of the second product is (lane half, register)
// on both operands, so its order inside the instruction does not matter.
//
// A work item (one query tile x one KV chunk of the plan, Sec. 3.3.1) runs on one of two paths:
//   * the scheduled loop: generated assembly (gen/gen_append_loop.py -> append_loop_*.inc) that
//     interleaves, inside every wavefront, the matrix instructions of one step with the softmax
//     and the LDS traffic of its neighbours, over triple-buffered tiles; it takes every chunk
//     of at least 128 tokens whose first tile all rows of the CTA see, and does the whole item
//     including masked tiles, epilogue and stores;
//   * the generic path (generic_work_item): compiler-scheduled, any length and masking.
//
// P is rounded to fp16 (11 significant bits).  For bf16 inputs V is converted to fp16 while it
// is staged into LDS (exact for 2^-14 <= |v| <= 65504, saturating above, absolute error
// < 2^-24 below), because a bf16 P (8 bits) would miss the 2e-3 output tolerance on rows that
// see few keys; Q.K^T stays in the input type.
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

constexpr int kTileKv = 64;        // tokens per LDS tile
constexpr int kRowElems = 136;     // K tile row pitch in 16-bit elements (272 B): rows 4 banks apart, conflict-free b128 reads
constexpr int kRowElemsV = 160;    // V tile row pitch (320 B): rows 16 banks apart, conflict-free transpose reads
constexpr int kCtaThreads = 512;   // 8 wavefronts, 32 query rows each
constexpr int kRowBlocks = 1;       // 32-row blocks per wavefront; CTA tile = 8 * 32 * kRowBlocks fused rows
constexpr int kLoopBuffers = 3;                                 // LDS tile buffers of the scheduled loop
// LDS map.  K tiles from 0 (the scheduled loop: three packed 16 KB buffers; the generic path: two of 17 KB);
// behind the loop's K buffers, up to 64 KB, 16 KB that together with K buffer 2 stage the V tiles requested for
// the CTA's next work item; V tiles from 64 KB (three buffers of 20 KB); the loop's output transpose area also
// from 64 KB, so that it leaves K buffers 0 and 1 and the staging area to the next work item's tiles, which are
// on their way while the outputs are written.  Everything a load writes directly lies below 64 KB.
constexpr int kLdsVOffset = 65536;
static_assert(kLoopBuffers * kTileKv * kRowElems * 2 <= kLdsVOffset, "K tiles end before the V tiles");
constexpr int kEpilogueRowBytes = 288;                          // row pitch of the loop's output transpose area
constexpr int kEpilogueLdsBytes = 32 * kEpilogueRowBytes;       // per wavefront
constexpr int kEpilogueBase = kLdsVOffset;
constexpr int kLdsTileEnd = kLdsVOffset + kLoopBuffers * kTileKv * kRowElemsV * 2;
constexpr int kLdsEpilogueEnd = kEpilogueBase + (kCtaThreads / 64) * kEpilogueLdsBytes;
constexpr int kLdsBytes = kLdsTileEnd > kLdsEpilogueEnd ? kLdsTileEnd : kLdsEpilogueEnd;
static_assert(kLdsBytes <= 160 * 1024, "fits the CU's LDS");
constexpr int kLoopMinTokens = 2 * kTileKv;                     // shorter chunks: generic path only (its start-up is cheaper)
constexpr int kLazyLog2 = 8;                                    // P may reach 2^8 before the reference is raised
constexpr uint16_t kLazyF16Bits = (15 + kLazyLog2) << 10;       // fp16 bit pattern of 2^kLazyLog2

typedef __attribute__((ext_vector_type(16))) float f32x16_t;

template <bool BF>
__device__ __forceinline__ f32x16_t mfma_qk(u32x4_t a, u32x4_t b, f32x16_t c) {
  if constexpr (BF) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                   c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c,
                                                  0, 0, 0);
  }
}
__device__ __forceinline__ f32x16_t mfma_pv(u32x4_t a, u32x4_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0,
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
typedef __attribute__((ext_vector_type(2))) uint16_t u16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
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

// Exchange between the two halves of a wavefront without going through LDS:
// v_permlane32_swap swaps the upper half of its first operand with the lower half of its
// second.  With both operands holding x, the pair afterwards holds (x of lane l, x of lane
// l ^ 32) in some order, which is all a max or a sum needs.
__device__ __forceinline__ void swap32(float x, float* a, float* b) {
  uint32_t u = __builtin_bit_cast(uint32_t, x), v = u;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32_e32 %0, %1" : "+v"(u), "+v"(v));
  *a = __builtin_bit_cast(float, u);
  *b = __builtin_bit_cast(float, v);
}
__device__ __forceinline__ float halves_max(float x) {
  float a, b;
  swap32(x, &a, &b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float halves_sum(float x) {
  float a, b;
  swap32(x, &a, &b);
  return a + b;
}

#ifndef FI355_APPEND_SCHEDULED_LOOP
#define FI355_APPEND_SCHEDULED_LOOP 1
#endif
constexpr bool kUseScheduledLoop = FI355_APPEND_SCHEDULED_LOOP != 0 && kRowBlocks == 1 && kCtaThreads == 512;

__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (__attribute__((address_space(3))) const uint8_t*)(static_cast<const uint8_t*>(p))));
}

// One entry of the plan's work list (Sec. 3.3.1), in scalar registers.  The fields are read with
// scalar loads (the plan arrays were written by an earlier kernel): the scalar path does not
// queue behind the previous item's output stores the way a vector load would.  Loads and wait
// are one statement, so the compiler never sees a register whose load is still in flight.
struct WorkItem {
  int q_row0, n_pos, kv_page0, kv_start, kv_len, diag0, out_slot;
  template <class Params>
  __device__ __forceinline__ void load(const Params& p, int w) {
    const int off = w * 4;
    asm volatile(
        "s_load_dword %0, %7, %14\n\t"
        "s_load_dword %1, %8, %14\n\t"
        "s_load_dword %2, %9, %14\n\t"
        "s_load_dword %3, %10, %14\n\t"
        "s_load_dword %4, %11, %14\n\t"
        "s_load_dword %5, %12, %14\n\t"
        "s_load_dword %6, %13, %14\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(q_row0), "=&s"(n_pos), "=&s"(kv_page0), "=&s"(kv_start), "=&s"(kv_len), "=&s"(diag0), "=&s"(out_slot)
        : "s"(p.w_q_row0), "s"(p.w_n_pos), "s"(p.w_kv_page0), "s"(p.w_kv_start), "s"(p.w_kv_len), "s"(p.w_diag0),
          "s"(p.w_out_slot), "s"(off)
        : "memory");
  }
};

// The hand-scheduled loop over the `n_tiles` KV tiles of a chunk of `kv_len` tokens, of which the
// first `n_full` >= 1 need no masking (gen/gen_append_loop.py writes it and documents its
// register map and schedule).  `cap` = chunk-local index of the last token this lane's row sees,
// minus 4 * (lane / 32).  Starts from the empty attention state, reads Q through `q_addr`,
// gathers pages through `page_ids` (the chunk's ids; `ids_clamp` = byte offset of the chunk's
// last one) and finishes the work item.  Output row of tile row R (position R >> g_log2, head
// R % g) is row_base + position * num_qo_heads + head, written if position < n_pos: o (512 B per
// row) to o_base, and, if has_cast, o in the input type to cast_base; the rows pass through the
// wavefront's LDS area (epi_write: this lane's accumulator column, epi_read: the 16-byte piece
// it stores).  lse goes to lse_base[o_off / 512] from the first 32 lanes of a wavefront whose row exists.
// What depends on the thread index alone (its staging row, the swizzle of its operand reads, the piece of an
// output row it stores) the block derives from `thread`: every per-lane operand occupies one of the sixteen
// vector registers the block leaves to the compiler for as long as it runs.
// Every wavefront of the CTA must call it with the same tile counts (it contains CTA barriers).
//
// Seam to the next work item: the block reads the plan entry at byte offset `next_off & ~3` of
// the work arrays (`w_fields` = the q_row0 array, the others follow `w_stride` bytes apart) into
// `next`; if bit 0 of `next_off` is set (there is a next item) and that item will run this loop
// too, it requests the item's first two K and V tiles into LDS (page ids from `all_ids`, the whole
// page table) before it writes its own outputs, and sets `prefetched_out`.  The next call is then
// made with bit 1 of `next_off` set.  Whoever uses the LDS otherwise after a block that set
// `prefetched_out` waits for vmcnt(0) first.
// CAP: the variant of the loop with the logits soft cap (Sec. 3.2.3).  The capped logits are in log2 units, the
// softmax scale after the transform is 1, and the block has no scalar register to spare: `scale_log2` then
// carries 2 * sm_scale * log2(e) / c, `wave_index` the bits of c * log2(e), and `g_log2` the wavefront index in
// bits 8.. above log2 of the group size.
// CONTIG: contiguous KV (page j of the chunk is page kv_page0 + j of the pool): the page ids are computed instead of
// loaded; `all_ids_lo` then carries the chunk's kv_page0, `page_ids` and `all_ids_hi` are unused.
// VARL: the variant of the loop with the ALiBi bias and the sliding window (Sec. 3.2.3; causal items): `cap` then
// carries lim - 4 * (lane / 32) uncapped, lim = chunk-local index of the row's own token; `slope` = the row's head's
// slope times log2(e) (0: none), `win` = window_left (a huge value: none).
// PSL: the variant for page sizes 4, 8 and 32: `g_log2` carries log2 of the page size in bits 8.., `ids_clamp` and
// `page_ids` count pages of that size, and the per-lane row offsets hold the row's place inside its page.
// ROWS: the variant for page sizes 1 and 2 (a page id per token row, 64-bit addresses per lane): operands as for PSL.
template <bool BF, bool CAP, bool CONTIG, bool VARL, bool PSL = false, bool ROWS = false>
__device__ __forceinline__ void run_scheduled_loop(int n_full, int n_tiles, int kv_len, int cap, int thread, int ids_clamp, const int32_t* page_ids, uint32_t k_lo,
                                                   uint32_t k_hi, uint32_t v_lo, uint32_t v_hi, uint32_t page_bytes,
                                                   float scale_log2, uint64_t q_addr, uint32_t st_off_bytes,
                                                   uint32_t k_off_bytes, uint32_t k_read,
                                                   uint32_t v_read, uint32_t k_dma, uint32_t v_write,
                                                   uint32_t o_off, float* o_base, float* lse_base,
                                                   void* cast_base, int has_cast, uint32_t epi_write, uint32_t epi_read,
                                                   int g_log2, int num_qo_heads, int row_base,
                                                   int n_pos, int wave_index, int next_off,
                                                   const int32_t* w_fields, int w_stride, uint32_t all_ids_lo,
                                                   uint32_t all_ids_hi, WorkItem& next, int& prefetched_out,
                                                   float& slope, int win = 0) {
#define FI355_LOOP_OPERANDS                                                                                              \
        : [nq] "=&s"(next.q_row0), [nn] "=&s"(next.n_pos), [npg] "=&s"(next.kv_page0), [nks] "=&s"(next.kv_start),          \
          [nkl] "=&s"(next.kv_len), [ndg] "=&s"(next.diag0), [nos] "=&s"(next.out_slot), [preo] "=&s"(prefetched_out)        \
          FI355_SLOPE_OPERAND                                                                                                  \
        : [nf] "s"(n_full), [nt] "s"(n_tiles), [kvl] "s"(kv_len), [cap] "{v1}"(cap), [tid] "{v4}"(thread), [npg1] "s"(ids_clamp), [idp] "s"(page_ids), [kblo] "s"(k_lo), [kbhi] "s"(k_hi), \
          [vblo] "s"(v_lo), [vbhi] "s"(v_hi), [sp] "s"(page_bytes), [sc] "s"(scale_log2),                                 \
          [qp] "{v[2:3]}"(q_addr), FI355_STAGING_OFFSETS [kb] "{v7}"(k_read),                               \
          [va] "{v8}"(v_read), [kd] "s"(k_dma), [wv] "{v9}"(v_write), [ooff] "{v10}"(o_off), [ob] "s"(o_base), [lb] "s"(lse_base), \
          [cb] "s"(cast_base), [oc] "s"(has_cast), [ew] "{v11}"(epi_write), [er] "{v12}"(epi_read),                                \
          [gl] "s"(g_log2), FI355_HEADS_AND_POSITIONS [rb] "s"(row_base), [stp8] "s"(wave_index),                          \
          [woff] "s"(next_off), [wq0] "s"(w_fields), [wstr] "s"(w_stride),                                                  \
          [idblo] "s"(all_ids_lo), [idbhi] "s"(all_ids_hi)
  // (the bias / window variant has a scalar operand more than there are registers left: it takes n_pos and
  // num_qo_heads packed into g_log2)
#define FI355_STAGING_OFFSETS [so] "{v5}"(st_off_bytes), [sok] "{v6}"(k_off_bytes),
#define FI355_HEADS_AND_POSITIONS
  // (the row's slope is loaded once per launch and handed from block to block in its register: read and written)
#define FI355_SLOPE_OPERAND , [slope] "+{v13}"(slope)
  if constexpr (VARL && BF) {
    asm volatile(
#include "append_loop_bf16_var.inc"
        FI355_LOOP_OPERANDS, [win] "s"(win)
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (VARL) {
    asm volatile(
#include "append_loop_f16_var.inc"
        FI355_LOOP_OPERANDS, [win] "s"(win)
        :
#include "append_loop_clobbers.inc"
    );
  }
#undef FI355_HEADS_AND_POSITIONS
#undef FI355_SLOPE_OPERAND
#define FI355_SLOPE_OPERAND
#define FI355_HEADS_AND_POSITIONS [hq] "s"(num_qo_heads), [np] "s"(n_pos),
  if constexpr (ROWS && CONTIG && BF) {
    asm volatile(
#include "append_loop_bf16_contig_rows.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (ROWS && CONTIG) {
    asm volatile(
#include "append_loop_f16_contig_rows.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (ROWS && BF) {
    asm volatile(
#include "append_loop_bf16_rows.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (ROWS) {
    asm volatile(
#include "append_loop_f16_rows.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  }
  if constexpr (VARL || ROWS) {
  } else if constexpr (PSL && CONTIG && BF) {
    asm volatile(
#include "append_loop_bf16_contig_ps.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (PSL && CONTIG) {
    asm volatile(
#include "append_loop_f16_contig_ps.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (PSL && BF) {
    asm volatile(
#include "append_loop_bf16_ps.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (PSL) {
    asm volatile(
#include "append_loop_f16_ps.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (CONTIG && BF) {
    asm volatile(
#include "append_loop_bf16_contig.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (CONTIG) {
    asm volatile(
#include "append_loop_f16_contig.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (CAP && BF) {
    asm volatile(
#include "append_loop_bf16_cap.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (CAP) {
    asm volatile(
#include "append_loop_f16_cap.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else if constexpr (BF) {
    asm volatile(
#include "append_loop_bf16.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  } else {
    asm volatile(
#include "append_loop_f16.inc"
        FI355_LOOP_OPERANDS
        :
#include "append_loop_clobbers.inc"
    );
  }
#undef FI355_LOOP_OPERANDS
#undef FI355_SLOPE_OPERAND
#undef FI355_HEADS_AND_POSITIONS
#undef FI355_STAGING_OFFSETS
}

// K tiles, then V tiles (three buffers each: the scheduled loop rotates over three, the generic
// path over the first two).
__shared__ __attribute__((aligned(16))) uint8_t lds_raw[kLdsBytes];

// Frequency tables of the rotary embedding (see RopeTable), one entry per pair of components, copied from the
// kernel's arguments at the start of the launch that rotates.
__shared__ __attribute__((aligned(16))) float rope_tab_lds[128];

// The second K tile of the rotary variant: the remainders of the rotated keys (the rotated keys enter the first
// product as head + remainder in the input type).  Buffer 0 behind the general path's two K buffers, buffer 1 in
// the third V buffer, which only the scheduled loop uses.
constexpr int kLdsKLo0 = 2 * kTileKv * kRowElems * 2;
constexpr int kLdsKLo1 = kLdsVOffset + 2 * kTileKv * kRowElemsV * 2;
static_assert(kLdsKLo0 + kTileKv * kRowElems * 2 <= kLdsVOffset && kLdsKLo1 + kTileKv * kRowElems * 2 <= kLdsBytes,
              "the remainder tiles fit into the gaps of the LDS map");

template <bool BF>
__device__ __forceinline__ float elem16(uint32_t word, int odd) {
  if constexpr (BF) {
    return __builtin_bit_cast(float, odd ? (word & 0xffff0000u) : (word << 16));
  } else {
    const f16x2_t h = __builtin_bit_cast(f16x2_t, word);
    return static_cast<float>(odd ? h[1] : h[0]);
  }
}

// cosines and sines of the eight pairs (d0 + e, d0 + e + 64), e = 0..7, at position t: the angle of pair d is
// t * rev[d] revolutions, reduced as fract(t1 * fract(256 rev[d]) + t0 * rev[d]) with t = 256 t1 + t0, so that large
// positions keep their low bits
__device__ __forceinline__ void rope_angles(int t, int d0, float* cs, float* sn) {
  const float t1 = static_cast<float>(t >> 8), t0 = static_cast<float>(t & 255);
  const f32x4_t* fr = reinterpret_cast<const f32x4_t*>(&rope_tab_lds[d0]);
  const f32x4_t* gr = reinterpret_cast<const f32x4_t*>(&rope_tab_lds[64 + d0]);
  const f32x4_t f0 = fr[0], f1 = fr[1], g0 = gr[0], g1 = gr[1];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float f = e < 4 ? f0[e & 3] : f1[e & 3], g = e < 4 ? g0[e & 3] : g1[e & 3];
    const float rev = __builtin_amdgcn_fractf(t1 * g + t0 * f);
    cs[e] = __builtin_amdgcn_cosf(rev);
    sn[e] = __builtin_amdgcn_sinf(rev);
  }
}

// v[e] (fp32) -> head in the input type and remainder v - head, also in the input type
template <bool BF>
__device__ __forceinline__ void split_head_remainder(const float* v, u32x4_t* head, u32x4_t* rem) {
  *head = u32x4_t{pack_out<BF>(v[0], v[1]), pack_out<BF>(v[2], v[3]), pack_out<BF>(v[4], v[5]), pack_out<BF>(v[6], v[7])};
  float r[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = v[e] - elem16<BF>((*head)[e >> 1], e & 1);
  *rem = u32x4_t{pack_out<BF>(r[0], r[1]), pack_out<BF>(r[2], r[3]), pack_out<BF>(r[4], r[5]), pack_out<BF>(r[6], r[7])};
}

// One work item on the generic path: any chunk length, any masking.  Kept out of line so that
// its loop-invariant registers do not have to live across the scheduled loop in the caller.
// Contains CTA barriers: every wavefront of the CTA calls it with the same item.
// (Arguments of a device function travel in vector registers: the item's fields and the address
// of the launch parameters, which the kernel takes from its argument segment, are made scalar
// again here.)
//
// VAR: attention variants (Sec. 3.2.3, logits transform and logits mask) for causal batches, where the item's
// diagonal gives every row its absolute position pos = diag0 + (row's position in the tile).  On the scaled
// logits, in this order: soft cap c * tanh(s / c), ALiBi bias slope[head] * (t - pos), sliding window (tokens
// t < pos - window hidden).  A window only masks: the tiles it hides are still read.
//
// ROPE (with VAR): rotary position embedding as query / key transform (Sec. 3.2.3; Sec. 4.3), pairing components
// (d, d + 64): the queries are rotated by their positions when they are loaded, the keys by theirs on the way from
// the staging registers into LDS (a thread holds one 8-wide block of a token and gets the partner block from lane
// ^ 8), once per CTA.  Rotated values are formed in fp32 and enter the first product as head + remainder in the input
// type (three matrix instructions per operand pair; a value rounded once costs 2^-9 (bf16) of relative accuracy per
// operand, about 1.6e-3 rms on a logit of N(0,1) data, more than the tolerance of lse).  The cache holds unrotated keys.
template <bool BF, bool VAR, bool ROPE = false>
__device__ __attribute__((noinline)) void generic_work_item(uint64_t params_addr, int a_q_row0, int a_n_pos,
                                                            int a_kv_page0, int a_kv_start, int a_kv_len, int a_diag0,
                                                            int a_out_slot) {
  typedef const __attribute__((address_space(4))) RunParams KernargParams;
  const uint64_t params_lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(params_addr)));
  const uint64_t params_hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(params_addr >> 32)));
  KernargParams& p = *reinterpret_cast<KernargParams*>(params_lo | (params_hi << 32));
  uint16_t* const lds_k = reinterpret_cast<uint16_t*>(lds_raw);
  uint16_t* const lds_v = reinterpret_cast<uint16_t*>(lds_raw + kLdsVOffset);
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int n = lane & 31;   // K: token of the 32-token step; V: column within a 32-wide block; S/O: query row
  const int c = lane >> 5;   // wavefront half
  const int kvh = static_cast<int>(blockIdx.x) % p.num_kv_heads;
  const int g = p.group;
  const int g_log2 = 31 - __builtin_clz(g);
  const int H = p.num_qo_heads;
  const float NEG_INF = -__builtin_inff();
  constexpr int kWaveRows = 32 * kRowBlocks;

  // staging role: in each of the two passes r over a 64-token tile this thread moves the 16-byte block
  // `st_chunk` of tile token 32 r + st_tok, i.e. slot st_tok % 16 of page 2 r + st_tok / 16 (wave-uniform)
  const int st_tok = tid >> 4;  // 0..31
  const int st_chunk = tid & 15;
  const int st_page = __builtin_amdgcn_readfirstlane(wave >> 2);  // = st_tok / 16
  const uint32_t st_off = static_cast<uint32_t>((st_tok & 15) * p.stride_tok + st_chunk * 8);  // within one (page, head) block
  const int st_lds_k = st_tok * kRowElems + st_chunk * 8;   // element offsets of this thread's block in a tile
  const int st_lds_v = st_tok * kRowElemsV + st_chunk * 8;
  const uint16_t* kpool = static_cast<const uint16_t*>(p.k_pool);
  const uint16_t* vpool = static_cast<const uint16_t*>(p.v_pool);

  // transpose-read role (see lds_read_tr16): in its 16-lane group this lane supplies the address of
  // token row (lane % 16) / 4, columns 4 * (lane % 4) .. + 3 of the group's 16 columns
  const int tr_row = (lane & 15) >> 2;
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  const int q_row0 = __builtin_amdgcn_readfirstlane(a_q_row0), n_pos = __builtin_amdgcn_readfirstlane(a_n_pos);
  const int kv_page0 = __builtin_amdgcn_readfirstlane(a_kv_page0), kv_start = __builtin_amdgcn_readfirstlane(a_kv_start);
  const int kv_len = __builtin_amdgcn_readfirstlane(a_kv_len), diag0 = __builtin_amdgcn_readfirstlane(a_diag0);
  const int out_slot = __builtin_amdgcn_readfirstlane(a_out_slot);
  const bool causal = diag0 != kNoDiagMarker;
  const int ps_log2 = p.page_log2;  // 4 on the tuned path; any power of two up to 64 here (64 % page_size == 0)
  const int n_pages = (kv_len + (1 << ps_log2) - 1) >> ps_log2;
  const int n_tiles = (kv_len + kTileKv - 1) / kTileKv;

  // ---- this lane's query rows, one per 32-row block ----
  int pos[kRowBlocks], hh[kRowBlocks], lim[kRowBlocks];
  float slope_log2[kRowBlocks];  // VAR: ALiBi slope of the row's head, times log2(e)
  bool row_ok[kRowBlocks];
  u32x4_t qreg[kRowBlocks][8];  // Q^T as B operand: row n of the block, d = 16 s + 8 c .. + 8
#pragma unroll
  for (int b = 0; b < kRowBlocks; ++b) {
    const int R = kWaveRows * wave + 32 * b + n;
    pos[b] = R >> g_log2;
    hh[b] = R & (g - 1);
    row_ok[b] = pos[b] < n_pos;
    // the row sees request tokens <= diag0 + pos; in chunk-local terms: local index <= lim
    lim[b] = causal ? diag0 + pos[b] - kv_start : 0x3FFFFFFF;
    slope_log2[b] = 0.f;
    if constexpr (VAR) {
      if (p.alibi_slopes != nullptr) slope_log2[b] = p.alibi_slopes[kvh * g + hh[b]] * 1.4426950408889634f;
    }
    if (row_ok[b]) {
      const uint16_t* qp = static_cast<const uint16_t*>(p.q) +
                           (static_cast<int64_t>(q_row0 + pos[b]) * H + kvh * g + hh[b]) * kHeadDim + c * 8;
#pragma unroll
      for (int s = 0; s < 8; ++s) qreg[b][s] = *reinterpret_cast<const u32x4_t*>(qp + 16 * s);
    } else {
#pragma unroll
      for (int s = 0; s < 8; ++s) qreg[b][s] = u32x4_t{0u, 0u, 0u, 0u};
    }
  }
  u32x4_t qlo[ROPE ? kRowBlocks : 1][8];  // remainders of the rotated queries
  if constexpr (ROPE) {
#pragma unroll
    for (int b = 0; b < kRowBlocks; ++b) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {  // blocks s and s + 4 hold the two components of pairs d = 16 s + 8 c .. + 8
        float cs[8], sn[8], xr[8], yr[8];
        rope_angles(diag0 + pos[b], 16 * s + 8 * c, cs, sn);  // the row's absolute position (causal plans only)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float xe = elem16<BF>(qreg[b][s][e >> 1], e & 1), ye = elem16<BF>(qreg[b][s + 4][e >> 1], e & 1);
          xr[e] = xe * cs[e] - ye * sn[e];
          yr[e] = ye * cs[e] + xe * sn[e];
        }
        split_head_remainder<BF>(xr, &qreg[b][s], &qlo[b][s]);
        split_head_remainder<BF>(yr, &qreg[b][s + 4], &qlo[b][s + 4]);
      }
    }
  }
  // wave-uniform bounds of lim per block (rows are position-major)
  int blk_lim_lo[kRowBlocks], blk_lim_hi[kRowBlocks];
#pragma unroll
  for (int b = 0; b < kRowBlocks; ++b) {
    const int r0 = kWaveRows * wave + 32 * b;
    blk_lim_lo[b] = causal ? diag0 + (r0 >> g_log2) - kv_start : 0x3FFFFFFF;
    blk_lim_hi[b] = causal ? diag0 + ((r0 + 31) >> g_log2) - kv_start : 0x3FFFFFFF;
  }

  f32x16_t acc[kRowBlocks][4];  // acc[b][db][r] = O^T[d = 32 db + 8 (r / 4) + 4 c + r % 4][row n of block b]
#pragma unroll
  for (int b = 0; b < kRowBlocks; ++b)
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[b][db][r] = 0.f;
  float m_run[kRowBlocks], neg_ms[kRowBlocks], l_run[kRowBlocks];
#pragma unroll
  for (int b = 0; b < kRowBlocks; ++b) {
    m_run[b] = NEG_INF;  // reference of the exponentials, raw-logit units (-inf: none yet)
    neg_ms[b] = 0.f;     // -reference * scale_log2 (0 while there is none)
    l_run[b] = 0.f;      // this lane's share of the row sum
  }

  // Two staging register sets: set t % 2 carries tile t from its loads to its LDS store, so two
  // tiles are in flight while a third is being consumed.
  u32x4_t stage_k[2][2], stage_v[2][2];
  // Page ids are fetched one tile ahead of the data they address (lane r holds page r of the
  // tile), so that the data loads never wait behind an index load.
  // (page size 16: lane r holds page r of the tile; other page sizes: every thread holds the pages of its own
  // two staging rows, in the low and the high half)
  // (contiguous KV, kv_indices == null: page j of the chunk is page kv_page0 + j of the pool)
  const bool contig = p.kv_indices == nullptr;
  auto fetch_page_ids = [&](int t) -> int64_t {
    if (ps_log2 != 4) {
      const int pa = min((kTileKv * t + st_tok) >> ps_log2, n_pages - 1);
      const int pb = min((kTileKv * t + 32 + st_tok) >> ps_log2, n_pages - 1);
      const uint32_t ia = static_cast<uint32_t>(contig ? kv_page0 + pa : p.kv_indices[kv_page0 + pa]);
      const uint32_t ib = static_cast<uint32_t>(contig ? kv_page0 + pb : p.kv_indices[kv_page0 + pb]);
      return static_cast<int64_t>(ia | (static_cast<uint64_t>(ib) << 32));
    }
    int pi = 4 * t + (lane & 3);
    pi = pi < n_pages ? pi : n_pages - 1;  // never index past the chunk's pages
    return contig ? kv_page0 + pi : p.kv_indices[kv_page0 + pi];
  };
  auto fetch_tile = [&](auto set_c, int64_t ids) {
    constexpr int SET = decltype(set_c)::value;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      if (ps_log2 != 4) {  // CTA-uniform
        const int64_t pg = static_cast<int32_t>(r == 0 ? ids : (ids >> 32));
        const int slot = (32 * r + st_tok) & ((1 << ps_log2) - 1);  // a tile starts on a page boundary
        const int64_t off = pg * p.stride_page + kvh * p.stride_head + slot * p.stride_tok + st_chunk * 8;
        stage_k[SET][r] = *reinterpret_cast<const u32x4_t*>(kpool + off);
        stage_v[SET][r] = *reinterpret_cast<const u32x4_t*>(vpool + off);
      } else {
        const int pg = __builtin_amdgcn_readlane(static_cast<int>(ids), 2 * r + st_page);
        const int64_t page_off = pg * p.stride_page + kvh * p.stride_head;  // wave-uniform
        stage_k[SET][r] = *reinterpret_cast<const u32x4_t*>(kpool + page_off + st_off);
        stage_v[SET][r] = *reinterpret_cast<const u32x4_t*>(vpool + page_off + st_off);
      }
    }
  };
  auto store_tile = [&](auto set_c, int t) {
    constexpr int SET = decltype(set_c)::value;
    uint16_t* dk = lds_k + (t & 1) * (kTileKv * kRowElems);
    uint16_t* dv = lds_v + (t & 1) * (kTileKv * kRowElemsV);
    if constexpr (BF) {
#pragma unroll
      for (int r = 0; r < 2; ++r)
        stage_v[SET][r] = u32x4_t{bf16x2_to_f16x2(stage_v[SET][r][0]), bf16x2_to_f16x2(stage_v[SET][r][1]),
                                  bf16x2_to_f16x2(stage_v[SET][r][2]), bf16x2_to_f16x2(stage_v[SET][r][3])};
    }
    if (kTileKv * (t + 1) > kv_len) {  // CTA-uniform: only the chunk's last tile has rows past its end
#pragma unroll
      for (int r = 0; r < 2; ++r)
        if (kTileKv * t + 32 * r + st_tok >= kv_len) stage_v[SET][r] = u32x4_t{0u, 0u, 0u, 0u};  // must not reach P.V
    }
    if constexpr (ROPE) {
      uint16_t* dk_lo = reinterpret_cast<uint16_t*>(lds_raw + ((t & 1) ? kLdsKLo1 : kLdsKLo0));
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        // this thread holds components 8 (st_chunk % 8) .. + 8 of the token's first (st_chunk < 8) or second half;
        // lane ^ 8 holds the other half of the same pairs
        u32x4_t other;
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) other[wd] = __shfl_xor(stage_k[SET][r][wd], 8);
        float cs[8], sn[8], out[8];
        rope_angles(kv_start + kTileKv * t + 32 * r + st_tok, 8 * (st_chunk & 7), cs, sn);
        const bool second = st_chunk >= 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float mine = elem16<BF>(stage_k[SET][r][e >> 1], e & 1), oth = elem16<BF>(other[e >> 1], e & 1);
          out[e] = second ? mine * cs[e] + oth * sn[e] : mine * cs[e] - oth * sn[e];
        }
        u32x4_t head, rem;
        split_head_remainder<BF>(out, &head, &rem);
        stage_k[SET][r] = head;
        *reinterpret_cast<u32x4_t*>(&dk_lo[st_lds_k + 32 * r * kRowElems]) = rem;
      }
    }
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      *reinterpret_cast<u32x4_t*>(&dk[st_lds_k + 32 * r * kRowElems]) = stage_k[SET][r];
      *reinterpret_cast<u32x4_t*>(&dv[st_lds_v + 32 * r * kRowElemsV]) = stage_v[SET][r];
    }
  };
  using set0_t = std::integral_constant<int, 0>;
  using set1_t = std::integral_constant<int, 1>;

  // Pipeline: while tile t is consumed from LDS buffer t % 2, tiles t + 1 and t + 2 are in the
  // staging registers (loads issued two tiles ahead); after the products of tile t have been
  // issued tile t + 1 is written to buffer (t + 1) % 2, its register set is reloaded with tile
  // t + 3, and one CTA barrier closes the tile.
  __syncthreads();   // the previous work item's last tile is no longer being read
  // One tile: consume tile t, then hand tile t + 1 over from staging set SET = (t + 1) % 2.  The
  // tile loop below is unrolled by two so that SET is a compile-time constant.
  auto do_tile = [&](auto set_c, int t, int64_t& ids_load, const int64_t& ids_use) {
    const uint16_t* tk = lds_k + (t & 1) * (kTileKv * kRowElems);
    const uint16_t* tv = lds_v + (t & 1) * (kTileKv * kRowElemsV);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int tok_base = kTileKv * t + 32 * u;  // chunk-local index of this 32-token step
      if (tok_base >= kv_len || tok_base > blk_lim_hi[kRowBlocks - 1]) continue;  // nothing visible to this wavefront
      // ---- S^T = K . Q^T: all eight A operands are requested before the first product ----
      u32x4_t ka[8];
      {
        const uint16_t* krow = &tk[(32 * u + n) * kRowElems + c * 8];
#pragma unroll
        for (int s = 0; s < 8; ++s) ka[s] = *reinterpret_cast<const u32x4_t*>(krow + 16 * s);
      }
      f32x16_t sacc[kRowBlocks];
#pragma unroll
      for (int b = 0; b < kRowBlocks; ++b) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[b][r] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) sacc[b] = mfma_qk<BF>(ka[s], qreg[b][s], sacc[b]);
      }
      if constexpr (ROPE) {  // + remainder x head + head x remainder
        const uint16_t* tk_lo = reinterpret_cast<const uint16_t*>(lds_raw + ((t & 1) ? kLdsKLo1 : kLdsKLo0));
        const uint16_t* krow_lo = &tk_lo[(32 * u + n) * kRowElems + c * 8];
        u32x4_t ka_lo[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) ka_lo[s] = *reinterpret_cast<const u32x4_t*>(krow_lo + 16 * s);
#pragma unroll
        for (int b = 0; b < kRowBlocks; ++b)
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            sacc[b] = mfma_qk<BF>(ka_lo[s], qreg[b][s], sacc[b]);
            sacc[b] = mfma_qk<BF>(ka[s], qlo[b][s], sacc[b]);
          }
      }
      // lane (n, c) now holds S^T[token 8 (r / 4) + 4 c + r % 4][row n of block b], r = 0..15

      // ---- V^T operands: requested now, they arrive while the softmax runs on the vector ALU.
      //      Operand (db, j) = columns d = 32 db + (lane % 32), token slots e = 0..7 <->
      //      tokens 16 j + 8 (e / 4) + 4 c + e % 4 (the order P^T has in the S^T registers) ----
      u32x4_t vt[4][2];
      {
        const uint16_t* vsrc = &tv[(32 * u + 4 * c + tr_row) * kRowElemsV + tr_col];
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const u32x2_t lo = lds_read_tr16(vsrc + (16 * j) * kRowElemsV + 32 * db);
            const u32x2_t hi = lds_read_tr16(vsrc + (16 * j + 8) * kRowElemsV + 32 * db);
            vt[db][j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
          }
      }

#pragma unroll
      for (int b = 0; b < kRowBlocks; ++b) {
        if (tok_base > blk_lim_hi[b]) continue;  // block wholly above the diagonal (wave-uniform)
        // ---- online softmax on the 16 logits of its row this lane owns ----
        float sv[16];  // raw logits q.k; the softmax scale is folded into the exponent below
#pragma unroll
        for (int r = 0; r < 16; ++r) sv[r] = sacc[b][r];
        // the factor that turns sv into the exponent's units: the variants leave sv in log2 units already
        const float to_log2 = VAR ? 1.0f : p.scale_log2;
        if constexpr (VAR) {
          const float cap = p.soft_cap;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int dist = tok_base + 8 * (r >> 2) + 4 * c + (r & 3) - lim[b];  // t - pos (chunk-local on both sides)
            float s = sv[r] * p.scale_log2;
            if (cap > 0.f) {  // cap * tanh(s / cap), s in log2 units: tanh(x) = 1 - 2 / (1 + exp(2 x))
              const float e2x = __builtin_amdgcn_exp2f(s * (2.0f / cap));
              s = cap * 1.4426950408889634f * (1.0f - 2.0f / (1.0f + e2x));
            }
            s += slope_log2[b] * static_cast<float>(dist);
            if (p.window_left >= 0 && dist < -p.window_left) s = NEG_INF;
            sv[r] = s;
          }
        }
        const bool need_mask = (tok_base + 32 > kv_len) || (tok_base + 31 > blk_lim_lo[b]);
        if (need_mask) {
          const int cap = min(lim[b], kv_len - 1);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int tkn = tok_base + 8 * (r >> 2) + 4 * c + (r & 3);
            sv[r] = (tkn <= cap) ? sv[r] : NEG_INF;
          }
        }
        // Optimistic softmax: exponentiate against the current reference first, and only if
        // some P came out above 2^kLazyLog2 (or the row has no reference yet) find the row
        // maximum, raise the reference, rescale, and redo the exponentials.  The reference
        // only has to keep P inside fp16 range; o = O / l does not depend on it.  The common
        // step therefore has no max reduction, no cross-lane exchange and no rescale.
        f16x2_t h[8];
        auto exponentiate = [&]() {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[2 * j], to_log2, neg_ms[b]));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[2 * j + 1], to_log2, neg_ms[b]));
            h[j] = __builtin_convertvector(f32x2_t{p0, p1}, f16x2_t);  // one v_cvt_pk_f16_f32
          }
        };
        exponentiate();
        // P >= 0, so fp16 order is unsigned-integer order on the bit patterns (inf included)
        u16x2_t hmax = __builtin_bit_cast(u16x2_t, h[0]);
#pragma unroll
        for (int j = 1; j < 8; ++j) hmax = __builtin_elementwise_max(hmax, __builtin_bit_cast(u16x2_t, h[j]));
        const bool redo = hmax[0] > kLazyF16Bits || hmax[1] > kLazyF16Bits || m_run[b] == NEG_INF;
        if (__builtin_amdgcn_ballot_w64(redo) != 0) {
          float tmax = sv[0];
#pragma unroll
          for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sv[r]);
          tmax = halves_max(tmax);
          const float m_new = fmaxf(m_run[b], tmax);
          const float m_use = (m_new == NEG_INF) ? 0.f : m_new;  // row has seen nothing yet
          const float alpha = __builtin_amdgcn_exp2f((m_run[b] - m_use) * to_log2);
          m_run[b] = m_new;
          neg_ms[b] = -m_use * to_log2;
          l_run[b] *= alpha;
#pragma unroll
          for (int db = 0; db < 4; ++db) acc[b][db] *= alpha;
          exponentiate();
        }
        // The row sum is taken over the fp16-rounded P that the second product consumes
        // (v_dot2_f32_f16 with a vector of ones, fp32 accumulation): o = O / l is then an exact
        // convex combination of V rows whatever the reference, and a single dominant key
        // returns its V row exactly.
        const f16x2_t ones = {static_cast<_Float16>(1.0f), static_cast<_Float16>(1.0f)};
        float l = l_run[b];
#pragma unroll
        for (int j = 0; j < 8; ++j) l = __builtin_amdgcn_fdot2(h[j], ones, l, false);
        l_run[b] = l;
        const u32x4_t pb0 = {__builtin_bit_cast(uint32_t, h[0]), __builtin_bit_cast(uint32_t, h[1]),
                             __builtin_bit_cast(uint32_t, h[2]), __builtin_bit_cast(uint32_t, h[3])};
        const u32x4_t pb1 = {__builtin_bit_cast(uint32_t, h[4]), __builtin_bit_cast(uint32_t, h[5]),
                             __builtin_bit_cast(uint32_t, h[6]), __builtin_bit_cast(uint32_t, h[7])};
        // ---- O^T += V^T . P^T ----
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          acc[b][db] = mfma_pv(vt[db][0], pb0, acc[b][db]);
          acc[b][db] = mfma_pv(vt[db][1], pb1, acc[b][db]);
        }
      }
    }
    // Hand the next tile over and reload its register set with the tile three ahead.  Every
    // iteration issues the same loads in the same order (tiles past the end re-read the last
    // page and are never stored), so the counted waits for the oldest loads leave the younger
    // ones in flight; the index load goes first so that its consumer, one iteration later,
    // does not wait for the data loads issued after it.
    ids_load = fetch_page_ids(t + 4);
    if (t + 1 < n_tiles) store_tile(set_c, t + 1);
    fetch_tile(set_c, ids_use);
    __syncthreads();  // tile t + 1 is visible; nobody reads tile t any more
  };
  if (n_tiles > 0) {  // one region, so that the loop is entered with this work item's Q loads known complete
    const int64_t ids0 = fetch_page_ids(0), ids1 = fetch_page_ids(1);
    int64_t ids_even = fetch_page_ids(2), ids_odd = fetch_page_ids(3);  // ids of the next even / odd tile to request
    fetch_tile(set0_t{}, ids0);
    fetch_tile(set1_t{}, ids1);
    store_tile(set0_t{}, 0);
    fetch_tile(set0_t{}, ids_even);
    __syncthreads();
    // A single-exit loop: with an odd tile count the last call finds no visible step and stores
    // nothing, which is cheaper than a second exit that would make every counted wait assume
    // the emptiest pipeline.
    for (int t = 0; t < n_tiles; t += 2) {
      do_tile(set1_t{}, t, ids_even, ids_odd);
      do_tile(set0_t{}, t + 1, ids_odd, ids_even);
    }
  }

  // ---- epilogue: o = O / l, lse = ln(sum exp) (Sec. 2.2) ----
#pragma unroll
  for (int b = 0; b < kRowBlocks; ++b) {
    const float l = halves_sum(l_run[b]);
    const bool live = l > 0.f;
    const float inv = live ? 1.0f / l : 0.f;
    const float lse_val =
        live ? (m_run[b] * (VAR ? 1.0f : p.scale_log2) + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : NEG_INF;
    if (row_ok[b]) {
      const int head = kvh * g + hh[b];
      const int64_t final_row = static_cast<int64_t>(q_row0 + pos[b]) * H + head;
      float* dst_o;
      float* dst_lse;
      if (out_slot < 0) {  // write-through (App. D.2)
        dst_o = p.o + final_row * kHeadDim;
        dst_lse = p.lse + final_row;
      } else {
        const int64_t row = (static_cast<int64_t>(out_slot) * p.t_pos + pos[b]) * H + head;
        dst_o = p.part_o + row * kHeadDim;
        dst_lse = p.part_lse + row;
      }
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int d0 = 32 * db + 8 * q + 4 * c;
          const f32x4_t v = {acc[b][db][4 * q] * inv, acc[b][db][4 * q + 1] * inv, acc[b][db][4 * q + 2] * inv,
                             acc[b][db][4 * q + 3] * inv};
          if (out_slot >= 0 || p.o != nullptr) *reinterpret_cast<f32x4_t*>(dst_o + d0) = v;
          if (out_slot < 0 && p.o_cast != nullptr) {
            uint16_t* dc = static_cast<uint16_t*>(p.o_cast) + final_row * kHeadDim + d0;
            *reinterpret_cast<u32x2_t*>(dc) = u32x2_t{pack_out<BF>(v[0], v[1]), pack_out<BF>(v[2], v[3])};
          }
        }
      if (c == 0) *dst_lse = lse_val;
    }
  }
}

// VAR: the logits hooks of RunParams are applied.  CAPLOOP (with VAR): the only hook in use is the soft cap, which
// the scheduled loop has a variant for; the other hooks run every item on the generic path.
// CONTIG: contiguous KV (kv_indices == null); the scheduled loop then computes its page ids.
// VARLOOP (with VAR): the hooks in use are the ALiBi bias and / or the sliding window, without the soft cap: the
// scheduled loop has a variant for them too.
// ROPE (with VAR, no loop variant): every item on the general path, queries and keys rotated by their positions.
struct NoRopeTable {};
template <bool BF, bool VAR = false, bool CAPLOOP = false, bool CONTIG = false, bool VARLOOP = false, bool ROPE = false,
          bool PSLOOP = false, bool ROWLOOP = false>
__global__ void __launch_bounds__(kCtaThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
append_kernel(const RunParams p_arg, const typename std::conditional<ROPE, RopeTable, NoRopeTable>::type rope) {
  static_assert(!CONTIG || !VAR, "affine addressing is built for the plain kernel");
  static_assert(!(CAPLOOP && VARLOOP) && (!VARLOOP || VAR), "one variant of the loop per instantiation");
  static_assert(!ROPE || (VAR && !CAPLOOP && !VARLOOP), "the rotary transform is built into the general path");
  static_assert(!PSLOOP || !VAR, "the loop for other page sizes is the plain one, with or without a page table");
  static_assert(!ROWLOOP || PSLOOP, "the per-row loop is a kind of the loop for other page sizes");
  const int tid = threadIdx.x;
  // The launch parameters are read from the argument segment again for every work item (scalar loads): the scheduled
  // loop takes every scalar register above s63, and parameters kept in registers across it would be spilled into
  // lanes of a vector register that is itself saved to scratch memory, whose reload after the loop would wait for the
  // output rows the item has just stored.
  typedef const __attribute__((address_space(4))) RunParams KernargParams;
  const uint64_t params_addr = reinterpret_cast<uint64_t>(__builtin_amdgcn_kernarg_segment_ptr());  // p_arg is the first argument
  KernargParams& p = *reinterpret_cast<KernargParams*>(params_addr);
  if constexpr (ROPE) {
    if (tid < 64) {
      rope_tab_lds[tid] = rope.rev[tid];
      rope_tab_lds[64 + tid] = rope.rev256[tid];
    }
    __syncthreads();
  }
  // Workgroups are handed to the eight XCDs round-robin: with the kv head as the fast index all
  // CTAs of a kv head (which re-read the same K/V) share one XCD's L2 when num_kv_heads is 8.
  const int cta = static_cast<int>(blockIdx.x) / p.num_kv_heads;
  const int w_begin = __builtin_amdgcn_readfirstlane(p.cta_indptr[cta]);
  const int w_end = __builtin_amdgcn_readfirstlane(p.cta_indptr[cta + 1]);

  // The plan entry of a work item is read while the item before it runs (by the scheduled loop's block, or
  // here); `prefetched`: that block has also requested this item's first tiles into LDS.
  WorkItem item;
  if (w_begin < w_end) item.load(p, w_begin);
  int prefetched = 0;
  // (opaque copy of the parameters' address: the parameter loads of a work item stay inside the loop)
#define FI355_ITEM_SCALARS                                                                                      \
  uint64_t params_again = params_addr;                                                                          \
  asm volatile("" : "+s"(params_again));                                                                         \
  KernargParams& p = *reinterpret_cast<KernargParams*>(params_again);                                            \
  const int kvh = static_cast<int>(blockIdx.x) % p.num_kv_heads;                                                 \
  const int g = p.group;                                                                                         \
  const int g_log2 = 31 - __builtin_clz(g);                                                                      \
  const int H = p.num_qo_heads;                                                                                  \
  const int q_row0 = item.q_row0, n_pos = item.n_pos, kv_page0 = item.kv_page0, kv_start = item.kv_start;        \
  const int kv_len = item.kv_len, diag0 = item.diag0, out_slot = item.out_slot;                                  \
  const bool causal = diag0 != kNoDiagMarker;
  const int wave_s = __builtin_amdgcn_readfirstlane(tid >> 6);
  // ALiBi slope of this lane's row (its head depends on the thread alone), times log2(e): one load per launch
  float slope_o = 0.f;
  if constexpr (VARLOOP) {
    if (p.alibi_slopes != nullptr) {
      const int R = 32 * (tid >> 6) + (tid & 31);
      const int head = (static_cast<int>(blockIdx.x) % p.num_kv_heads) * p.group + (R & (p.group - 1));
      slope_o = p.alibi_slopes[head] * 1.4426950408889634f;
    }
  }
  int w = w_begin;
  while (w < w_end) {
    // ---- work items whose first tile every row of the CTA sees in full: the scheduled loop, one item after the
    // other in a loop of their own (the general path below is a function call, after which the compiler must
    // assume loads in flight into any register: at a common loop head it would wait for all of memory before
    // every item, which is where the rows that the item before has just stored are still on their way) ----
    if constexpr (kUseScheduledLoop && (!VAR || CAPLOOP || VARLOOP)) {
     for (;;) {
      FI355_ITEM_SCALARS
      (void)g;
      int vis = kv_len;  // tokens visible to the CTA's first position, which sees the fewest
      if (causal) vis = min(vis, max(0, diag0 - kv_start + 1));
      const int n_full = __builtin_amdgcn_readfirstlane(vis / kTileKv);
      const int64_t page_bytes = p.stride_page * 2;
      // (the loop addresses its outputs with 32-bit byte offsets)
      const int64_t out_rows_bound = (out_slot < 0 ? static_cast<int64_t>(q_row0) + p.t_pos : (static_cast<int64_t>(out_slot) + 1) * p.t_pos) * H;
      // (PSLOOP: page sizes 4, 8, 32: a wavefront's four consecutive rows per load lie in one page, and the two
      // 32-token halves of a tile in different pages or in the two halves of one;
      // ROWLOOP: page sizes 1 and 2: a page id per token row, 64-bit addresses per lane)
      if ((ROWLOOP  ? p.page_log2 <= 1
           : PSLOOP ? (p.page_log2 == 2 || p.page_log2 == 3 || p.page_log2 == 5)
                    : p.page_log2 == 4) &&
          n_full >= 1 && kv_len >= kLoopMinTokens && page_bytes > 0 && page_bytes < (int64_t(1) << 32) &&
          (!VARLOOP || H < 65536) &&  // (that variant takes num_qo_heads in 16 bits of an operand)
          out_rows_bound * (kHeadDim * 4) < (int64_t(1) << 32)) {
        // The loop clobbers nearly every vector register, so its lane-dependent operands are
        // derived here from a thread index that is formed anew for every item (wavefront index,
        // a scalar, and the lane's number): the compiler can neither hoist them out of the work loop
        // nor keep the index itself in scratch memory across the loop, whose reload would wait for
        // the rows that the item before has just stored.
        int lane_o;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_o));
        const int tid_o = wave_s * 64 + lane_o;
        const int wave_o = tid_o >> 6, n_o = tid_o & 31, c_o = (tid_o >> 5) & 1;
        const int st_tok_o = tid_o >> 4, st_chunk_o = tid_o & 15;
        const int tr_row_o = (tid_o & 15) >> 2, tr_col_o = 16 * ((tid_o >> 4) & 1) + 4 * (tid_o & 3);
        const int R = 32 * wave_o + n_o;
        const int pos_r = R >> g_log2;
        const int head = kvh * g + (R & (g - 1));
        const int pos_c = min(pos_r, n_pos - 1);  // rows past the tile's end compute on a valid row; never stored
        const uint64_t q_addr = reinterpret_cast<uint64_t>(static_cast<const uint16_t*>(p.q) +
                                (static_cast<int64_t>(q_row0 + pos_c) * H + head) * kHeadDim + c_o * 8);
        const uint64_t k_base = reinterpret_cast<uint64_t>(static_cast<const uint16_t*>(p.k_pool) + kvh * p.stride_head);
        const uint64_t v_base = reinterpret_cast<uint64_t>(static_cast<const uint16_t*>(p.v_pool) + kvh * p.stride_head);
        const uint64_t all_ids = reinterpret_cast<uint64_t>(p.kv_indices);
        const uint32_t lds0 = lds_offset(lds_raw);
        const int chunk_pages = PSLOOP ? (kv_len + (1 << p.page_log2) - 1) >> p.page_log2 : (kv_len + kPageSize - 1) / kPageSize;
        const int row_in_page = PSLOOP ? st_tok_o & (min(1 << p.page_log2, 32) - 1) : st_tok_o & 15;
        const int last_seen = causal ? min(diag0 + pos_r - kv_start, kv_len - 1) : kv_len - 1;
        // where the rows go: the final output (write-through, App. D.2) or this item's partial slot
        const bool final_out = out_slot < 0;
        const int64_t out_row = (final_out ? static_cast<int64_t>(q_row0 + pos_r)
                                           : static_cast<int64_t>(out_slot) * p.t_pos + pos_r) * H + head;
        const uint32_t st_off_bytes = static_cast<uint32_t>(row_in_page * p.stride_tok + st_chunk_o * 8) * 2;
        // K goes straight to LDS in packed 256-byte rows whose 16-byte chunks are XOR-swizzled by the
        // row index (conflict-free operand reads without padding): LDS slot st_chunk of row st_tok
        // holds chunk st_chunk ^ (st_tok % 16) of that token
        const uint32_t k_off_bytes =
            static_cast<uint32_t>(row_in_page * p.stride_tok + ((st_chunk_o ^ st_tok_o) & 15) * 8) * 2;
        const uint32_t epi0 = lds0 + kEpilogueBase + wave_o * kEpilogueLdsBytes;
        WorkItem next;
        int prefetched_next;
        __syncthreads();  // the previous work item is done with the tile buffers and the transpose area
        // (with the bias / window variant the loop caps the bound itself and also needs it uncapped)
        const int seen_bound = VARLOOP ? diag0 + pos_r - kv_start : last_seen;
        run_scheduled_loop<BF, CAPLOOP, CONTIG, VARLOOP, PSLOOP, ROWLOOP>(n_full, (kv_len + kTileKv - 1) / kTileKv, kv_len, seen_bound - 4 * c_o, tid_o,
                               (chunk_pages - 1) * 4, p.kv_indices + kv_page0, static_cast<uint32_t>(k_base),
                               static_cast<uint32_t>(k_base >> 32), static_cast<uint32_t>(v_base),
                               static_cast<uint32_t>(v_base >> 32), static_cast<uint32_t>(page_bytes),
                               CAPLOOP ? p.cap_k1 : p.scale_log2,
                               q_addr, st_off_bytes, k_off_bytes,
                               lds0 + n_o * 256 + ((c_o ^ n_o) & 1) * 16,
                               lds0 + kLdsVOffset + (4 * c_o + tr_row_o) * (kRowElemsV * 2) + tr_col_o * 2,
                               lds0 + __builtin_amdgcn_readfirstlane(wave_o) * 1024,
                               lds0 + kLdsVOffset + st_tok_o * (kRowElemsV * 2) + st_chunk_o * 16,
                               static_cast<uint32_t>(out_row * (kHeadDim * 4) + c_o * 16),
                               final_out ? p.o : p.part_o,
                               final_out ? p.lse : p.part_lse, p.o_cast,
                               __builtin_amdgcn_readfirstlane(final_out && p.o_cast != nullptr ? (p.o != nullptr ? 1 : 2) : 0),
                               epi0 + n_o * kEpilogueRowBytes + c_o * 16,
                               epi0 + ((tid_o >> 4) & 3) * kEpilogueRowBytes + st_chunk_o * 16,
                               CAPLOOP   ? g_log2 | (__builtin_amdgcn_readfirstlane(wave_o) << 8)
                               : VARLOOP ? g_log2 | (n_pos << 5) | (H << 16)
                               : PSLOOP  ? g_log2 | (p.page_log2 << 8)
                                         : g_log2,
                               H,
                               static_cast<int>((final_out ? static_cast<int64_t>(q_row0)
                                                           : static_cast<int64_t>(out_slot) * p.t_pos) * H + kvh * g),
                               n_pos,
                               CAPLOOP ? __builtin_bit_cast(int, p.cap_a) : __builtin_amdgcn_readfirstlane(wave_o),
                               __builtin_amdgcn_readfirstlane(min(w + 1, w_end - 1) * 4 + (w + 1 < w_end ? 1 : 0) + 2 * prefetched), p.w_q_row0,
                               static_cast<int>((p.w_n_pos - p.w_q_row0) * static_cast<int64_t>(sizeof(int32_t))),
                               CONTIG ? static_cast<uint32_t>(kv_page0) : static_cast<uint32_t>(all_ids),
                               static_cast<uint32_t>(all_ids >> 32), next, prefetched_next, slope_o,
                               p.window_left >= 0 ? p.window_left : 0x3FFFFFFF);
        item = next;
        prefetched = prefetched_next;
        if (++w >= w_end) return;  // (the same for every thread of the CTA)
        continue;                  // the work item is finished
      }
      break;
     }
    }
    FI355_ITEM_SCALARS
    (void)kvh; (void)g; (void)g_log2; (void)H; (void)causal;
    if (prefetched) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // tiles requested for this item: not used, but on their way into LDS
    prefetched = 0;
    __syncthreads();  // the previous work item is done with the tile buffers
    // (the kernel's only argument sits at the start of its argument segment)
    generic_work_item<BF, VAR, ROPE>(params_addr, q_row0, n_pos,
                                     kv_page0, kv_start, kv_len, diag0, out_slot);
    if (w + 1 < w_end) item.load(p, w + 1);
    ++w;
  }
#undef FI355_ITEM_SCALARS
}

}  // namespace

int append_tile_rows() { return (kCtaThreads / 64) * 32 * kRowBlocks; }

hipError_t launch_append(const RunParams& p, bool is_bf16, bool variant, const RopeTable* rope, hipStream_t stream) {
  const dim3 grid(static_cast<unsigned>(p.ctas_per_head) * static_cast<unsigned>(p.num_kv_heads), 1, 1);
  const dim3 block(kCtaThreads, 1, 1);
  if (rope) {  // (variant launches only) every item on the general path, with the other hooks on top
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, true, false, false, false, true>), grid, block, 0, stream, p, *rope);
    else
      hipLaunchKernelGGL((append_kernel<false, true, false, false, false, true>), grid, block, 0, stream, p, *rope);
    return hipGetLastError();
  }
  if (variant && p.soft_cap > 0.f && p.alibi_slopes == nullptr && p.window_left < 0) {
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, true, true>), grid, block, 0, stream, p, NoRopeTable{});
    else
      hipLaunchKernelGGL((append_kernel<false, true, true>), grid, block, 0, stream, p, NoRopeTable{});
    return hipGetLastError();
  }
  if (variant && p.soft_cap == 0.f) {  // bias and / or window: their variant of the scheduled loop
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, true, false, false, true>), grid, block, 0, stream, p, NoRopeTable{});
    else
      hipLaunchKernelGGL((append_kernel<false, true, false, false, true>), grid, block, 0, stream, p, NoRopeTable{});
    return hipGetLastError();
  }
  if (variant) {  // the soft cap together with a bias or a window: every item on the general path
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, true>), grid, block, 0, stream, p, NoRopeTable{});
    else
      hipLaunchKernelGGL((append_kernel<false, true>), grid, block, 0, stream, p, NoRopeTable{});
    return hipGetLastError();
  }
  if (p.kv_indices == nullptr && p.page_log2 <= 1) {  // contiguous KV (the caller has refused variants), page sizes 1 and 2
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, false, false, true, false, false, true, true>), grid, block, 0, stream, p, NoRopeTable{});
    else
      hipLaunchKernelGGL((append_kernel<false, false, false, true, false, false, true, true>), grid, block, 0, stream, p, NoRopeTable{});
    return hipGetLastError();
  }
  if (p.kv_indices == nullptr && (p.page_log2 == 2 || p.page_log2 == 3 || p.page_log2 == 5)) {  // contiguous, page sizes 4, 8, 32
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, false, false, true, false, false, true>), grid, block, 0, stream, p, NoRopeTable{});
    else
      hipLaunchKernelGGL((append_kernel<false, false, false, true, false, false, true>), grid, block, 0, stream, p, NoRopeTable{});
    return hipGetLastError();
  }
  if (p.kv_indices != nullptr && p.page_log2 <= 1) {  // page sizes 1 and 2: the loop with a page id per token row
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, false, false, false, false, false, true, true>), grid, block, 0, stream, p, NoRopeTable{});
    else
      hipLaunchKernelGGL((append_kernel<false, false, false, false, false, false, true, true>), grid, block, 0, stream, p, NoRopeTable{});
    return hipGetLastError();
  }
  if (p.kv_indices != nullptr && (p.page_log2 == 2 || p.page_log2 == 3 || p.page_log2 == 5)) {  // their variant of the loop
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, false, false, false, false, false, true>), grid, block, 0, stream, p, NoRopeTable{});
    else
      hipLaunchKernelGGL((append_kernel<false, false, false, false, false, false, true>), grid, block, 0, stream, p, NoRopeTable{});
    return hipGetLastError();
  }
  if (p.kv_indices == nullptr) {  // contiguous KV (the caller has refused variants)
    if (is_bf16)
      hipLaunchKernelGGL((append_kernel<true, false, false, true>), grid, block, 0, stream, p, NoRopeTable{});
    else
      hipLaunchKernelGGL((append_kernel<false, false, false, true>), grid, block, 0, stream, p, NoRopeTable{});
    return hipGetLastError();
  }
  if (is_bf16)
    hipLaunchKernelGGL((append_kernel<true>), grid, block, 0, stream, p, NoRopeTable{});
  else
    hipLaunchKernelGGL((append_kernel<false>), grid, block, 0, stream, p, NoRopeTable{});
  return hipGetLastError();
}

}  // namespace fi355
