"""Seeded synthetic inputs for paged (block-sparse-row) attention.

This module only *draws and lays out* inputs: lengths, page tables, random
Q/K/V values rounded to the storage dtype.  It contains none of the method's
arithmetic (no softmax, no scheduling, no merging) so that both the CPU oracle
and the GPU library can be fed from it without sharing any logic.

Storage convention: 16-bit values are carried as ``numpy.uint16`` bit patterns
(``*_bits`` fields) so that fp16 and bf16 travel through NumPy unchanged;
``widen`` turns them into exact float64 values.  An 8-bit KV cache (App. F: fp8 K/V with
16-bit queries) carries ``numpy.uint8`` codes of the OCP E4M3 format, produced here by
``f32_to_e4m3_bits``; their values are ``code value * k_scale`` (``v_scale``).

Layouts (Sec. 3.1.1 of the paper: ragged query/output, BSR KV-cache):
  q_bits        [nnz_qo, H_qo, D]
  k_bits/v_bits [num_pages, H_kv, page_size, D]   (last dimension contiguous)
  qo_indptr     [B+1]   request i owns query rows qo_indptr[i]:qo_indptr[i+1]
  kv_indptr     [B+1]   request i owns kv_indices[kv_indptr[i]:kv_indptr[i+1]]
  kv_indices    [nnz_pages] page ids (BSR column indices, B_c = page_size)
  last_page_len [B]     valid tokens in the request's last page (1..page_size)
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor
from typing import Optional, Sequence

import numpy as np

F16 = "f16"
BF16 = "bf16"
FP8 = "fp8_e4m3"   # OCP 8-bit float: 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinities, 0x7f / 0xff = NaN
E4M3_NAN = np.uint8(0x7F)

_NAN_BITS = {F16: np.uint16(0x7E00), BF16: np.uint16(0x7FC0)}


# --------------------------------------------------------------------------
# 16-bit storage helpers (pure data conversion)
# --------------------------------------------------------------------------
def f32_to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the storage dtype (nearest-even), return bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        u = x.view(np.uint32)
        lsb = (u >> np.uint32(16)) & np.uint32(1)
        r = u + np.uint32(0x7FFF) + lsb
        out = (r >> np.uint32(16)).astype(np.uint16)
        nan = np.isnan(x)
        if nan.any():
            out[nan] = _NAN_BITS[BF16]
        return out
    raise ValueError(f"unknown dtype {dtype!r}")


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to E4M3 codes: nearest, ties to even, magnitudes above 448 saturate
    to 448 (the format has no infinity).  NaN inputs are not expected here."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    sign = np.signbit(x).astype(np.uint8) << np.uint8(7)
    a = np.minimum(np.abs(x).astype(np.float64), 448.0)
    _, ex = np.frexp(a)                     # a = f * 2**ex, f in [0.5, 1)
    e = np.maximum(ex - 1, -6)              # exponent of the binade; subnormals share the smallest one
    q = np.rint(a / np.exp2(e.astype(np.float64)) * 8.0).astype(np.int64)   # value in eighths of 2**e: 0..16
    # q = 16: rounded up into the next binade; q < 8: subnormal (only at e = -6)
    up = q == 16
    e = np.where(up, e + 1, e)
    q = np.where(up, 8, q)
    code = np.where(q < 8, q, ((e + 7) << 3) | (q - 8))
    return (code.astype(np.uint8) | sign).astype(np.uint8)


def widen(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of each stored 16-bit pattern."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# container
# --------------------------------------------------------------------------
@dataclasses.dataclass
class PagedBatch:
    name: str
    dtype: str
    num_qo_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    causal: bool
    sm_scale: float
    qo_indptr: np.ndarray      # int32 [B+1]
    kv_indptr: np.ndarray      # int32 [B+1]
    kv_indices: np.ndarray     # int32 [nnz_pages]
    last_page_len: np.ndarray  # int32 [B]
    q_bits: np.ndarray         # uint16 [nnz_qo, H_qo, D]
    k_bits: np.ndarray         # uint16 [P, H_kv, page_size, D]  (uint8 E4M3 codes when kv_dtype is FP8)
    v_bits: np.ndarray         # uint16 [P, H_kv, page_size, D]
    kv_dtype: str = ""         # "" = same as dtype; FP8 = 8-bit KV cache
    k_scale: float = 1.0       # value of a stored K element = decoded code * k_scale (FP8 only)
    v_scale: float = 1.0

    @property
    def batch(self) -> int:
        return len(self.last_page_len)

    @property
    def num_pages(self) -> int:
        return int(self.k_bits.shape[0])

    def qo_lens(self) -> np.ndarray:
        return np.diff(self.qo_indptr)

    def kv_lens(self) -> np.ndarray:
        n_pg = np.diff(self.kv_indptr).astype(np.int64)
        return np.where(n_pg > 0, (n_pg - 1) * self.page_size + self.last_page_len, 0)

    def kv_bytes(self) -> int:
        """K+V bytes of all tokens the batch attends to (each kv-head once)."""
        return int(self.kv_lens().sum()) * self.num_kv_heads * self.head_dim * 2 * (1 if self.kv_dtype == FP8 else 2)


def _fill_normal_bits(out: np.ndarray, seed_seq: np.random.SeedSequence, dtype: str,
                      scale: float, threads: int = 8, slab: int = 1 << 22) -> None:
    """out.flat[:] = bits(round(scale * N(0,1))), drawn slab by slab (dtype FP8: E4M3 codes).

    Every slab has its own child seed, so the result does not depend on the
    number of threads."""
    flat = out.reshape(-1)
    n = flat.size
    n_slabs = (n + slab - 1) // slab
    children = seed_seq.spawn(max(n_slabs, 1))

    def work(s: int) -> None:
        lo, hi = s * slab, min((s + 1) * slab, n)
        g = np.random.Generator(np.random.PCG64(children[s]))
        x = g.standard_normal(hi - lo, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        flat[lo:hi] = f32_to_e4m3_bits(x) if dtype == FP8 else f32_to_bits(x, dtype)

    if n_slabs <= 1 or threads <= 1:
        for s in range(n_slabs):
            work(s)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(n_slabs)))


def make_batch(name: str, seed: int, dtype: str, num_qo_heads: int, num_kv_heads: int,
               head_dim: int, page_size: int, qo_lens: Sequence[int], kv_lens: Sequence[int],
               causal: bool, *, num_pages: Optional[int] = None, value_scale: float = 1.0,
               permute_pages: bool = True, poison: bool = True,
               sm_scale: Optional[float] = None, kv_dtype: str = "", k_scale: float = 1.0,
               v_scale: float = 1.0) -> PagedBatch:
    """Build one paged batch: random page placement, N(0,1)*value_scale data.

    Pages are handed to requests as consecutive slices of one random
    permutation of the pool.  With ``poison`` every slot that no request may
    read (unused pages, slots past ``last_page_len``) holds NaN, so that a
    kernel reading out of range shows up as NaN in the output."""
    qo_lens = np.asarray(qo_lens, dtype=np.int64)
    kv_lens = np.asarray(kv_lens, dtype=np.int64)
    assert qo_lens.shape == kv_lens.shape and qo_lens.ndim == 1
    B = len(qo_lens)
    n_pg = (kv_lens + page_size - 1) // page_size
    need = int(n_pg.sum())
    P = need if num_pages is None else int(num_pages)
    assert P >= need, "pool too small"
    P = max(P, 1)

    root = np.random.SeedSequence(seed)
    s_perm, s_q, s_k, s_v = root.spawn(4)
    g = np.random.Generator(np.random.PCG64(s_perm))
    perm = g.permutation(P).astype(np.int32) if permute_pages else np.arange(P, dtype=np.int32)

    kv_indptr = np.zeros(B + 1, dtype=np.int32)
    kv_indptr[1:] = np.cumsum(n_pg)
    kv_indices = perm[:need].copy()
    last_page_len = np.where(n_pg > 0, kv_lens - (n_pg - 1) * page_size, 0).astype(np.int32)
    qo_indptr = np.zeros(B + 1, dtype=np.int32)
    qo_indptr[1:] = np.cumsum(qo_lens)
    nnz = int(qo_indptr[-1])

    q_bits = np.empty((nnz, num_qo_heads, head_dim), dtype=np.uint16)
    _fill_normal_bits(q_bits, s_q, dtype, value_scale)
    if kv_dtype == FP8:   # stored code = round(value / scale); the values themselves are scale * N(0,1) * value_scale
        k_bits = np.empty((P, num_kv_heads, page_size, head_dim), dtype=np.uint8)
        v_bits = np.empty((P, num_kv_heads, page_size, head_dim), dtype=np.uint8)
        _fill_normal_bits(k_bits, s_k, FP8, value_scale)
        _fill_normal_bits(v_bits, s_v, FP8, value_scale)
    else:
        assert kv_dtype in ("", dtype), "the KV cache is stored in the query type or in FP8"
        k_bits = np.empty((P, num_kv_heads, page_size, head_dim), dtype=np.uint16)
        v_bits = np.empty((P, num_kv_heads, page_size, head_dim), dtype=np.uint16)
        _fill_normal_bits(k_bits, s_k, dtype, value_scale)
        _fill_normal_bits(v_bits, s_v, dtype, value_scale)

    if poison:
        nanb = E4M3_NAN if kv_dtype == FP8 else _NAN_BITS[dtype]
        if P > need:
            unused = perm[need:]
            k_bits[unused] = nanb
            v_bits[unused] = nanb
        for i in range(B):
            if n_pg[i] > 0 and last_page_len[i] < page_size:
                pg = kv_indices[kv_indptr[i + 1] - 1]
                k_bits[pg, :, last_page_len[i]:, :] = nanb
                v_bits[pg, :, last_page_len[i]:, :] = nanb

    if sm_scale is None:
        sm_scale = 1.0 / math.sqrt(head_dim)
    return PagedBatch(name=name, dtype=dtype, num_qo_heads=num_qo_heads, num_kv_heads=num_kv_heads,
                      head_dim=head_dim, page_size=page_size, causal=causal, sm_scale=float(sm_scale),
                      qo_indptr=qo_indptr, kv_indptr=kv_indptr, kv_indices=kv_indices,
                      last_page_len=last_page_len, q_bits=q_bits, k_bits=k_bits, v_bits=v_bits,
                      kv_dtype=FP8 if kv_dtype == FP8 else "", k_scale=float(k_scale), v_scale=float(v_scale))


# --------------------------------------------------------------------------
# length distributions
# --------------------------------------------------------------------------
def zipf_lengths(g: np.random.Generator, n: int, lo: int, hi: int, s: float) -> np.ndarray:
    """n integers in [lo, hi] with P(k) proportional to k**-s (inverse-CDF sampling)."""
    ks = np.arange(lo, hi + 1, dtype=np.float64)
    cdf = np.cumsum(ks ** (-s))
    cdf /= cdf[-1]
    u = g.random(n)
    return (lo + np.searchsorted(cdf, u, side="left")).astype(np.int64)


# --------------------------------------------------------------------------
# the five benchmark configurations (full = as named; small = same structure,
# sizes an fp64 CPU oracle finishes in seconds)
# --------------------------------------------------------------------------
def config1(small: bool = False) -> PagedBatch:
    """MHA decode: batch 4, 8/8 heads, D 128, fp16, page 16, l_kv ~ U{64..512},
    256-page pool, random page permutation."""
    g = np.random.Generator(np.random.PCG64(1001))
    kv = g.integers(64, 513, size=4)
    return make_batch("c1_mha_decode", 1001, F16, 8, 8, 128, 16, [1] * 4, kv, causal=False, num_pages=256)


def config2(small: bool = False, permute_pages: bool = True, kv_dtype: str = "", page_size: int = 16) -> PagedBatch:
    """GQA decode (Llama-3-8B layer shape): batch 128, 32/8 heads, D 128, bf16,
    page 16, l_kv Zipf(s=1.2) over [256, 32768], request 0 forced to 32768.
    small: batch 12, range [64, 2048], request 0 forced to 2048."""
    g = np.random.Generator(np.random.PCG64(1002))
    if small:
        kv = zipf_lengths(g, 12, 64, 2048, 1.2)
        kv[0] = 2048
    else:
        kv = zipf_lengths(g, 128, 256, 32768, 1.2)
        kv[0] = 32768
    need = int(((kv + page_size - 1) // page_size).sum())
    return make_batch("c2_gqa_decode_zipf" + ("_small" if small else ""), 1002, BF16, 32, 8, 128, page_size,
                      [1] * len(kv), kv, causal=False, num_pages=need + need // 10,
                      poison=small, permute_pages=permute_pages, kv_dtype=kv_dtype,
                      k_scale=0.5 if kv_dtype == FP8 else 1.0, v_scale=2.0 if kv_dtype == FP8 else 1.0)


def config3(small: bool = False, permute_pages: bool = True, page_size: int = 16) -> PagedBatch:
    """Causal append/prefill: batch 16, GQA 32/8, D 128, bf16, page 16,
    l_qo ~ U{128..1024}, cached prefix ~ U{0..4096}, l_kv = prefix + l_qo.
    One request has prefix 0, one has l_qo not a multiple of 128.
    small: batch 4, l_qo ~ U{16..200}, prefix ~ U{0..300}."""
    g = np.random.Generator(np.random.PCG64(1003))
    if small:
        qo = g.integers(16, 201, size=4)
        pre = g.integers(0, 301, size=4)
    else:
        qo = g.integers(128, 1025, size=16)
        pre = g.integers(0, 4097, size=16)
    pre[1] = 0
    if qo[2] % 128 == 0:
        qo[2] += 37
    kv = qo + pre
    return make_batch("c3_causal_append" + ("_small" if small else ""), 1003, BF16, 32, 8, 128, page_size,
                      qo, kv, causal=True, permute_pages=permute_pages)


def config4(small: bool = False, permute_pages: bool = True, kv_dtype: str = "") -> PagedBatch:
    """Long-context decode with split-KV: batch 2, GQA 32/8, D 128, bf16,
    l_kv = [131072, 65536], values 0.5*N(0,1).  small: [8192, 4096]."""
    kv = [8192, 4096] if small else [131072, 65536]
    return make_batch("c4_long_decode" + ("_small" if small else ""), 1004, BF16, 32, 8, 128, 16,
                      [1, 1], kv, causal=False, value_scale=0.5, poison=small, permute_pages=permute_pages,
                      kv_dtype=kv_dtype, k_scale=0.5 if kv_dtype == FP8 else 1.0, v_scale=2.0 if kv_dtype == FP8 else 1.0)


def config_e2(kind: str, dist: str, constant_len: int = 1024) -> PagedBatch:
    """The paper's kernel experiment on input dynamism (Sec. 4.2): batch 16, sequence lengths constant (1024),
    uniform (512..1024) or skewed (Zipf, average about 1024); `kind` "decode": l_qo = 1, l_kv = the length;
    "prefill": causal, l_qo = l_kv = the length.  GQA 32/8, D 128, bf16, page 16 as in the other configurations.
    Zipf: P(l) proportional to l**-1.2 on [256, 3048], whose mean is 1024 (the paper gives only the average).
    `constant_len`: another length for the constant distribution (to see how a kernel's time splits into a part per
    work item and a part per KV tile)."""
    seed = 1100 + 10 * ("decode", "prefill").index(kind) + ("constant", "uniform", "zipf").index(dist)
    g = np.random.Generator(np.random.PCG64(seed))
    if dist == "constant":
        lens = np.full(16, constant_len, dtype=np.int64)
    elif dist == "uniform":
        lens = g.integers(512, 1025, size=16)
    else:
        lens = zipf_lengths(g, 16, 256, 3048, 1.2)
    qo = np.ones(16, dtype=np.int64) if kind == "decode" else lens
    name = f"e2_{kind}_{dist}" + (f"_len{constant_len}" if dist == "constant" and constant_len != 1024 else "")
    return make_batch(name, seed, BF16, 32, 8, 128, 16, qo, lens, causal=kind == "prefill", poison=False)


@dataclasses.dataclass
class SharedPrefixCase:
    """Composable-format decomposition (Sec. 3.1.2) of one decode step where all
    requests share a prefix: ``prefix`` is one row block holding every query
    against the prefix pages stored once; ``suffix`` is the per-request paged
    remainder; ``single`` is the same problem in one format (every request
    lists the prefix pages and then its own).  All three share q and the pools."""
    prefix: PagedBatch
    suffix: PagedBatch
    single: PagedBatch


def config5(small: bool = False) -> SharedPrefixCase:
    """64 requests share a 4096-token prefix; unique suffix ~ U{64..512} tokens
    (the current token included); one query token each; GQA 32/8, D 128, bf16.
    small: 8 requests, prefix 512, suffix ~ U{16..96}."""
    g = np.random.Generator(np.random.PCG64(1005))
    if small:
        n, prefix_len = 8, 512
        suf = g.integers(16, 97, size=n)
    else:
        n, prefix_len = 64, 4096
        suf = g.integers(64, 513, size=n)
    page = 16
    # lay out as n+1 "requests": the prefix first, then the suffixes
    base = make_batch("c5_pool", 1005, BF16, 32, 8, 128, page, [0] + [1] * n,
                      [prefix_len] + list(suf), causal=False)
    n_pre_pages = prefix_len // page
    pre_pages = base.kv_indices[:n_pre_pages]
    common = dict(dtype=base.dtype, num_qo_heads=32, num_kv_heads=8, head_dim=128, page_size=page,
                  causal=False, sm_scale=base.sm_scale, q_bits=base.q_bits, k_bits=base.k_bits,
                  v_bits=base.v_bits)
    tag = "_small" if small else ""
    prefix = PagedBatch(name="c5_prefix" + tag, qo_indptr=np.array([0, n], dtype=np.int32),
                        kv_indptr=np.array([0, n_pre_pages], dtype=np.int32),
                        kv_indices=pre_pages.copy(),
                        last_page_len=np.array([page], dtype=np.int32), **common)
    suffix = PagedBatch(name="c5_suffix" + tag, qo_indptr=np.arange(n + 1, dtype=np.int32),
                        kv_indptr=(base.kv_indptr[1:] - n_pre_pages).astype(np.int32),
                        kv_indices=base.kv_indices[n_pre_pages:].copy(),
                        last_page_len=base.last_page_len[1:].copy(), **common)
    idx, indptr = [], [0]
    for i in range(n):
        own = suffix.kv_indices[suffix.kv_indptr[i]:suffix.kv_indptr[i + 1]]
        idx.append(pre_pages)
        idx.append(own)
        indptr.append(indptr[-1] + n_pre_pages + len(own))
    single = PagedBatch(name="c5_single" + tag, qo_indptr=np.arange(n + 1, dtype=np.int32),
                        kv_indptr=np.array(indptr, dtype=np.int32),
                        kv_indices=np.concatenate(idx).astype(np.int32),
                        last_page_len=suffix.last_page_len.copy(), **common)
    return SharedPrefixCase(prefix=prefix, suffix=suffix, single=single)


def short_append(qo_len: int, batch: int, kv_max: int) -> PagedBatch:
    """Every request appends `qo_len` tokens (a verification step of speculative decoding, a chunk of a chunked
    prefill) to a cache of U{kv_max/4 .. kv_max - 1} tokens (the new tokens included); causal; GQA 32/8, D 128, bf16,
    page 16.  No NaN poisoning (these are timing inputs)."""
    g = np.random.Generator(np.random.PCG64(1100 + qo_len))
    kv = np.maximum(g.integers(kv_max // 4, kv_max, size=batch), qo_len)
    return make_batch(f"short_append_qo{qo_len}_bs{batch}_kv{kv_max}", 1100 + qo_len, BF16, 32, 8, 128, 16,
                      [qo_len] * batch, kv, causal=True, poison=False)


def random_case(seed: int, *, dtype: str = BF16, num_qo_heads: int = 32, num_kv_heads: int = 8,
                head_dim: int = 128, page_size: int = 16, batch: int = 5, max_qo: int = 1,
                max_kv: int = 300, causal: bool = False, allow_empty: bool = True,
                value_scale: float = 1.0, kv_dtype: str = "", k_scale: float = 1.0,
                v_scale: float = 1.0) -> PagedBatch:
    """Small adversarial batch: ragged lengths, optional empty requests, spare pages."""
    g = np.random.Generator(np.random.PCG64(seed))
    qo = g.integers(1, max_qo + 1, size=batch) if max_qo > 1 else np.ones(batch, dtype=np.int64)
    if causal:
        pre = g.integers(0, max(max_kv - max_qo, 0) + 1, size=batch)
        kv = qo + pre
    else:
        kv = g.integers(1, max_kv + 1, size=batch)
        if allow_empty and batch >= 3:
            kv[g.integers(0, batch)] = 0
    need = int(((kv + page_size - 1) // page_size).sum())
    return make_batch(f"rand{seed}", seed, dtype, num_qo_heads, num_kv_heads, head_dim, page_size,
                      qo, kv, causal=causal, num_pages=need + 3, value_scale=value_scale, kv_dtype=kv_dtype,
                      k_scale=k_scale, v_scale=v_scale)
