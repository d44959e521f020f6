"""ctypes binding of include/fi355.h.  Same names as the C entry points; argument
marshalling only.  `PagedAttention` is a convenience holder of the caller-owned buffers
(device workspace, pinned staging) allocated with torch."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

__all__ = [
    "FI_OK", "FI_ERR_INVALID_ARG", "FI_ERR_UNSUPPORTED", "FI_ERR_WORKSPACE_TOO_SMALL", "FI_ERR_NOT_PLANNED",
    "FI_ERR_HIP", "FI_ERR_HOST_MEMORY", "FI_DTYPE_F16", "FI_DTYPE_BF16", "FI_MODE_DECODE", "FI_MODE_APPEND", "FI_MODE_TILE16", "FI_MODE_TILE64",
    "Fi355Error", "fi_config", "fi_plan_arrays", "lib", "library_path",
    "fi_create", "fi_destroy", "fi_workspace_bytes", "fi_plan", "fi_plan_formats", "fi_plan_view", "fi_run", "fi_run_kv8",
    "fi_run_variant", "fi_run_composed", "fi_run_composed_static", "fi_variant", "fi_merge_states", "fi_merge_state_pair", "fi_check_indices", "fi_suggest_mode", "fi_set_timing_events", "fi_last_error",
    "PagedAttention",
]

FI_OK = 0
FI_ERR_INVALID_ARG = -1
FI_ERR_UNSUPPORTED = -2
FI_ERR_WORKSPACE_TOO_SMALL = -3
FI_ERR_NOT_PLANNED = -4
FI_ERR_HIP = -5
FI_ERR_HOST_MEMORY = -6
FI_DTYPE_F16 = 0
FI_DTYPE_BF16 = 1
FI_MODE_DECODE = 0
FI_MODE_APPEND = 1
FI_MODE_TILE16 = 2
FI_MODE_TILE64 = 3

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    """The built library; FI355_LIBRARY overrides the in-tree path (e.g. an instrumented build)."""
    return os.environ.get("FI355_LIBRARY") or os.path.join(_HERE, "lib", "libfi355.so")


class Fi355Error(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"fi355 error {code}: {message}")
        self.code = code
        self.message = message


class fi_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "dtype", "num_qo_heads", "num_kv_heads", "head_dim", "page_size", "mode", "num_ctas", "max_batch",
        "max_qo_tiles", "alpha", "beta", "min_chunk", "literal_lkv", "balance", "merge", "plan_window", "max_formats")]


_I32P = ctypes.POINTER(ctypes.c_int32)


class fi_variant(ctypes.Structure):
    _fields_ = [("logits_soft_cap", ctypes.c_float), ("window_left", ctypes.c_int32), ("alibi_slopes", ctypes.c_void_p),
                ("rope_theta", ctypes.c_float), ("rope_scale", ctypes.c_float)]


class fi_plan_arrays(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "t_pos", "group", "ctas_per_head", "l_kv_chunk", "n_work", "n_merge", "n_slots", "pad_")] + [
        (n, _I32P) for n in (
            "cta_indptr", "w_request", "w_q_row0", "w_n_pos", "w_kv_page0", "w_kv_start", "w_kv_len", "w_diag0",
            "w_out_slot", "w_merge", "m_q_row0", "m_n_pos", "m_slot_base", "m_n_chunks")] + [
        ("n_rows", ctypes.c_int32), ("pad2_", ctypes.c_int32), ("row_indptr", _I32P), ("row_entry", _I32P)]


def _load() -> ctypes.CDLL:
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is not built: run `python -m paper_2501_01005_amd.build` (hipcc, gfx950). "
            "There is no fallback path.")
    try:  # share torch's HIP runtime (streams and pointers cross this boundary)
        import torch  # noqa: F401
    except Exception:  # pragma: no cover - host-only use (plan) works without torch
        pass
    L = ctypes.CDLL(path)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    L.fi_create.argtypes = [ctypes.POINTER(fi_config), ctypes.POINTER(vp)]
    L.fi_destroy.argtypes = [vp]
    L.fi_workspace_bytes.argtypes = [vp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.fi_plan.argtypes = [vp, vp, vp, vp, i32, i32, vp, sz, vp, sz, vp]
    L.fi_plan_formats.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp, vp, sz, vp, sz, vp]
    L.fi_plan_view.argtypes = [vp, ctypes.POINTER(fi_plan_arrays)]
    L.fi_run.argtypes = [vp, vp, vp, vp, ctypes.POINTER(i64), vp, ctypes.c_float, vp, vp, vp, vp]
    L.fi_run_variant.argtypes = [vp, vp, vp, vp, ctypes.POINTER(i64), vp, vp, vp, ctypes.c_float,
                                 ctypes.POINTER(fi_variant), vp, vp, vp, vp]
    L.fi_run_kv8.argtypes = [vp, vp, vp, vp, ctypes.POINTER(i64), vp, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                             vp, vp, vp, vp]
    L.fi_merge_states.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    L.fi_merge_state_pair.argtypes = [vp, vp, vp, vp, i64, i32, vp, vp, vp]
    L.fi_run_composed.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(i64), vp, vp, ctypes.c_float, vp, vp, vp, vp, i64,
                                  vp, vp, vp, vp]
    L.fi_run_composed_static.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(i64), vp, vp, ctypes.c_float, i64, vp, vp, vp, vp]
    L.fi_check_indices.argtypes = [vp, i64, i32]
    L.fi_suggest_mode.argtypes = [i32, i32, ctypes.c_double]
    L.fi_suggest_mode.restype = i32
    L.fi_set_timing_events.argtypes = [vp, vp, vp]
    L.fi_last_error.argtypes = []
    L.fi_last_error.restype = ctypes.c_char_p
    for name in ("fi_create", "fi_destroy", "fi_workspace_bytes", "fi_plan", "fi_plan_formats", "fi_plan_view", "fi_run", "fi_run_kv8",
                 "fi_run_variant", "fi_run_composed", "fi_run_composed_static", "fi_merge_states", "fi_merge_state_pair", "fi_check_indices", "fi_set_timing_events"):
        getattr(L, name).restype = i32
    return L


lib = _load()


def fi_last_error() -> str:
    return lib.fi_last_error().decode()


def _check(rc: int) -> None:
    if rc != FI_OK:
        raise Fi355Error(rc, fi_last_error())


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(t) -> Optional[int]:
    """Device/host address of a torch tensor, numpy array, int or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def fi_create(**kw) -> int:
    cfg = fi_config()
    for k, v in kw.items():
        setattr(cfg, k, v)
    out = ctypes.c_void_p()
    _check(lib.fi_create(ctypes.byref(cfg), ctypes.byref(out)))
    return out.value


def fi_destroy(handle: int) -> None:
    _check(lib.fi_destroy(handle))


def fi_workspace_bytes(handle: int):
    d, p = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.fi_workspace_bytes(handle, ctypes.byref(d), ctypes.byref(p)))
    return d.value, p.value


def fi_plan(handle: int, qo_indptr, kv_indptr, last_page_len, causal: bool, workspace=None,
            workspace_bytes: int = 0, pinned=None, pinned_bytes: int = 0, stream: int = 0) -> None:
    qo = _host_i32(qo_indptr)
    kv = _host_i32(kv_indptr)
    lp = _host_i32(last_page_len)
    batch = len(lp)
    if len(qo) != batch + 1 or len(kv) != batch + 1:
        raise ValueError("indptr arrays must have batch + 1 entries")
    _check(lib.fi_plan(handle, qo.ctypes.data, kv.ctypes.data, lp.ctypes.data if batch else None, batch,
                       1 if causal else 0, _ptr(workspace), workspace_bytes, _ptr(pinned), pinned_bytes,
                       stream or None))


def fi_plan_formats(handle: int, formats, workspace=None, workspace_bytes: int = 0, pinned=None, pinned_bytes: int = 0,
                    stream: int = 0) -> None:
    """formats: sequence of (qo_indptr, kv_indptr, last_page_len, kv_indices_base) per format."""
    n = len(formats)
    keep = []
    ptrs = [(ctypes.c_void_p * n)() for _ in range(3)]
    batch = np.zeros(n, dtype=np.int32)
    base = np.zeros(n, dtype=np.int32)
    for f, (qo, kv, lp, kv_base) in enumerate(formats):
        arrs = (_host_i32(qo), _host_i32(kv), _host_i32(lp))
        if len(arrs[0]) != len(arrs[2]) + 1 or len(arrs[1]) != len(arrs[2]) + 1:
            raise ValueError("indptr arrays must have batch + 1 entries")
        keep.append(arrs)
        for k in range(3):
            ptrs[k][f] = arrs[k].ctypes.data if len(arrs[k]) else None
        batch[f], base[f] = len(arrs[2]), int(kv_base)
    _check(lib.fi_plan_formats(handle, n, ptrs[0], ptrs[1], ptrs[2], batch.ctypes.data, base.ctypes.data,
                               _ptr(workspace), workspace_bytes, _ptr(pinned), pinned_bytes, stream or None))


def fi_plan_view(handle: int) -> dict:
    pa = fi_plan_arrays()
    _check(lib.fi_plan_view(handle, ctypes.byref(pa)))
    out = {k: getattr(pa, k) for k in ("t_pos", "group", "ctas_per_head", "l_kv_chunk", "n_work", "n_merge", "n_slots")}

    def arr(p, n):
        return np.ctypeslib.as_array(p, shape=(n,)).copy() if n > 0 else np.zeros(0, dtype=np.int32)

    out["cta_indptr"] = arr(pa.cta_indptr, pa.ctas_per_head + 1)
    for k in ("w_request", "w_q_row0", "w_n_pos", "w_kv_page0", "w_kv_start", "w_kv_len", "w_diag0", "w_out_slot",
              "w_merge"):
        out[k] = arr(getattr(pa, k), pa.n_work)
    for k in ("m_q_row0", "m_n_pos", "m_slot_base", "m_n_chunks"):
        out[k] = arr(getattr(pa, k), pa.n_merge)
    out["n_rows"] = pa.n_rows
    if pa.n_rows > 0:   # a plan over several formats: the partial states every query row folds
        out["row_indptr"] = arr(pa.row_indptr, pa.n_rows + 1)
        out["row_entry"] = arr(pa.row_entry, int(out["row_indptr"][-1]))
    return out


def fi_run(handle: int, q, k_pool, v_pool, kv_strides: Sequence[int], kv_indices, sm_scale: float, o, lse,
           o_cast=None, stream: int = 0) -> None:
    st = (ctypes.c_int64 * 3)(*[int(s) for s in kv_strides])
    _check(lib.fi_run(handle, _ptr(q), _ptr(k_pool), _ptr(v_pool), st, _ptr(kv_indices), float(sm_scale),
                      _ptr(o), _ptr(lse), _ptr(o_cast), stream or None))


def fi_run_variant(handle: int, q, k_pool, v_pool, kv_strides: Sequence[int], kv_indices, kv_indptr, last_page_len,
                   sm_scale: float, o, lse, o_cast=None, stream: int = 0, *, logits_soft_cap: float = 0.0,
                   window_left: int = -1, alibi_slopes=None, rope_theta: float = 0.0,
                   rope_scale: float = 0.0) -> None:
    st = (ctypes.c_int64 * 3)(*[int(s) for s in kv_strides])
    var = fi_variant(float(logits_soft_cap), int(window_left), _ptr(alibi_slopes), float(rope_theta), float(rope_scale))
    _check(lib.fi_run_variant(handle, _ptr(q), _ptr(k_pool), _ptr(v_pool), st, _ptr(kv_indices), _ptr(kv_indptr),
                              _ptr(last_page_len), float(sm_scale), ctypes.byref(var), _ptr(o), _ptr(lse),
                              _ptr(o_cast), stream or None))


def fi_run_kv8(handle: int, q, k_pool, v_pool, kv_strides: Sequence[int], kv_indices, sm_scale: float,
               k_scale: float, v_scale: float, o, lse, o_cast=None, stream: int = 0) -> None:
    st = (ctypes.c_int64 * 3)(*[int(s) for s in kv_strides])
    _check(lib.fi_run_kv8(handle, _ptr(q), _ptr(k_pool), _ptr(v_pool), st, _ptr(kv_indices), float(sm_scale),
                          float(k_scale), float(v_scale), _ptr(o), _ptr(lse), _ptr(o_cast), stream or None))


def fi_merge_states(o_parts, lse_parts, n_rows: int, n_states: int, head_dim: int, o, lse, stream: int = 0) -> None:
    _check(lib.fi_merge_states(_ptr(o_parts), _ptr(lse_parts), n_rows, n_states, head_dim, _ptr(o), _ptr(lse),
                               stream or None))


def fi_merge_state_pair(o_a, lse_a, o_b, lse_b, n_rows: int, head_dim: int, o, lse, stream: int = 0) -> None:
    _check(lib.fi_merge_state_pair(_ptr(o_a), _ptr(lse_a), _ptr(o_b), _ptr(lse_b), n_rows, head_dim, _ptr(o),
                                   _ptr(lse), stream or None))


def fi_run_composed(handle_a: int, handle_b: int, q, k_pool, v_pool, kv_strides: Sequence[int], kv_indices_a,
                    kv_indices_b, sm_scale: float, o_a, lse_a, o_b, lse_b, nnz_qo: int, o, lse, o_cast=None,
                    stream: int = 0) -> None:
    strides = (ctypes.c_int64 * 3)(*[int(s) for s in kv_strides])
    _check(lib.fi_run_composed(handle_a, handle_b, _ptr(q), _ptr(k_pool), _ptr(v_pool), strides, _ptr(kv_indices_a),
                               _ptr(kv_indices_b), float(sm_scale), _ptr(o_a), _ptr(lse_a), _ptr(o_b), _ptr(lse_b),
                               int(nnz_qo), _ptr(o), _ptr(lse), _ptr(o_cast), stream or None))


def fi_run_composed_static(handle_a: int, handle_b: int, q, k_pool, v_pool, kv_strides: Sequence[int], kv_indices_a,
                           kv_indices_b, sm_scale: float, nnz_qo: int, o, lse, o_cast=None, stream: int = 0) -> None:
    strides = (ctypes.c_int64 * 3)(*[int(s) for s in kv_strides])
    _check(lib.fi_run_composed_static(handle_a, handle_b, _ptr(q), _ptr(k_pool), _ptr(v_pool), strides,
                                      _ptr(kv_indices_a), _ptr(kv_indices_b), float(sm_scale), int(nnz_qo), _ptr(o),
                                      _ptr(lse), _ptr(o_cast), stream or None))


def fi_set_timing_events(handle: int, before, after) -> None:
    _check(lib.fi_set_timing_events(handle, before, after))


def fi_suggest_mode(num_qo_heads: int, num_kv_heads: int, mean_qo_len: float) -> str:
    """the PagedAttention mode name for a batch of that average query length"""
    rc = lib.fi_suggest_mode(num_qo_heads, num_kv_heads, float(mean_qo_len))
    if rc < 0:
        _check(rc)
    return {FI_MODE_DECODE: "decode", FI_MODE_APPEND: "append", FI_MODE_TILE16: "tile16", FI_MODE_TILE64: "tile64"}[rc]


def fi_check_indices(indices, num_pages: int) -> None:
    a = _host_i32(indices)
    _check(lib.fi_check_indices(a.ctypes.data if len(a) else None, len(a), num_pages))


class PagedAttention:
    """Owns what the C ABI leaves to the caller: handle, device workspace, pinned staging.

    torch provides device memory and the stream; every step of the computation runs in
    the library's kernels."""

    def __init__(self, *, dtype: str, num_qo_heads: int, num_kv_heads: int, head_dim: int = 128,
                 page_size: int = 16, mode: str = "decode", max_batch: int, max_qo_tiles: Optional[int] = None,
                 num_ctas: int = 0, min_chunk: int = 0, alpha: int = 0, beta: int = 0, literal_lkv: bool = False,
                 balance: int = 0, merge: int = 0, plan_window: int = 0, max_formats: int = 0,
                 device: str = "cuda:0"):
        import torch

        self.torch = torch
        self.device = torch.device(device)
        self.dtype = dtype
        self.mode = mode
        self.torch_dtype = {"f16": torch.float16, "bf16": torch.bfloat16}[dtype]
        with torch.cuda.device(self.device):
            self.handle = fi_create(
                dtype={"f16": FI_DTYPE_F16, "bf16": FI_DTYPE_BF16}[dtype], num_qo_heads=num_qo_heads,
                num_kv_heads=num_kv_heads, head_dim=head_dim, page_size=page_size,
                mode={"decode": FI_MODE_DECODE, "append": FI_MODE_APPEND, "tile16": FI_MODE_TILE16, "tile64": FI_MODE_TILE64}[mode], num_ctas=num_ctas,
                max_batch=max_batch, max_qo_tiles=max_qo_tiles if max_qo_tiles is not None else max_batch,
                alpha=alpha, beta=beta, min_chunk=min_chunk, literal_lkv=1 if literal_lkv else 0, balance=balance,
                merge=merge, plan_window=plan_window, max_formats=max_formats)
        self.num_qo_heads, self.num_kv_heads, self.head_dim = num_qo_heads, num_kv_heads, head_dim
        dev_bytes, pin_bytes = fi_workspace_bytes(self.handle)
        self.workspace = torch.empty(dev_bytes, dtype=torch.uint8, device=self.device)
        # ring of staging buffers: a buffer is rewritten only after the copy that read it has executed
        self._ring = [torch.empty(pin_bytes, dtype=torch.uint8, pin_memory=True) for _ in range(4)]
        self._ring_events = [None] * len(self._ring)
        self._ring_pos = 0
        self.ws_bytes, self.pin_bytes = dev_bytes, pin_bytes

    def close(self) -> None:
        if self.handle:
            fi_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def plan(self, qo_indptr, kv_indptr, last_page_len, causal: bool = False) -> None:
        i = self._ring_pos
        self._ring_pos = (i + 1) % len(self._ring)
        if self._ring_events[i] is not None:
            self._ring_events[i].synchronize()
        fi_plan(self.handle, qo_indptr, kv_indptr, last_page_len, causal, self.workspace, self.ws_bytes,
                self._ring[i], self.pin_bytes, self._stream())
        if self._ring_events[i] is None:
            self._ring_events[i] = self.torch.cuda.Event()
        self._ring_events[i].record(self.torch.cuda.current_stream(self.device))

    def plan_formats(self, formats) -> None:
        """formats: sequence of (qo_indptr, kv_indptr, last_page_len, kv_indices_base); see fi_plan_formats."""
        i = self._ring_pos
        self._ring_pos = (i + 1) % len(self._ring)
        if self._ring_events[i] is not None:
            self._ring_events[i].synchronize()
        fi_plan_formats(self.handle, formats, self.workspace, self.ws_bytes, self._ring[i], self.pin_bytes, self._stream())
        if self._ring_events[i] is None:
            self._ring_events[i] = self.torch.cuda.Event()
        self._ring_events[i].record(self.torch.cuda.current_stream(self.device))

    def run(self, q, k_pool, v_pool, kv_indices, sm_scale: float, o=None, lse=None, o_cast=None,
            k_scale: Optional[float] = None, v_scale: Optional[float] = None, variant: Optional[dict] = None):
        """k_scale / v_scale given: the pools are an 8-bit KV cache (uint8 tensors of E4M3 codes).
        variant: dict(kv_indptr=, last_page_len= (device int32 tensors), logits_soft_cap=, window_left=,
        alibi_slopes= (device float32 tensor), rope_theta=, rope_scale=) runs fi_run_variant.
        o=False with an o_cast tensor: the output is written in the input type only (returns o_cast, lse)."""
        torch = self.torch
        kv8 = k_scale is not None or v_scale is not None
        kv_dtype = torch.uint8 if kv8 else self.torch_dtype
        assert q.dtype == self.torch_dtype and k_pool.dtype == kv_dtype and v_pool.dtype == kv_dtype
        assert q.is_contiguous() and q.shape[1:] == (self.num_qo_heads, self.head_dim)
        assert k_pool.dim() == 4 and k_pool.stride(3) == 1 and k_pool.stride() == v_pool.stride()
        assert kv_indices is None or (kv_indices.dtype == torch.int32 and kv_indices.is_contiguous())  # None: contiguous KV
        nnz = q.shape[0]
        if o is False:
            assert o_cast is not None
            o = None
        elif o is None:
            o = torch.empty((nnz, self.num_qo_heads, self.head_dim), dtype=torch.float32, device=q.device)
        if lse is None:
            lse = torch.empty((nnz, self.num_qo_heads), dtype=torch.float32, device=q.device)
        # k_pool is [pages, kv_heads, page_size, D] (or any permutation of the first three through strides)
        strides = (k_pool.stride(0), k_pool.stride(1), k_pool.stride(2))
        if variant is not None:
            fi_run_variant(self.handle, q, k_pool, v_pool, strides, kv_indices, variant["kv_indptr"],
                           variant["last_page_len"], sm_scale, o, lse, o_cast, self._stream(),
                           logits_soft_cap=variant.get("logits_soft_cap", 0.0),
                           window_left=variant.get("window_left", -1), alibi_slopes=variant.get("alibi_slopes"),
                           rope_theta=variant.get("rope_theta", 0.0), rope_scale=variant.get("rope_scale", 0.0))
        elif kv8:
            fi_run_kv8(self.handle, q, k_pool, v_pool, strides, kv_indices, sm_scale,
                       1.0 if k_scale is None else k_scale, 1.0 if v_scale is None else v_scale, o, lse, o_cast,
                       self._stream())
        else:
            fi_run(self.handle, q, k_pool, v_pool, strides, kv_indices, sm_scale, o, lse, o_cast, self._stream())
        return (o_cast if o is None else o), lse

    def run_composed(self, other: "PagedAttention", q, k_pool, v_pool, kv_indices, kv_indices_other, sm_scale: float,
                     o=None, lse=None, o_cast=None):
        """This handle's format and `other`'s over the same query rows, composed by one contraction launch
        (fi_run_composed).  The per-pass state rows are kept on the handles between calls."""
        torch = self.torch
        nnz = q.shape[0]
        for w in (self, other):
            rows = getattr(w, "_pass_rows", None)
            if rows is None or rows[0].shape[0] < nnz:
                w._pass_rows = (torch.empty((nnz, self.num_qo_heads, self.head_dim), dtype=torch.float32, device=q.device),
                                torch.empty((nnz, self.num_qo_heads), dtype=torch.float32, device=q.device))
        if o is False:
            assert o_cast is not None
            o = None
        elif o is None:
            o = torch.empty((nnz, self.num_qo_heads, self.head_dim), dtype=torch.float32, device=q.device)
        if lse is None:
            lse = torch.empty((nnz, self.num_qo_heads), dtype=torch.float32, device=q.device)
        strides = (k_pool.stride(0), k_pool.stride(1), k_pool.stride(2))
        fi_run_composed(self.handle, other.handle, q, k_pool, v_pool, strides, kv_indices, kv_indices_other, sm_scale,
                        self._pass_rows[0], self._pass_rows[1], other._pass_rows[0], other._pass_rows[1], nnz, o, lse,
                        o_cast, self._stream())
        return (o_cast if o is None else o), lse
