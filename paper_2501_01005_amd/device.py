"""Moves a host-side paged batch (the `workloads.PagedBatch` fields: 16-bit patterns of q, the K/V
pools, page table) into device memory and runs it through the C-ABI library.  Used by the
benchmark, the smoke check and the GPU tests; no arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np

from .binding import PagedAttention


def bits_to_torch(bits: np.ndarray, dtype: str, device):
    """uint16 bit patterns -> a torch tensor of the 16-bit type they encode, on `device`."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    t = t.view(torch.float16 if dtype == "f16" else torch.bfloat16)
    return t.to(device)


class DeviceBatch:
    """q, k_pool, v_pool, kv_indices of a batch as device tensors (8-bit K/V: uint8 codes + scales)."""

    def __init__(self, batch, device="cuda:0", kv_layout="HND"):
        import torch
        self.batch = batch
        self.device = torch.device(device)
        self.q = bits_to_torch(batch.q_bits, batch.dtype, self.device)
        if getattr(batch, "kv_dtype", "") == "fp8_e4m3":   # 8-bit KV cache: uint8 tensors of E4M3 codes
            k = torch.from_numpy(np.ascontiguousarray(batch.k_bits)).to(self.device)
            v = torch.from_numpy(np.ascontiguousarray(batch.v_bits)).to(self.device)
            self.scales = {"k_scale": batch.k_scale, "v_scale": batch.v_scale}
        else:
            k = bits_to_torch(batch.k_bits, batch.dtype, self.device)
            v = bits_to_torch(batch.v_bits, batch.dtype, self.device)
            self.scales = {}
        if kv_layout == "NHD":   # [pages, page_size, kv_heads, D] in memory, presented through strides
            k = k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
            v = v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        self.k_pool, self.v_pool = k, v
        self.kv_indices = torch.from_numpy(np.ascontiguousarray(batch.kv_indices, dtype=np.int32)).to(self.device)
        if self.kv_indices.numel() == 0:
            self.kv_indices = torch.zeros(1, dtype=torch.int32, device=self.device)


def make_wrapper(batch, mode, **kw) -> PagedAttention:
    """A PagedAttention sized for this batch (max_batch, max_qo_tiles from its lengths)."""
    g = batch.num_qo_heads // batch.num_kv_heads
    t_pos = {"decode": 1, "tile16": 16 // g, "tile64": 64 // g, "append": 256 // g}[mode]
    tiles = int(sum(-(-int(l) // t_pos) for l in batch.qo_lens()))
    return PagedAttention(dtype=batch.dtype, num_qo_heads=batch.num_qo_heads, num_kv_heads=batch.num_kv_heads,
                          head_dim=batch.head_dim, page_size=batch.page_size, mode=mode,
                          max_batch=max(batch.batch, 1), max_qo_tiles=max(tiles, 1), **kw)


def run_gpu(batch, mode="decode", dev: DeviceBatch | None = None, wrapper=None, poison=True, with_cast=False,
            contiguous=False, **kw):
    """fi_plan + fi_run of the batch; returns (o, lse) as float64 numpy (and the rounded output when
    with_cast).  poison: the partial-state sections of the workspace and the outputs start as NaN.
    contiguous: run without a page table (kv_indices = NULL; the batch's page table must be the identity)."""
    import torch
    dev = dev or DeviceBatch(batch)
    own = wrapper is None
    w = wrapper or make_wrapper(batch, mode, **kw)
    if poison:
        w.workspace.view(torch.float32)[w.pin_bytes // 4:].fill_(float("nan"))
    w.plan(batch.qo_indptr, batch.kv_indptr, batch.last_page_len, causal=batch.causal)
    nnz = dev.q.shape[0]
    o = torch.full((nnz, batch.num_qo_heads, batch.head_dim), float("nan"), dtype=torch.float32, device=dev.device)
    lse = torch.full((nnz, batch.num_qo_heads), float("nan"), dtype=torch.float32, device=dev.device)
    oc = torch.zeros((nnz, batch.num_qo_heads, batch.head_dim), dtype=dev.q.dtype, device=dev.device) if with_cast else None
    if contiguous:
        assert np.array_equal(batch.kv_indices, np.arange(len(batch.kv_indices))), "not a contiguous cache"
    w.run(dev.q, dev.k_pool, dev.v_pool, None if contiguous else dev.kv_indices, batch.sm_scale, o=o, lse=lse, o_cast=oc,
          **dev.scales)
    torch.cuda.synchronize()
    res = (o.double().cpu().numpy(), lse.double().cpu().numpy())
    if with_cast:
        res = res + (oc.double().cpu().numpy(),)
    if own:
        w.close()
    return res


def make_formats_wrapper(batches, mode="tile16", **kw) -> PagedAttention:
    """A 16-row-tile or 64-row-tile PagedAttention sized for planning these formats (views of one pool over the same
    query rows) as one work list."""
    b0 = batches[0]
    t_pos = {"tile16": 16, "tile64": 64}[mode] // (b0.num_qo_heads // b0.num_kv_heads)
    tiles = int(sum(-(-int(l) // t_pos) for b in batches for l in b.qo_lens()))
    return PagedAttention(dtype=b0.dtype, num_qo_heads=b0.num_qo_heads, num_kv_heads=b0.num_kv_heads,
                          head_dim=b0.head_dim, page_size=b0.page_size, mode=mode,
                          max_batch=max(sum(b.batch for b in batches), 1), max_qo_tiles=max(tiles, 1), **kw)


def formats_of(batches):
    """(the argument of PagedAttention.plan_formats, the formats' page ids one after the other as a host array)"""
    formats, ids, base = [], [], 0
    for b in batches:
        formats.append((b.qo_indptr, b.kv_indptr, b.last_page_len, base))
        ids.append(np.asarray(b.kv_indices, dtype=np.int32))
        base += len(b.kv_indices)
    return formats, (np.concatenate(ids) if base else np.zeros(1, dtype=np.int32))
