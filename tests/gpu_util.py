"""Helpers for the GPU parity tests: ship a workloads.PagedBatch to the device, run it
through the C-ABI library, bring (o, lse) back as float64."""
from __future__ import annotations

import numpy as np

O_TOL = 2e-3     # max-abs on o for fp16/bf16 inputs with fp32 accumulation
LSE_TOL = 1e-3   # max-abs on lse


def bits_to_torch(bits: np.ndarray, dtype: str, device):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    t = t.view(torch.float16 if dtype == "f16" else torch.bfloat16)
    return t.to(device)


class DeviceBatch:
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


def make_wrapper(batch, mode, **kw):
    import paper_2501_01005_amd as fi
    t_pos = 1 if mode == "decode" else 256 // (batch.num_qo_heads // batch.num_kv_heads)
    tiles = int(sum(-(-int(l) // t_pos) for l in batch.qo_lens()))
    return fi.PagedAttention(dtype=batch.dtype, num_qo_heads=batch.num_qo_heads, num_kv_heads=batch.num_kv_heads,
                             head_dim=batch.head_dim, page_size=batch.page_size, mode=mode,
                             max_batch=max(batch.batch, 1), max_qo_tiles=max(tiles, 1), **kw)


def run_gpu(batch, mode="decode", dev: DeviceBatch | None = None, wrapper=None, poison=True, with_cast=False, **kw):
    """Returns (o, lse) as float64 numpy (and the rounded output when with_cast)."""
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
    w.run(dev.q, dev.k_pool, dev.v_pool, dev.kv_indices, batch.sm_scale, o=o, lse=lse, o_cast=oc, **dev.scales)
    torch.cuda.synchronize()
    res = (o.double().cpu().numpy(), lse.double().cpu().numpy())
    if with_cast:
        res = res + (oc.double().cpu().numpy(),)
    if own:
        w.close()
    return res


def assert_close(o, lse, o_ref, lse_ref, what=""):
    sel = ~np.isnan(lse_ref)                       # rows the oracle computed
    assert sel.any(), "nothing to compare"
    empty = np.isneginf(lse_ref) & sel
    assert np.array_equal(np.isneginf(lse) & sel, empty), f"{what}: empty rows differ"
    fin = sel & ~empty
    assert not np.isnan(o[sel]).any() and not np.isnan(lse[sel]).any(), f"{what}: NaN in output"
    err_o = np.abs(o[sel] - o_ref[sel]).max()
    err_l = np.abs(lse[fin] - lse_ref[fin]).max() if fin.any() else 0.0
    assert err_o <= O_TOL, f"{what}: max |o - o_ref| = {err_o:.3e} > {O_TOL}"
    assert err_l <= LSE_TOL, f"{what}: max |lse - lse_ref| = {err_l:.3e} > {LSE_TOL}"
    return err_o, err_l
