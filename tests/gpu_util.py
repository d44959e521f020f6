"""Helpers for the GPU parity tests: the tolerances of the comparison with the oracle.  Shipping a
batch to the device and running it through the C-ABI library is the package's `device` module."""
from __future__ import annotations

import numpy as np

from paper_2501_01005_amd.device import DeviceBatch, bits_to_torch, make_wrapper, run_gpu  # noqa: F401

O_TOL = 2e-3     # max-abs on o for fp16/bf16 inputs with fp32 accumulation
LSE_TOL = 1e-3   # max-abs on lse


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
