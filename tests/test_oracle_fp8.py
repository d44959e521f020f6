"""Pins for the oracle's decoding of the 8-bit KV cache (App. F: fp8 K/V, 16-bit queries, wider
arithmetic).  The format is OCP E4M3; the decoder is checked against the values the format
definition fixes, against a library routine (torch's float8_e4m3fn on the CPU), against the
independent encoder of the input generators (round trip), and the fp8 oracle path against the
already pinned 16-bit path on inputs both can represent."""
import dataclasses

import numpy as np

import oracle
import workloads
from oracle.fp8 import e4m3_to_f64


def test_values_fixed_by_the_format_definition():
    # (code, value): zero, smallest subnormal 2^-9, largest subnormal 7/8 * 2^-6, smallest normal 2^-6,
    # one, 1.5, largest finite 448 = 1.75 * 2^8, and their negatives
    table = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 0.875 * 2.0 ** -6, 0x08: 2.0 ** -6, 0x38: 1.0, 0x3C: 1.5, 0x40: 2.0,
             0x7E: 448.0, 0x80: -0.0, 0x81: -(2.0 ** -9), 0xB8: -1.0, 0xFE: -448.0, 0x77: 240.0, 0x78: 256.0}
    for code, val in table.items():
        got = float(e4m3_to_f64(np.array([code], dtype=np.uint8))[0])
        assert got == val and np.signbit(got) == np.signbit(val), (hex(code), got, val)
    assert np.isnan(e4m3_to_f64(np.array([0x7F, 0xFF], dtype=np.uint8))).all()


def test_every_code_is_finite_except_two_and_the_order_is_the_code_order():
    v = e4m3_to_f64(np.arange(256, dtype=np.uint8))
    assert np.isnan(v).sum() == 2
    pos = v[:0x7F]
    assert np.all(np.diff(pos) > 0), "positive codes are strictly increasing"
    assert np.array_equal(v[0x80:0xFF], -pos)
    assert len(np.unique(v[~np.isnan(v)])) == 253    # 254 finite codes, +0 and -0 equal


def test_matches_the_library_conversion_for_all_codes():
    import torch
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = e4m3_to_f64(codes)
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    fin = ~np.isnan(mine)
    assert np.array_equal(lib[fin], mine[fin])
    assert np.array_equal(np.signbit(lib[fin]), np.signbit(mine[fin]))


def test_round_trip_through_the_generators_encoder_and_its_rounding():
    codes = np.arange(256, dtype=np.uint8)
    v = e4m3_to_f64(codes)
    fin = ~np.isnan(v)
    assert np.array_equal(workloads.f32_to_e4m3_bits(v[fin].astype(np.float32)), codes[fin])
    # nearest, ties to even mantissa, saturation at 448, underflow to zero
    x = np.array([1.0625, 1.0626, 1.1875, 2.0 ** -10, 1.01 * 2.0 ** -10, 1.5 * 2.0 ** -9, 447.0, 500.0, -1e9, 1e-9],
                 dtype=np.float32)
    want = np.array([1.0, 1.125, 1.25, 0.0, 2.0 ** -9, 2.0 ** -8, 448.0, 448.0, -448.0, 0.0])
    assert np.array_equal(e4m3_to_f64(workloads.f32_to_e4m3_bits(x)), want)
    # the encoder is the nearest code: brute force over random values
    g = np.random.Generator(np.random.PCG64(7))
    r = (g.standard_normal(4000) * np.exp2(g.integers(-10, 9, size=4000))).astype(np.float32)
    fin_vals = np.unique(v[fin])
    near = fin_vals[np.abs(r.astype(np.float64)[:, None] - fin_vals[None, :]).argmin(axis=1)]
    got = e4m3_to_f64(workloads.f32_to_e4m3_bits(r))
    d_got, d_near = np.abs(got - np.clip(r, -448, 448)), np.abs(near - np.clip(r, -448, 448))
    assert np.all(d_got <= d_near), "never farther than the nearest representable value"


def test_fp8_batch_equals_the_same_values_stored_in_16_bits():
    # E4M3 values and power-of-two scales are exact in bf16: the 8-bit path of the oracle must give, bit for bit,
    # what the pinned 16-bit path gives on the widened values
    for seed, causal in ((11, False), (12, True)):
        b8 = workloads.random_case(seed, num_qo_heads=4, num_kv_heads=2, head_dim=32, batch=4, max_qo=5 if causal else 1,
                                   max_kv=70, causal=causal, kv_dtype=workloads.FP8, k_scale=0.5, v_scale=4.0)
        assert b8.k_bits.dtype == np.uint8 and b8.kv_dtype == workloads.FP8
        k = e4m3_to_f64(b8.k_bits) * b8.k_scale
        v = e4m3_to_f64(b8.v_bits) * b8.v_scale
        k16 = workloads.f32_to_bits(np.nan_to_num(k, nan=0.0).astype(np.float32), workloads.BF16)
        v16 = workloads.f32_to_bits(np.nan_to_num(v, nan=0.0).astype(np.float32), workloads.BF16)
        assert np.array_equal(workloads.widen(k16, workloads.BF16), np.nan_to_num(k, nan=0.0)), "exact in bf16"
        k16[np.isnan(k)] = 0x7FC0
        v16[np.isnan(v)] = 0x7FC0
        b16 = dataclasses.replace(b8, k_bits=k16, v_bits=v16, kv_dtype="", k_scale=1.0, v_scale=1.0)
        o8, l8 = oracle.run_batch(b8)
        o16, l16 = oracle.run_batch(b16)
        assert np.array_equal(o8, o16, equal_nan=True) and np.array_equal(l8, l16, equal_nan=True)
        assert not np.isnan(o8[~np.isnan(l8)]).any(), "poisoned slots (NaN codes) must not leak"
