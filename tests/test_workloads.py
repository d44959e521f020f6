"""Structure checks of the seeded synthetic inputs (no arithmetic of the method here)."""
import numpy as np

import workloads


def test_rounding_round_trips_and_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.3895314e38], dtype=np.float32)
    b = workloads.f32_to_bits(x, workloads.BF16)
    y = workloads.widen(b, workloads.BF16)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert y[0] == 1.0 and y[1] == 1.0 and y[2] == 1.015625 and y[3] == -2.5 and y[4] == 0.0
    assert np.array_equal(workloads.f32_to_bits(y.astype(np.float32), workloads.BF16), b)
    h = workloads.f32_to_bits(np.array([0.1], dtype=np.float32), workloads.F16)
    assert workloads.widen(h, workloads.F16)[0] == float(np.float16(0.1))


def test_config1_shape():
    b = workloads.config1()
    assert b.dtype == workloads.F16 and b.batch == 4 and b.num_pages == 256
    assert b.num_qo_heads == b.num_kv_heads == 8 and b.head_dim == 128 and b.page_size == 16
    kv = b.kv_lens()
    assert (kv >= 64).all() and (kv <= 512).all()
    assert len(set(b.kv_indices.tolist())) == len(b.kv_indices)             # no page shared
    assert not np.array_equal(b.kv_indices, np.sort(b.kv_indices))          # scattered
    again = workloads.config1()
    assert np.array_equal(again.k_bits, b.k_bits) and np.array_equal(again.kv_indices, b.kv_indices)


def test_config2_lengths_are_skewed():
    g = np.random.Generator(np.random.PCG64(1002))
    kv = workloads.zipf_lengths(g, 128, 256, 32768, 1.2)
    assert kv.min() >= 256 and kv.max() <= 32768
    assert np.median(kv) < kv.mean()                                        # long tail
    small = workloads.config2(small=True)
    assert small.kv_lens()[0] == 2048 and small.batch == 12 and small.dtype == workloads.BF16


def test_config3_has_the_forced_cases():
    b = workloads.config3(small=True)
    assert b.causal and (b.kv_lens() >= b.qo_lens()).all()
    assert (b.kv_lens() - b.qo_lens())[1] == 0


def test_config5_views_share_storage_and_pages():
    c = workloads.config5(small=True)
    assert c.prefix.k_bits is c.suffix.k_bits is c.single.k_bits
    assert c.prefix.batch == 1 and c.prefix.qo_lens()[0] == c.suffix.batch
    n_pre = len(c.prefix.kv_indices)
    for i in range(c.single.batch):
        row = c.single.kv_indices[c.single.kv_indptr[i]:c.single.kv_indptr[i + 1]]
        assert np.array_equal(row[:n_pre], c.prefix.kv_indices)
        own = c.suffix.kv_indices[c.suffix.kv_indptr[i]:c.suffix.kv_indptr[i + 1]]
        assert np.array_equal(row[n_pre:], own)
    assert (c.single.kv_lens() == c.suffix.kv_lens() + c.prefix.kv_lens()[0]).all()
