"""Pins for the oracle's rotary position embedding (query / key transform of Sec. 3.2.3; fused-RoPE attention,
Sec. 4.3): what a rotation must satisfy, a closed form, a pure-Python brute force with explicit 2 x 2 rotations,
and the equivalence of the fused form with rotating the stored keys first and running plain attention."""
import cmath
import math

import numpy as np

import oracle
import workloads
from oracle.attention import attention_state, rope


def rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def test_rotation_properties():
    x = rand((9, 16), 1)
    pos = np.array([0, 1, 2, 5, 100, 1000, 4095, 70000, 131071])
    y = rope(x, pos, 10000.0)
    assert np.array_equal(y[0], x[0])                                        # position 0: identity
    assert np.allclose((y ** 2).sum(axis=1), (x ** 2).sum(axis=1), rtol=1e-13)   # a rotation keeps the norm
    # every pair keeps its own norm; the pairing is (d, d + D/2)
    assert np.allclose(y[:, :8] ** 2 + y[:, 8:] ** 2, x[:, :8] ** 2 + x[:, 8:] ** 2, rtol=1e-12)
    # rotating by a and then by b is rotating by a + b
    z = rope(rope(x, pos, 10000.0), 3 * pos + 7, 10000.0)
    assert np.allclose(z, rope(x, 4 * pos + 7, 10000.0), atol=1e-9)
    # scale divides the position
    assert np.allclose(rope(x, pos, 10000.0, scale=4.0), rope(x, pos / 4.0, 10000.0), atol=1e-12)


def test_closed_form_per_pair():
    # the pair (d, d + D/2) as a complex number is multiplied by exp(i * pos * theta ** (-2 d / D))
    D, theta = 8, 50.0
    x = rand((5, D), 2)
    pos = np.array([3, 0, 17, 1, 250])
    y = rope(x, pos, theta)
    for n in range(5):
        for d in range(D // 2):
            z = complex(x[n, d], x[n, d + D // 2]) * cmath.exp(1j * pos[n] * theta ** (-2.0 * d / D))
            assert abs(y[n, d] - z.real) < 1e-12 and abs(y[n, d + D // 2] - z.imag) < 1e-12
    # first pair: frequency 1 -> angle = position in radians; a quarter turn swaps the components
    e = np.zeros((1, 4)); e[0, 0] = 1.0
    q = rope(e, np.array([math.pi / 2]), 10000.0)
    assert abs(q[0, 0]) < 1e-15 and abs(q[0, 2] - 1.0) < 1e-15


def test_logits_depend_on_the_distance_only():
    q, k = rand((1, 32), 3), rand((1, 32), 4)
    ref = float(rope(q, [40], 1e4)[0] @ rope(k, [25], 1e4)[0])
    for shift in (1, 7, 1000, 65536):
        s = float(rope(q, [40 + shift], 1e4)[0] @ rope(k, [25 + shift], 1e4)[0])
        assert abs(s - ref) < 1e-8
    assert abs(float(rope(q, [15], 1e4)[0] @ k[0]) - ref) < 1e-9          # = rotating q by the distance alone


def brute_rope_attention(q, K, V, sm_scale, theta, q_pos):
    """pure Python: rotate pair by pair with explicit sines and cosines, then softmax attention"""
    D = len(q)
    half = D // 2

    def rot(x, p):
        y = list(x)
        for d in range(half):
            a = p * theta ** (-2.0 * d / D)
            y[d] = x[d] * math.cos(a) - x[d + half] * math.sin(a)
            y[d + half] = x[d + half] * math.cos(a) + x[d] * math.sin(a)
        return y

    qr = rot(q, q_pos)
    s = [sm_scale * sum(a * b for a, b in zip(qr, rot(K[t], t))) for t in range(len(K))]
    m = max(s)
    w = [math.exp(x - m) for x in s]
    o = [sum(w[t] * V[t][d] for t in range(len(K))) / sum(w) for d in range(len(V[0]))]
    return o, m + math.log(sum(w))


def test_batch_oracle_against_pure_python_and_against_rotating_the_cache_first():
    import dataclasses
    qo, kv = [1, 3, 1], [9, 7, 1]
    for causal in (False, True):
        b = workloads.make_batch("rope", 5, workloads.F16, 2, 1, 4, 2, qo, kv, causal, poison=False, permute_pages=False)
        o, lse = oracle.run_batch(b, rope_theta=100.0)
        q = workloads.widen(b.q_bits, b.dtype)
        k = workloads.widen(b.k_bits, b.dtype)
        v = workloads.widen(b.v_bits, b.dtype)
        for i in range(3):
            p0 = int(b.kv_indptr[i])
            K = [k[p0 + t // 2, 0, t % 2].tolist() for t in range(kv[i])]
            V = [v[p0 + t // 2, 0, t % 2].tolist() for t in range(kv[i])]
            for j in range(qo[i]):
                pos = kv[i] - qo[i] + j
                n_vis = pos + 1 if causal else kv[i]
                for h in range(2):
                    r = int(b.qo_indptr[i]) + j
                    o_b, l_b = brute_rope_attention(q[r, h].tolist(), K[:n_vis], V[:n_vis], b.sm_scale, 100.0, pos)
                    assert np.allclose(o[r, h], o_b, atol=1e-12) and abs(lse[r, h] - l_b) < 1e-12
    # fused = rotate queries and stored keys first (in float64), then the plain oracle on the rotated values
    b = workloads.make_batch("rope2", 6, workloads.BF16, 4, 2, 16, 4, [1, 2], [13, 6], True, poison=False, permute_pages=False)
    o, lse = oracle.run_batch(b, rope_theta=1e4, rope_scale=2.0)
    q = workloads.widen(b.q_bits, b.dtype)
    k = workloads.widen(b.k_bits, b.dtype)
    v = workloads.widen(b.v_bits, b.dtype)
    for i, (lq, lk) in enumerate(((1, 13), (2, 6))):
        p0, p1 = int(b.kv_indptr[i]), int(b.kv_indptr[i + 1])
        for h in range(4):
            K = k[p0:p1, h // 2].reshape(-1, 16)[:lk]
            V = v[p0:p1, h // 2].reshape(-1, 16)[:lk]
            Kr = rope(K, np.arange(lk), 1e4, 2.0)
            r0 = int(b.qo_indptr[i])
            qr = rope(q[r0:r0 + lq, h], lk - lq + np.arange(lq), 1e4, 2.0)
            vis = np.arange(lk)[None, :] <= (lk - lq + np.arange(lq))[:, None]
            o2, l2 = attention_state(qr, Kr, V, b.sm_scale, vis)
            assert np.allclose(o[r0:r0 + lq, h], o2, atol=1e-13) and np.allclose(lse[r0:r0 + lq, h], l2, atol=1e-13)
