"""Pins for the oracle's attention variants (Sec. 3.2.3: logits transform and logits mask; the paper's
evaluation uses soft cap, sliding window and ALiBi): each variant is checked against a special case that
reduces to plain attention, against a closed form, and all together against a pure-Python brute force."""
import math

import numpy as np

import oracle
import workloads
from oracle.attention import attention_state, batch_attention, variant_mask_and_bias


def rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def test_window_equals_plain_attention_over_the_last_tokens():
    q, K, V = rand((1, 8), 1), rand((37, 8), 2), rand((37, 8), 3)
    for W in (0, 1, 5, 36, 100):
        vis, bias = variant_mask_and_bias(1, 37, False, window_left=W)
        o, lse = attention_state(q, K, V, 0.3, vis)
        n = min(37, W + 1)
        o2, lse2 = attention_state(q, K[-n:], V[-n:], 0.3)
        assert np.allclose(o, o2, atol=1e-13) and np.allclose(lse, lse2, atol=1e-13)
    # causal append: row j sees tokens [pos - W, pos], pos = l_kv - l_qo + j
    q = rand((6, 8), 4)
    vis, _ = variant_mask_and_bias(6, 37, True, window_left=4)
    o, lse = attention_state(q, K, V, 0.3, vis)
    for j in range(6):
        pos = 37 - 6 + j
        o2, lse2 = attention_state(q[j:j + 1], K[pos - 4:pos + 1], V[pos - 4:pos + 1], 0.3)
        assert np.allclose(o[j], o2[0], atol=1e-13) and np.allclose(lse[j], lse2[0], atol=1e-13)


def test_soft_cap_limits():
    q, K, V = rand((3, 8), 5), rand((20, 8), 6), rand((20, 8), 7)
    o0, l0 = attention_state(q, K, V, 0.5)
    o1, l1 = attention_state(q, K, V, 0.5, logits_soft_cap=1e9)       # no cap in effect
    assert np.allclose(o0, o1, atol=1e-9) and np.allclose(l0, l1, atol=1e-9)
    o2, l2 = attention_state(q, K, V, 0.5, logits_soft_cap=1e-7)      # all logits ~ 0: uniform weights
    assert np.allclose(o2, V.mean(axis=0)[None, :], atol=1e-6) and np.allclose(l2, math.log(20), atol=1e-6)
    o3, l3 = attention_state(q, K, V, 0.5, logits_soft_cap=2.0)       # |s| <= cap
    assert np.all(l3 <= 2.0 + math.log(20) + 1e-12) and np.all(l3 >= -2.0 + math.log(20) - 1e-12)


def test_alibi_closed_form_on_identical_keys():
    # identical keys: the logits differ by the bias only, the weights are geometric in the distance
    n, slope = 12, 0.25
    q = rand((1, 4), 8)
    K = np.tile(rand((1, 4), 9), (n, 1))
    V = rand((n, 4), 10)
    vis, bias = variant_mask_and_bias(1, n, False, alibi_slope=slope)
    o, lse = attention_state(q, K, V, 1.0, vis, bias=bias)
    w = np.exp(-slope * np.arange(n - 1, -1, -1.0))       # token t is n - 1 - t behind the query
    assert np.allclose(o[0], (w[:, None] * V).sum(axis=0) / w.sum(), atol=1e-13)
    s = float(q[0] @ K[0])
    assert abs(lse[0] - (s + math.log(w.sum()))) < 1e-12
    o0, l0 = attention_state(q, K, V, 1.0, *variant_mask_and_bias(1, n, False, alibi_slope=0.0)[:1])
    assert np.allclose(o0, V.mean(axis=0)[None, :], atol=1e-13)


def test_all_variants_against_a_pure_python_loop_on_a_paged_batch():
    b = workloads.make_batch("var", 5, workloads.F16, 4, 2, 8, 4, [3, 1, 2], [9, 6, 2], True, sm_scale=0.4)
    slopes = np.array([0.5, 0.25, 0.125, 0.0625])
    cap, W = 1.5, 3
    o, lse = oracle.run_batch(b, logits_soft_cap=cap, window_left=W, alibi_slopes=slopes)
    q = workloads.widen(b.q_bits, b.dtype)
    k = workloads.widen(b.k_bits, b.dtype)
    v = workloads.widen(b.v_bits, b.dtype)
    for i in range(3):
        l_qo = int(b.qo_indptr[i + 1] - b.qo_indptr[i])
        n_pg = int(b.kv_indptr[i + 1] - b.kv_indptr[i])
        l_kv = (n_pg - 1) * 4 + int(b.last_page_len[i])
        for j in range(l_qo):
            row = int(b.qo_indptr[i]) + j
            pos = l_kv - l_qo + j
            for h in range(4):
                num, den, mx = [0.0] * 8, 0.0, -math.inf
                logits = []
                for t in range(l_kv):
                    if t > pos or t < pos - W:
                        continue
                    pg = int(b.kv_indices[int(b.kv_indptr[i]) + t // 4])
                    s = 0.4 * sum(float(q[row, h, d]) * float(k[pg, h // 2, t % 4, d]) for d in range(8))
                    s = cap * math.tanh(s / cap) + float(slopes[h]) * (t - pos)
                    logits.append((s, pg, t))
                    mx = max(mx, s)
                for s, pg, t in logits:
                    w = math.exp(s - mx)
                    den += w
                    for d in range(8):
                        num[d] += w * float(v[pg, h // 2, t % 4, d])
                assert abs(lse[row, h] - (mx + math.log(den))) < 1e-12
                assert all(abs(o[row, h, d] - num[d] / den) < 1e-12 for d in range(8))
