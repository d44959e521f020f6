"""Pins for the fp64 attention oracle: brute force on tiny inputs, closed forms,
invariants of the attention-state algebra (Sec. 2.2) and of the paged layout
(Sec. 3.1).  None of these re-types the oracle's own vectorised formula: the
brute force below is scalar Python with `math.exp` / `math.log`."""
import math

import numpy as np
import pytest

import oracle
import workloads
from oracle import attention as A


# ---------------------------------------------------------------------------
# brute force: scalar loops, textbook softmax attention over a paged cache
# ---------------------------------------------------------------------------
def brute_force(batch):
    dt = batch.dtype
    q = workloads.widen(batch.q_bits, dt)
    k = workloads.widen(batch.k_bits, dt)
    v = workloads.widen(batch.v_bits, dt)
    H, Hk, D, ps = batch.num_qo_heads, batch.num_kv_heads, batch.head_dim, batch.page_size
    g = H // Hk
    nnz = q.shape[0]
    o = [[[0.0] * D for _ in range(H)] for _ in range(nnz)]
    lse = [[-math.inf] * H for _ in range(nnz)]
    for i in range(batch.batch):
        n_pg = int(batch.kv_indptr[i + 1] - batch.kv_indptr[i])
        l_kv = 0 if n_pg == 0 else (n_pg - 1) * ps + int(batch.last_page_len[i])
        r0, r1 = int(batch.qo_indptr[i]), int(batch.qo_indptr[i + 1])
        l_qo = r1 - r0
        for j in range(l_qo):
            for h in range(H):
                scores = []
                vals = []
                for t in range(l_kv):
                    if batch.causal and t > l_kv - l_qo + j:
                        continue
                    page = int(batch.kv_indices[int(batch.kv_indptr[i]) + t // ps])
                    dot = 0.0
                    for d in range(D):
                        dot += q[r0 + j, h, d] * k[page, h // g, t % ps, d]
                    scores.append(batch.sm_scale * dot)
                    vals.append(v[page, h // g, t % ps])
                if not scores:
                    continue
                denom = sum(math.exp(s) for s in scores)
                lse[r0 + j][h] = math.log(denom)
                for s, vv in zip(scores, vals):
                    w = math.exp(s) / denom
                    for d in range(D):
                        o[r0 + j][h][d] += w * vv[d]
    return np.array(o), np.array(lse)


@pytest.mark.parametrize("seed,causal,ps,g", [(1, False, 1, 1), (2, False, 2, 2), (3, True, 4, 2),
                                              (4, True, 2, 1), (5, False, 4, 3), (6, True, 1, 2)])
def test_brute_force_tiny(seed, causal, ps, g):
    b = workloads.random_case(seed, dtype=workloads.F16 if seed % 2 else workloads.BF16,
                              num_qo_heads=2 * g, num_kv_heads=2, head_dim=4, page_size=ps, batch=3,
                              max_qo=4 if causal else 1, max_kv=9, causal=causal, value_scale=0.7)
    o, lse = oracle.run_batch(b)
    bo, blse = brute_force(b)
    live = np.isfinite(blse)
    assert np.array_equal(np.isneginf(lse), ~live)
    np.testing.assert_allclose(o, bo, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse[live], blse[live], rtol=0, atol=1e-12)
    assert not np.isnan(o).any()


# ---------------------------------------------------------------------------
# closed forms
# ---------------------------------------------------------------------------
def test_single_key_returns_its_value():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((3, 8)); K = rng.standard_normal((1, 8)); V = rng.standard_normal((1, 8))
    o, lse = A.attention_state(q, K, V, 0.37)
    for r in range(3):
        assert np.array_equal(o[r], V[0])
        assert lse[r] == pytest.approx(0.37 * float(q[r] @ K[0]), abs=1e-14)


def test_identical_keys_return_mean_value():
    rng = np.random.default_rng(1)
    n = 7
    q = rng.standard_normal((2, 8)); k = rng.standard_normal(8); V = rng.standard_normal((n, 8))
    o, lse = A.attention_state(q, np.tile(k, (n, 1)), V, 0.5)
    np.testing.assert_allclose(o, np.tile(V.mean(0), (2, 1)), atol=1e-14)
    np.testing.assert_allclose(lse, 0.5 * (q @ k) + math.log(n), atol=1e-13)


def test_zero_query_returns_mean_value():
    rng = np.random.default_rng(2)
    n = 11
    K = rng.standard_normal((n, 8)); V = rng.standard_normal((n, 8))
    o, lse = A.attention_state(np.zeros((1, 8)), K, V, 1.0)
    np.testing.assert_allclose(o[0], V.mean(0), atol=1e-14)
    assert lse[0] == pytest.approx(math.log(n), abs=1e-14)


def test_two_keys_is_a_sigmoid_blend():
    # softmax over two scores s0, s1 puts weight 1/(1+exp(s1-s0)) on v0
    q = np.array([[1.0, 2.0]]); K = np.array([[0.5, -1.0], [2.0, 0.25]]); V = np.array([[1.0, 0.0], [0.0, 1.0]])
    sc = 0.3
    s0, s1 = sc * (0.5 - 2.0), sc * (2.0 + 0.5)
    w0 = 1.0 / (1.0 + math.exp(s1 - s0))
    o, lse = A.attention_state(q, K, V, sc)
    np.testing.assert_allclose(o[0], [w0, 1 - w0], atol=1e-15)
    assert lse[0] == pytest.approx(math.log(math.exp(s0) + math.exp(s1)), abs=1e-15)


def test_scale_and_operand_orientation():
    # a transposed operand or a dropped scale changes this hand-computable case:
    # q = e0 * a, keys = c_t * e0  ->  scores = sm_scale * a * c_t
    a, sc = 2.0, 0.25
    c = np.array([0.0, 1.0, 3.0])
    q = np.array([[a, 0.0, 0.0]])
    K = np.stack([c, 7 * np.ones(3), -5 * np.ones(3)], axis=1)       # only column 0 may matter
    V = np.array([[1.0, 10.0], [2.0, 20.0], [3.0, 30.0]])
    w = np.exp(sc * a * c); w /= w.sum()
    o, lse = A.attention_state(q, K, V, sc)
    np.testing.assert_allclose(o[0], w @ V, atol=1e-14)
    assert lse[0] == pytest.approx(math.log(np.exp(sc * a * c).sum()), abs=1e-14)


def test_large_scores_do_not_overflow():
    q = np.array([[100.0]]); K = np.array([[10.0], [10.0]]); V = np.array([[1.0], [3.0]])
    o, lse = A.attention_state(q, K, V, 1.0)
    assert o[0, 0] == pytest.approx(2.0) and lse[0] == pytest.approx(1000.0 + math.log(2.0))


def test_empty_set():
    o, lse = A.attention_state(np.ones((2, 4)), np.zeros((0, 4)), np.zeros((0, 4)), 1.0)
    assert np.array_equal(o, np.zeros((2, 4))) and np.all(np.isneginf(lse))


# ---------------------------------------------------------------------------
# merge operator (Sec. 2.2): any split, any order
# ---------------------------------------------------------------------------
def test_merge_every_cut_point_equals_unsplit():
    rng = np.random.default_rng(3)
    n = 13
    q = rng.standard_normal((4, 16)); K = rng.standard_normal((n, 16)); V = rng.standard_normal((n, 16))
    o, lse = A.attention_state(q, K, V, 0.4)
    for cut in range(0, n + 1):
        oa, la = A.attention_state(q, K[:cut], V[:cut], 0.4)
        ob, lb = A.attention_state(q, K[cut:], V[cut:], 0.4)
        om, lm = A.merge_pair(oa, la, ob, lb)
        np.testing.assert_allclose(om, o, atol=1e-12)
        np.testing.assert_allclose(lm, lse, atol=1e-12)
        om2, lm2 = A.merge_pair(ob, lb, oa, la)          # commutative
        np.testing.assert_allclose(om2, o, atol=1e-12)
        np.testing.assert_allclose(lm2, lse, atol=1e-12)


def test_merge_many_pieces_shuffled_order():
    rng = np.random.default_rng(4)
    n = 40
    q = rng.standard_normal((3, 8)); K = rng.standard_normal((n, 8)); V = rng.standard_normal((n, 8))
    o, lse = A.attention_state(q, K, V, 0.3)
    for trial in range(5):
        cuts = np.sort(rng.choice(np.arange(1, n), size=4, replace=False))
        pieces = np.split(np.arange(n), cuts)
        rng.shuffle(pieces)
        states = [A.attention_state(q, K[p], V[p], 0.3) for p in pieces]
        op = np.stack([s[0] for s in states], axis=1)
        lp = np.stack([s[1] for s in states], axis=1)
        om, lm = A.merge_states(op, lp)
        np.testing.assert_allclose(om, o, atol=1e-12)
        np.testing.assert_allclose(lm, lse, atol=1e-12)


def test_merge_two_states_by_hand():
    # weights exp(lse) = 1 and 3  ->  o = (1*oa + 3*ob)/4, lse = log 4
    o, lse = A.merge_pair(np.array([[4.0, 0.0]]), np.array([0.0]), np.array([[0.0, 8.0]]), np.array([math.log(3.0)]))
    np.testing.assert_allclose(o, [[1.0, 6.0]], atol=1e-15)
    assert lse[0] == pytest.approx(math.log(4.0), abs=1e-15)


def test_merge_identity_and_both_empty():
    oa = np.array([[1.0, 2.0]]); la = np.array([0.7])
    z = np.zeros((1, 2)); ninf = np.array([-np.inf])
    for (x, y) in (((oa, la), (z, ninf)), ((z, ninf), (oa, la))):
        o, lse = A.merge_pair(x[0], x[1], y[0], y[1])
        assert np.array_equal(o, oa) and np.array_equal(lse, la)
    o, lse = A.merge_pair(z, ninf, z, ninf)
    assert np.array_equal(o, z) and np.isneginf(lse[0])
    # garbage (even NaN) riding on an empty state must not leak: weight is exactly 0 only if finite
    o, lse = A.merge_pair(oa, la, np.array([[5.0, -5.0]]), ninf)
    assert np.array_equal(o, oa)


# ---------------------------------------------------------------------------
# paging (Sec. 3.1.1)
# ---------------------------------------------------------------------------
def _dense_reference(batch, i, h):
    """Dense K/V of request i built by scalar indexing (independent of gather_rows)."""
    dt = batch.dtype
    ps = batch.page_size
    g = batch.num_qo_heads // batch.num_kv_heads
    l_kv = int(batch.kv_lens()[i])
    rows_k, rows_v = [], []
    for t in range(l_kv):
        pg = int(batch.kv_indices[int(batch.kv_indptr[i]) + t // ps])
        rows_k.append(workloads.widen(batch.k_bits[pg, h // g, t % ps], dt))
        rows_v.append(workloads.widen(batch.v_bits[pg, h // g, t % ps], dt))
    D = batch.head_dim
    return (np.array(rows_k).reshape(l_kv, D), np.array(rows_v).reshape(l_kv, D))


def test_gather_matches_scalar_indexing_and_poison_never_leaks():
    b = workloads.random_case(11, batch=4, max_kv=70, num_qo_heads=4, num_kv_heads=2, head_dim=8)
    assert np.isnan(workloads.widen(b.k_bits, b.dtype)).any()     # the pool is poisoned
    o, lse = oracle.run_batch(b)
    assert not np.isnan(o).any() and not np.isnan(lse).any()
    q = workloads.widen(b.q_bits, b.dtype)
    for i in range(b.batch):
        for h in range(4):
            K, V = _dense_reference(b, i, h)
            oo, ll = A.attention_state(q[b.qo_indptr[i]:b.qo_indptr[i + 1], h], K, V, b.sm_scale)
            np.testing.assert_array_equal(o[b.qo_indptr[i]:b.qo_indptr[i + 1], h], oo)


def test_page_permutation_invariance():
    b = workloads.random_case(12, batch=4, max_kv=90, num_qo_heads=4, num_kv_heads=2, head_dim=8)
    o, lse = oracle.run_batch(b)
    rng = np.random.default_rng(5)
    perm = rng.permutation(b.num_pages)            # new_id = perm[old_id]
    k2 = np.empty_like(b.k_bits); v2 = np.empty_like(b.v_bits)
    k2[perm] = b.k_bits; v2[perm] = b.v_bits
    import dataclasses
    b2 = dataclasses.replace(b, k_bits=k2, v_bits=v2, kv_indices=perm[b.kv_indices].astype(np.int32))
    o2, lse2 = oracle.run_batch(b2)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)


def test_identity_page_table_equals_dense_attention():
    b = workloads.make_batch("dense", 13, workloads.F16, 2, 2, 8, 4, [1, 1], [12, 7], False,
                             permute_pages=False, poison=True)
    assert np.array_equal(b.kv_indices, np.arange(5))
    o, lse = oracle.run_batch(b)
    k = workloads.widen(b.k_bits, b.dtype); v = workloads.widen(b.v_bits, b.dtype)
    q = workloads.widen(b.q_bits, b.dtype)
    for h in range(2):
        K0 = k[0:3, h].reshape(12, 8); V0 = v[0:3, h].reshape(12, 8)
        K1 = k[3:5, h].reshape(8, 8)[:7]; V1 = v[3:5, h].reshape(8, 8)[:7]
        np.testing.assert_array_equal(o[0, h], A.attention_state(q[0:1, h], K0, V0, b.sm_scale)[0][0])
        np.testing.assert_array_equal(o[1, h], A.attention_state(q[1:2, h], K1, V1, b.sm_scale)[0][0])


# ---------------------------------------------------------------------------
# causal masking: bottom-right aligned (appended tokens are already cached)
# ---------------------------------------------------------------------------
def test_causal_square_equals_lower_triangular_softmax():
    rng = np.random.default_rng(6)
    n = 9
    q = rng.standard_normal((n, 8)); K = rng.standard_normal((n, 8)); V = rng.standard_normal((n, 8))
    o, lse = A.attention_state(q, K, V, 0.5, A.causal_visible(n, n))
    s = 0.5 * q @ K.T
    for j in range(n):
        w = np.exp(s[j, :j + 1]); w /= w.sum()
        np.testing.assert_allclose(o[j], w @ V[:j + 1], atol=1e-13)


def test_causal_row_equals_decode_at_shorter_length():
    b = workloads.random_case(14, batch=3, max_qo=6, max_kv=40, causal=True, num_qo_heads=4,
                              num_kv_heads=2, head_dim=8, page_size=4)
    o, lse = oracle.run_batch(b)
    q = workloads.widen(b.q_bits, b.dtype)
    for i in range(b.batch):
        l_qo = int(b.qo_lens()[i]); l_kv = int(b.kv_lens()[i])
        for j in range(l_qo):
            for h in range(4):
                K, V = _dense_reference(b, i, h)
                n_vis = l_kv - l_qo + j + 1
                oo, ll = A.attention_state(q[b.qo_indptr[i] + j:b.qo_indptr[i] + j + 1, h], K[:n_vis], V[:n_vis], b.sm_scale)
                np.testing.assert_allclose(o[b.qo_indptr[i] + j, h], oo[0], atol=1e-13)
                assert lse[b.qo_indptr[i] + j, h] == pytest.approx(ll[0], abs=1e-13)


def test_causal_more_queries_than_keys_gives_empty_rows():
    vis = A.causal_visible(5, 3)           # rows 0,1 see nothing; row 2 sees key 0
    assert not vis[0].any() and not vis[1].any() and vis[2].tolist() == [True, False, False]
    o, lse = A.attention_state(np.ones((5, 2)), np.ones((3, 2)), np.ones((3, 2)), 1.0, vis)
    assert np.isneginf(lse[:2]).all() and np.isfinite(lse[2:]).all() and not np.isnan(o).any()


# ---------------------------------------------------------------------------
# head-group fusion (App. A) is only a re-indexing; composable formats (Sec. 3.1.2)
# ---------------------------------------------------------------------------
def test_gqa_equals_mha_with_repeated_kv_heads():
    import dataclasses
    b = workloads.random_case(15, batch=3, max_kv=50, num_qo_heads=6, num_kv_heads=2, head_dim=8)
    o, lse = oracle.run_batch(b)
    b2 = dataclasses.replace(b, num_kv_heads=6, k_bits=np.repeat(b.k_bits, 3, axis=1),
                             v_bits=np.repeat(b.v_bits, 3, axis=1))
    o2, lse2 = oracle.run_batch(b2)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)


def test_shared_prefix_composition_equals_single_format():
    c = workloads.config5(small=True)
    o1, l1 = oracle.run_batch(c.single)
    op, lp = oracle.run_batch(c.prefix)
    os_, ls = oracle.run_batch(c.suffix)
    om, lm = A.merge_pair(op, lp, os_, ls)
    np.testing.assert_allclose(om, o1, atol=1e-12)
    np.testing.assert_allclose(lm, l1, atol=1e-12)


def test_second_opinion_torch_sdpa_fp64_dense():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(7)
    q = rng.standard_normal((5, 16)); K = rng.standard_normal((23, 16)); V = rng.standard_normal((23, 16))
    o, _ = A.attention_state(q, K, V, 0.25)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None], scale=0.25)[0].numpy()
    np.testing.assert_allclose(o, ref, atol=1e-13)
