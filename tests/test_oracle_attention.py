"""Pins for the oracle's attention side: brute force on tiny inputs, softmax/RoPE/GQA invariants, the
full-rank special case, associativity of the latent formulation, and prefill <-> decode consistency."""
import math

import numpy as np
import pytest

import lorc_inputs as gen
from oracle import lorc_oracle as orc


def tiny_problem(seed=0, D=24, h_q=4, h_kv=2, d=8, N=9):
    rng = np.random.default_rng(seed)
    W_k, _ = gen.power_law_weight(D, h_kv * d, seed=seed + 100)
    W_v, _ = gen.power_law_weight(D, h_kv * d, seed=seed + 200)
    X = rng.standard_normal((N, D))
    q = rng.standard_normal((h_q, d))
    return W_k, W_v, X, q


# ------------------------------------------------------------------------------ brute force (scalar loops)
def brute_rope(vec, pos, base):
    d = len(vec)
    out = [0.0] * d
    for i in range(d // 2):
        ang = pos * base ** (-2.0 * i / d)
        c, s = math.cos(ang), math.sin(ang)
        out[i] = vec[i] * c - vec[i + d // 2] * s
        out[i + d // 2] = vec[i + d // 2] * c + vec[i] * s
    return out


def brute_decode(X, q, q_pos, Wt_k, Wt_v, h_kv, d, base):
    N, D = X.shape
    h_q = q.shape[0]
    G = h_q // h_kv
    n = h_kv * d
    K = [[sum(X[t][k] * Wt_k[k][c] for k in range(D)) for c in range(n)] for t in range(N)]
    V = [[sum(X[t][k] * Wt_v[k][c] for k in range(D)) for c in range(n)] for t in range(N)]
    out = np.zeros((h_q, d))
    for h in range(h_q):
        g = h // G
        qr = brute_rope(list(q[h]), q_pos, base)
        s = []
        for t in range(N):
            kr = brute_rope(K[t][g * d:(g + 1) * d], t, base)
            s.append(sum(a * b for a, b in zip(qr, kr)) / math.sqrt(d))
        m = max(s)
        e = [math.exp(v - m) for v in s]
        z = sum(e)
        for c in range(d):
            out[h][c] = sum(e[t] / z * V[t][g * d + c] for t in range(N))
    return out


@pytest.mark.parametrize("seed,r", [(0, 5), (1, 16), (2, 1)])
def test_decode_matches_scalar_brute_force(seed, r):
    W_k, W_v, X, q = tiny_problem(seed)
    Wt_k, _ = orc.low_rank_weight(W_k, r)
    Wt_v, _ = orc.low_rank_weight(W_v, r)
    ref = brute_decode(X, q, X.shape[0] - 1, Wt_k, Wt_v, 2, 8, 10000.0)
    got = orc.lorc_decode(X, q, X.shape[0] - 1, W_k, W_v, r, r, 2, 8, 10000.0)
    assert np.max(np.abs(got - ref)) < 1e-12


def test_brute_force_on_config0_shape():
    c = gen.CONFIGS[0]
    D, h_q, h_kv, d, r = c["d_model"], c["n_q_heads"], c["n_kv_heads"], c["head_dim"], c["rank"]
    W_k, _ = gen.power_law_weight(D, h_kv * d, seed=1)
    W_v, _ = gen.power_law_weight(D, h_kv * d, seed=2)
    X = gen.hidden_states(6, D, seed=3).astype(np.float64)
    q = gen.queries(1, h_q, d, seed=4)[0].astype(np.float64)
    Wt_k, _ = orc.low_rank_weight(W_k, r)
    Wt_v, _ = orc.low_rank_weight(W_v, r)
    ref = brute_decode(X, q, 5, Wt_k, Wt_v, h_kv, d, c["rope_base"])
    got = orc.lorc_decode(X, q, 5, W_k, W_v, r, r, h_kv, d, c["rope_base"])
    assert np.max(np.abs(got - ref)) < 1e-12


# ------------------------------------------------------------------------------ full rank == uncompressed
def plain_attention(X, q, q_pos, W_k, W_v, h_kv, d, base):
    """Uncompressed attention written independently of the oracle's helpers (explicit rotation matrices)."""
    N = X.shape[0]
    h_q = q.shape[0]
    G = h_q // h_kv

    def R(pos):
        M = np.zeros((d, d))
        for i in range(d // 2):
            a = pos * base ** (-2.0 * i / d)
            M[i, i] = M[i + d // 2, i + d // 2] = math.cos(a)
            M[i, i + d // 2] = -math.sin(a)
            M[i + d // 2, i] = math.sin(a)
        return M

    K = (X @ W_k).reshape(N, h_kv, d)
    V = (X @ W_v).reshape(N, h_kv, d)
    out = np.zeros((h_q, d))
    for h in range(h_q):
        g = h // G
        qr = R(q_pos) @ q[h]
        s = np.array([(R(t) @ K[t, g]) @ qr for t in range(N)]) / math.sqrt(d)
        p = np.exp(s - s.max())
        p /= p.sum()
        out[h] = p @ V[:, g]
    return out


def test_full_rank_reproduces_uncompressed_attention():
    W_k, W_v, X, q = tiny_problem(5, D=40, h_q=6, h_kv=3, d=8, N=17)
    got = orc.lorc_decode(X, q, 16, W_k, W_v, 24, 24, 3, 8, 10000.0)
    ref = plain_attention(X, q, 16, W_k, W_v, 3, 8, 10000.0)
    assert np.max(np.abs(got - ref)) < 1e-10


def test_truncation_changes_the_answer_by_a_bounded_amount():
    # The rank-r model is an approximation: outputs differ from uncompressed attention, and the K error
    # per token obeys Theorem 1.
    W_k, W_v, X, q = tiny_problem(6, D=40, h_q=4, h_kv=2, d=8, N=12)
    r = 6
    K_full = X @ W_k
    K_lr, _, s_k, _ = orc.compressed_kv(X, W_k, W_v, r, r, 2, 8)
    err = np.linalg.norm(K_full - K_lr.reshape(12, 16), axis=1)
    assert np.all(err <= s_k[r] * np.linalg.norm(X, axis=1) * (1 + 1e-12))
    assert np.max(err) > 1e-3


# ------------------------------------------------------------------------------ associativity
@pytest.mark.parametrize("r_k,r_v", [(4, 4), (7, 3), (16, 16)])
def test_latent_formulation_equals_materialised(r_k, r_v):
    W_k, W_v, X, q = tiny_problem(7)
    A_k, B_k, _ = orc.latent_factors(W_k, r_k)
    A_v, B_v, _ = orc.latent_factors(W_v, r_v)
    Wt_k, _ = orc.low_rank_weight(W_k, r_k)
    assert np.allclose((X @ A_k) @ B_k, X @ Wt_k, atol=1e-11)
    a = orc.lorc_decode(X, q, 8, W_k, W_v, r_k, r_v, 2, 8, 10000.0)
    b = orc.lorc_decode_from_latents(X @ A_k, X @ A_v, B_k, B_v, q, 8, 2, 8, 10000.0)
    assert np.max(np.abs(a - b)) < 1e-10


# ------------------------------------------------------------------------------ softmax invariants
def test_softmax_rows_sum_to_one_and_output_is_convex_combination():
    W_k, W_v, X, q = tiny_problem(8, N=33)
    K, V, _, _ = orc.compressed_kv(X, W_k, W_v, 5, 5, 2, 8)
    P = orc.attention_weights(q, 32, K, np.arange(33), 10000.0)
    assert P.shape == (4, 33)
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-14) and np.all(P >= 0)
    out = orc.attention_decode(q, 32, K, V, np.arange(33), 10000.0)
    for h in range(4):
        g = h // 2
        assert np.all(out[h] <= V[:, g].max(axis=0) + 1e-12)
        assert np.all(out[h] >= V[:, g].min(axis=0) - 1e-12)


def test_single_position_returns_its_value():
    W_k, W_v, X, q = tiny_problem(9, N=1)
    K, V, _, _ = orc.compressed_kv(X, W_k, W_v, 5, 5, 2, 8)
    out = orc.attention_decode(q, 0, K, V, [0], 10000.0)
    assert np.allclose(out, np.repeat(V[0], 2, axis=0), atol=1e-14)


def test_identical_keys_give_uniform_average():
    rng = np.random.default_rng(1)
    N, h_kv, d = 6, 2, 8
    K = np.zeros((N, h_kv, d))   # zero keys stay zero under rotation -> all scores equal
    V = rng.standard_normal((N, h_kv, d))
    q = rng.standard_normal((4, d))
    out = orc.attention_decode(q, 5, K, V, np.arange(N), 10000.0)
    assert np.allclose(out, np.repeat(V.mean(axis=0), 2, axis=0), atol=1e-14)


def test_softmax_is_stable_for_large_scores():
    S = np.array([[1000.0, 1001.0, 999.0]])
    P = orc.softmax_rows(S)
    e = np.exp([-1.0, 0.0, -2.0])
    assert np.allclose(P, e / e.sum())


def test_scale_defaults_to_inverse_sqrt_head_dim():
    W_k, W_v, X, q = tiny_problem(10)
    K, V, _, _ = orc.compressed_kv(X, W_k, W_v, 5, 5, 2, 8)
    a = orc.attention_decode(q, 8, K, V, np.arange(9), 10000.0)
    b = orc.attention_decode(q, 8, K, V, np.arange(9), 10000.0, scale=1 / math.sqrt(8))
    c = orc.attention_decode(q, 8, K, V, np.arange(9), 10000.0, scale=1.0)
    assert np.array_equal(a, b) and not np.allclose(a, c)


# ------------------------------------------------------------------------------ RoPE
def test_rope_is_a_rotation():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 3, 16))
    pos = np.arange(5)[:, None] * np.ones((1, 3)) + 40
    y = orc.apply_rope(x, pos, 500000.0)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))
    assert np.array_equal(orc.apply_rope(x, np.zeros((5, 3)), 500000.0), x)
    # against explicit scalar formula
    for t in range(5):
        assert np.allclose(y[t, 1], brute_rope(list(x[t, 1]), 40 + t, 500000.0), atol=1e-14)


def test_rope_frequencies():
    ang = orc.rope_angles([1, 3], 8, 10000.0)
    assert np.allclose(ang[0], [1.0, 0.1, 0.01, 0.001])
    assert np.allclose(ang[1], [3.0, 0.3, 0.03, 0.003])


def test_rope_scores_depend_only_on_relative_position():
    # q_m . k_n is a function of n - m (Appendix on the adjusted position embedding).
    rng = np.random.default_rng(3)
    q = rng.standard_normal(16)
    k = rng.standard_normal(16)
    s1 = orc.apply_rope(q, 10, 10000.0) @ orc.apply_rope(k, 3, 10000.0)
    s2 = orc.apply_rope(q, 110, 10000.0) @ orc.apply_rope(k, 103, 10000.0)
    s3 = orc.apply_rope(q, 11, 10000.0) @ orc.apply_rope(k, 3, 10000.0)
    assert np.isclose(s1, s2, atol=1e-12) and not np.isclose(s1, s3)


def test_shifting_all_positions_leaves_output_unchanged():
    W_k, W_v, X, q = tiny_problem(11)
    K, V, _, _ = orc.compressed_kv(X, W_k, W_v, 5, 5, 2, 8)
    a = orc.attention_decode(q, 8, K, V, np.arange(9), 10000.0)
    b = orc.attention_decode(q, 8 + 77, K, V, np.arange(9) + 77, 10000.0)
    assert np.max(np.abs(a - b)) < 1e-11


# ------------------------------------------------------------------------------ GQA
def test_gqa_equals_mha_with_repeated_kv_heads():
    W_k, W_v, X, q = tiny_problem(12, h_q=6, h_kv=2)
    K, V, _, _ = orc.compressed_kv(X, W_k, W_v, 5, 5, 2, 8)
    a = orc.attention_decode(q, 8, K, V, np.arange(9), 10000.0)
    K_rep = np.repeat(K, 3, axis=1)   # consecutive query heads share a KV head
    V_rep = np.repeat(V, 3, axis=1)
    b = orc.attention_decode(q, 8, K_rep, V_rep, np.arange(9), 10000.0)
    assert np.array_equal(a, b)


# ------------------------------------------------------------------------------ prefill
def test_prefill_rows_equal_decode_calls():
    rng = np.random.default_rng(13)
    W_k, W_v, X, _ = tiny_problem(13, N=11)
    Q = rng.standard_normal((11, 4, 8))
    full = orc.lorc_prefill(X, Q, W_k, W_v, 6, 6, 2, 8, 10000.0)
    for i in (0, 1, 5, 10):
        one = orc.lorc_decode(X[: i + 1], Q[i], i, W_k, W_v, 6, 6, 2, 8, 10000.0)
        assert np.max(np.abs(full[i] - one)) < 1e-12


def test_prefill_is_causal():
    rng = np.random.default_rng(14)
    W_k, W_v, X, _ = tiny_problem(14, N=8)
    Q = rng.standard_normal((8, 4, 8))
    a = orc.lorc_prefill(X, Q, W_k, W_v, 6, 6, 2, 8, 10000.0)
    X2 = X.copy()
    X2[5:] += 1.0                         # changing later tokens must not change earlier rows
    b = orc.lorc_prefill(X2, Q, W_k, W_v, 6, 6, 2, 8, 10000.0)
    assert np.array_equal(a[:5], b[:5]) and not np.allclose(a[5:], b[5:])


def test_latent_output_times_up_projection_is_the_materialised_decode():
    """Eq. 9 reading: stopping before the value up-projection and applying B_v afterwards gives the rank-r
    model's decode output (pins lorc_decode_latent_output to lorc_decode, which is pinned above); and with a
    single cached position the latent output is that position's value latent for every head."""
    rng = np.random.default_rng(5)
    D, h_q, h_kv, d, r_k, r_v, N = 48, 6, 2, 8, 10, 7, 19
    W_k, W_v = rng.standard_normal((D, h_kv * d)), rng.standard_normal((D, h_kv * d))
    X, q = rng.standard_normal((N, D)), rng.standard_normal((h_q, d))
    A_k, B_k = orc.latent_factors(W_k, r_k)[:2]
    A_v, B_v = orc.latent_factors(W_v, r_v)[:2]
    o_lat = orc.lorc_decode_latent_output(X @ A_k, X @ A_v, B_k, q, N - 1, h_kv, d, 10000.0)
    assert o_lat.shape == (h_q, r_v)
    ref = orc.lorc_decode(X, q, N - 1, W_k, W_v, r_k, r_v, h_kv, d, 10000.0)
    G = h_q // h_kv
    got = np.stack([o_lat[h] @ B_v[:, (h // G) * d:(h // G + 1) * d] for h in range(h_q)])
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)
    one = orc.lorc_decode_latent_output((X @ A_k)[:1], (X @ A_v)[:1], B_k, q, 0, h_kv, d, 10000.0)
    np.testing.assert_allclose(one, np.tile((X @ A_v)[:1], (h_q, 1)), rtol=1e-12)


# ------------------------------------------------------------------------------ Eq. (7): no rotation, absorbed query
def test_plain_attention_is_rope_attention_at_position_zero():
    """A rotation by angle 0 is the identity: with every position 0 the rotary path must give the plain result."""
    W_k, W_v, X, q = tiny_problem(seed=21, N=11)
    K, V, _, _ = orc.compressed_kv(X, W_k, W_v, 6, 5, 2, 8)
    ref = orc.attention_decode(q, 0, K, V, np.zeros(K.shape[0], dtype=np.int64), 10000.0)
    np.testing.assert_allclose(orc.attention_decode_plain(q, K, V), ref, rtol=0, atol=1e-12)


def test_plain_attention_matches_scalar_loops():
    W_k, W_v, X, q = tiny_problem(seed=22, N=7)
    K, V, _, _ = orc.compressed_kv(X, W_k, W_v, 16, 16, 2, 8)
    got = orc.attention_decode_plain(q, K, V)
    h_q, d = q.shape
    for h in range(h_q):
        g = h // 2
        s = [sum(q[h][i] * K[j][g][i] for i in range(d)) / math.sqrt(d) for j in range(K.shape[0])]
        m = max(s)
        e = [math.exp(x - m) for x in s]
        z = sum(e)
        for i in range(d):
            want = sum(e[j] / z * V[j][g][i] for j in range(K.shape[0]))
            assert abs(got[h][i] - want) < 1e-12


@pytest.mark.parametrize("r_k,r_v", [(16, 16), (6, 9), (1, 3)])
def test_absorbed_query_formulation_equals_materialised(r_k, r_v):
    """(B_k^g q) . c = q . (c B_k^g): scores taken in latent space give the materialised no-rotation decode."""
    W_k, W_v, X, q = tiny_problem(seed=23, N=10)
    A_k, B_k = orc.latent_factors(W_k, r_k)[:2]
    A_v, B_v = orc.latent_factors(W_v, r_v)[:2]
    q_lat = orc.absorb_query(q, B_k, 2, 8)
    assert q_lat.shape == (4, r_k)
    got = orc.lorc_decode_absorbed(X @ A_k, X @ A_v, B_v, q_lat, 2, 8)
    ref = orc.lorc_decode_plain(X, q, W_k, W_v, r_k, r_v, 2, 8)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-10)
    # a transposed or mis-blocked factor must not pass: head blocks of B_k differ
    wrong = orc.absorb_query(q[::-1], B_k, 2, 8)
    assert np.abs(orc.lorc_decode_absorbed(X @ A_k, X @ A_v, B_v, wrong, 2, 8) - ref).max() > 1e-6
