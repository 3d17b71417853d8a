"""Pins for the oracle's factorisation side: Eckart-Young, Theorem 1, relative Frobenius error, the rank
schedule of Section 4.2, and the memory accounting the paper prints."""
import numpy as np
import pytest

import lorc_inputs as gen
from oracle import lorc_oracle as orc


@pytest.fixture(scope="module")
def small_w():
    return gen.power_law_weight(96, 48, seed=11)


def test_generator_spectrum_is_what_it_says(small_w):
    W, sigma = small_w
    s = np.linalg.svd(W, compute_uv=False)
    assert np.allclose(s, sigma, rtol=1e-12, atol=1e-13)
    assert np.isclose(np.sum(W * W), 48.0)
    assert np.all(np.diff(sigma) < 0)


@pytest.mark.parametrize("r", [1, 7, 24, 47])
def test_eckart_young_spectral_and_frobenius(small_w, r):
    # Residual of the truncated SVD is diag(0,...,0,sigma_{r+1},...) in the singular bases (proof of Thm 1).
    W, sigma = small_w
    Wt, s = orc.low_rank_weight(W, r)
    R = W - Wt
    assert np.isclose(np.linalg.norm(R, 2), sigma[r], rtol=1e-10)
    assert np.isclose(np.sum(R * R), np.sum(sigma[r:] ** 2), rtol=1e-10)
    assert np.linalg.matrix_rank(Wt, tol=1e-9) == r


def test_truncation_is_best_rank_r(small_w):
    # Eckart-Young optimality: random rank-r matrices and perturbed factors never beat the truncation.
    W, _ = small_w
    r = 10
    Wt, _ = orc.low_rank_weight(W, r)
    best = np.linalg.norm(W - Wt, "fro")
    rng = np.random.default_rng(0)
    A, B, _ = orc.latent_factors(W, r)
    for _ in range(20):
        A2 = A + 1e-3 * rng.standard_normal(A.shape)
        B2 = B + 1e-3 * rng.standard_normal(B.shape)
        assert np.linalg.norm(W - A2 @ B2, "fro") >= best - 1e-12


@pytest.mark.parametrize("n,r,expected", [(1024, 512, 0.1300), (1024, 768, 0.0803), (1024, 384, 0.1594), (128, 32, 0.3092)])
def test_relative_frobenius_error_closed_form(n, r, expected):
    # Under sigma_i ~ i^-0.7 the relative error is sqrt(sum_{i>r} i^-1.4 / sum_i i^-1.4).
    i = np.arange(1, n + 1, dtype=np.float64)
    closed = np.sqrt(np.sum(i[r:] ** -1.4) / np.sum(i ** -1.4))
    assert abs(closed - expected) < 5e-4
    rows = 2 * n if n <= 128 else n  # keep the SVD cheap
    W, _ = gen.power_law_weight(rows, n, seed=5)
    Wt, _ = orc.low_rank_weight(W, r)
    assert np.isclose(orc.rel_frobenius_error(W, Wt), closed, rtol=1e-9)


def test_theorem1_bound(small_w):
    # ||x W - x W~||_2 <= sigma_{r+1} ||x||_2, and the bound is attained along the (r+1)-th left vector.
    W, sigma = small_w
    r = 12
    Wt, _ = orc.low_rank_weight(W, r)
    rng = np.random.default_rng(3)
    for _ in range(50):
        x = rng.standard_normal(W.shape[0])
        assert np.linalg.norm(x @ W - x @ Wt) <= sigma[r] * np.linalg.norm(x) * (1 + 1e-12)
    U, _, _ = orc.svd(W)
    x = U[:, r]
    assert np.isclose(np.linalg.norm(x @ W - x @ Wt), sigma[r], rtol=1e-10)


def test_latent_factors_reproduce_low_rank_weight(small_w):
    W, sigma = small_w
    r = 16
    A, B, s = orc.latent_factors(W, r)
    Wt, _ = orc.low_rank_weight(W, r)
    assert A.shape == (96, r) and B.shape == (r, 48)
    assert np.allclose(A @ B, Wt, atol=1e-12)
    assert np.allclose(B @ B.T, np.eye(r), atol=1e-12)          # read-side factor has orthonormal rows
    assert np.allclose(np.linalg.norm(A, axis=0), sigma[:r])    # singular values travel with the latent
    assert np.allclose(s, sigma)


def test_full_rank_is_lossless(small_w):
    W, _ = small_w
    Wt, _ = orc.low_rank_weight(W, 48)
    assert np.max(np.abs(W - Wt)) < 1e-12


# ------------------------------------------------------------------------------ accounting pins
def _records(golden_dir, tag):
    out = []
    with open(f"{golden_dir}/paper_tables.txt") as f:
        for line in f:
            line = line.split("#")[0].split()
            if line and line[0] == tag:
                out.append(line[1:])
    return out


def test_table2_memory_footprint(golden_dir):
    recs = _records(golden_dir, "table2")
    assert len(recs) == 3
    for model, width, dim_c, layers, full_gib, ours_gib, ratio in recs:
        width, dim_c, layers = int(width), int(dim_c), int(layers)
        # Eq. (4) with h*d = width, 16-bit elements, summed over layers, one of K or V.
        elems = orc.kv_cache_elements(64, 2048, 1, width) * layers
        assert elems * 2 / 2 ** 30 == pytest.approx(float(full_gib), rel=1e-12), model
        assert float(full_gib) * float(ratio) == pytest.approx(float(ours_gib), rel=1e-9), model


def test_table1_caption_overall_ratios(golden_dir):
    recs = _records(golden_dir, "table1_caption")
    assert len(recs) == 2
    for case, frac, layer_ratio, overall_pct in recs:
        L = 32
        k = round(float(frac) * L)
        ratios = [float(layer_ratio)] * k + [1.0] * (L - k)
        assert round(100 * orc.overall_ratio(ratios), 2) == float(overall_pct), case


def test_layer_ratio_matches_table2(golden_dir):
    for model, width, dim_c, *_ in _records(golden_dir, "table2"):
        rho = orc.layer_ratio(int(dim_c), 1, int(width))
        assert rho == int(dim_c) / int(width)
    assert orc.layer_ratio(512, 8, 128) == 0.5


def test_workload_shapes_match_table3(golden_dir):
    recs = {r[0]: [int(v) for v in r[1:]] for r in _records(golden_dir, "table3")}
    c1, c4 = gen.CONFIGS[1], gen.CONFIGS[4]
    assert [c1["n_q_heads"], c1["n_kv_heads"], c1["head_dim"], c1["d_model"]] == recs["llama3-8b"][1:5]
    assert [c4["n_q_heads"], c4["n_kv_heads"], c4["head_dim"], c4["d_model"]] == recs["llama3-70b"][1:5]
    assert recs["llama3-8b"][6] == c1["n_kv_heads"] * c1["head_dim"]


# ------------------------------------------------------------------------------ rank schedule (Section 4.2)
def test_condition_number_definition():
    assert orc.condition_number([4.0, 2.0, 0.5]) == 8.0
    assert orc.condition_number([1.0, 0.0]) == np.inf
    W, sigma = gen.power_law_weight(40, 20, seed=2)
    # kappa = ||W||_2 ||W^+||_2 for a full-column-rank matrix
    k = np.linalg.norm(W, 2) * np.linalg.norm(np.linalg.pinv(W), 2)
    assert np.isclose(orc.condition_number(np.linalg.svd(W, compute_uv=False)), k, rtol=1e-9)


def test_cumulative_condition_is_suffix_product():
    kk = np.array([2.0, 3.0, 5.0])
    kv = np.array([7.0, 11.0, 13.0])
    lc = orc.cumulative_log_condition(kk, kv)
    expect = [2 * 7 * 3 * 11 * 5 * 13, 3 * 11 * 5 * 13, 5 * 13]
    assert np.allclose(np.exp(lc), expect)


def test_compression_dims_endpoints_and_monotone():
    rng = np.random.default_rng(7)
    for _ in range(10):
        L = 12
        kk = 1.0 + rng.random(L) * 50
        kv = 1.0 + rng.random(L) * 50
        lc = orc.cumulative_log_condition(kk, kv)
        assert np.all(np.diff(lc) <= 0)                 # every kappa >= 1, so the suffix product shrinks
        d = orc.compression_dims(lc, d_max=1024, d_min=384)
        assert np.isclose(d[0], 1024) and np.isclose(d[-1], 384)
        assert np.all(np.diff(d) <= 1e-9)               # progressive: shallow layers keep more
    # hand-computed instance of Eq. (dc): log kappa~ = [3, 2, 0] -> d = 100*[1-(0, 1/3, 1)*(1-0.4)]
    d = orc.compression_dims(np.array([3.0, 2.0, 0.0]), d_max=100, d_min=40)
    assert np.allclose(d, [100.0, 80.0, 40.0])
    assert np.allclose(orc.compression_dims(np.array([1.0, 1.0]), 64, 16), [64.0, 64.0])


def test_round_dims_and_ramp_generator():
    assert list(orc.round_dims([100.0, 80.0, 47.9, 16.0], 32, 32, 96)) == [96, 96, 32, 32]
    ramp = gen.rank_ramp(32, 768, 384)
    assert ramp[0] == 768 and ramp[-1] == 384 and all(r % 32 == 0 for r in ramp)
    assert all(a >= b for a, b in zip(ramp, ramp[1:]))
    assert sum(ramp) / 32 == 576


# ------------------------------------------------------------------------------ Theorems 1 and 3 (error bounds)
def test_error_bound_of_one_layer_is_the_first_dropped_singular_value():
    s = np.array([5.0, 3.0, 2.0, 0.5])
    assert orc.truncation_error_constant(s, 2) == 2.0
    assert orc.truncation_error_constant(s, 4) == 0.0
    bound, terms = orc.network_error_bound([s], [1])
    assert bound == 3.0 and terms.tolist() == [3.0]


def test_error_bound_hand_computed_three_layers():
    """sum_i sigma_{k_i+1} L^(L-i) prod_{j>i} sigma_1^{(j)}, by hand for L = 3, L_phi = 2."""
    s1, s2, s3 = np.array([4.0, 2.0, 1.0]), np.array([3.0, 0.5, 0.25]), np.array([2.0, 1.5, 0.1])
    bound, terms = orc.network_error_bound([s1, s2, s3], [1, 2, 1], lipschitz=2.0)
    want = [2.0 * 2.0 ** 2 * 3.0 * 2.0, 0.25 * 2.0 * 2.0, 1.5]
    np.testing.assert_allclose(terms, want, rtol=0, atol=1e-15)
    assert abs(bound - sum(want)) < 1e-14
    # a transposed product (norms of the layers before i instead of after) must not pass
    assert abs(bound - (2.0 + 0.25 * 2.0 * 4.0 + 1.5 * 4.0 * 4.0 * 3.0)) > 1.0


def test_error_bound_holds_on_a_simulated_relu_network():
    """Layer inputs of norm <= 1 (weights scaled to spectral norm <= 1, ReLU is 1-Lipschitz with phi(0) = 0): the
    measured output error of the truncated network must stay below the bound, and be of its order for some input."""
    rng = np.random.default_rng(5)
    L, n = 4, 24
    Ws, sig, ranks = [], [], [6, 10, 4, 12]
    for i in range(L):
        W, _ = gen.power_law_weight(n, n, seed=300 + i)
        W = W / (np.linalg.svd(W, compute_uv=False)[0] * 1.25)      # spectral norm 0.8
        Ws.append(W)
        sig.append(np.linalg.svd(W, compute_uv=False))
    Wt = [orc.low_rank_weight(W, r)[0] for W, r in zip(Ws, ranks)]
    bound, _ = orc.network_error_bound(sig, ranks)
    worst = 0.0
    for _ in range(200):
        x = rng.standard_normal(n)
        x /= np.linalg.norm(x)
        a, b = x.copy(), x.copy()
        for W, V in zip(Ws, Wt):
            a, b = np.maximum(a @ W, 0.0), np.maximum(b @ V, 0.0)
        worst = max(worst, float(np.linalg.norm(a - b)))
    assert worst <= bound
    assert worst >= 1e-3 * bound
