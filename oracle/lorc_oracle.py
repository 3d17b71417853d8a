"""CPU oracle for LoRC attention over a rank-r KV cache.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy.  It writes out the *definition* of what the GPU path must produce: factor the
K/V projection weights by truncated SVD, materialise the full rank-r keys and values, rotate, and run dense
softmax attention.  It shares no code with the HIP library and must only be imported by the tests, the
smoke check and the benchmark's CPU-baseline leg.

Paper passages followed (LoRC, arXiv 2410.03111):
  * attention                     -- Preliminary section, Eq. (1)
  * KV-cache size                 -- Preliminary section, Eq. (4)
  * truncated SVD of W_k / W_v    -- Section 4.1 (key / value matrix compression), Algorithm 1
  * layer compression ratio       -- Section 4.1, "Compression Ratio"
  * condition numbers, d_c^l      -- Section 4.2, Eq. (10), Eq. (12), Eq. (dc)
  * GQA repeat                    -- Section 4.3
  * un-rotated latents, RoPE at read time -- Appendix "Adjusted Position Embedding"
  * Theorem 1 / relative Frobenius error  -- Section 5.1, Appendix B

Conventions: K = X W with W of shape [D, n], n = h_kv * d; the n columns are h_kv contiguous blocks of d.
RoPE pairs coordinate i with i + d/2, theta_i = base**(-2 i / d); query head h reads KV head h // G.
All pins for these functions live in tests/test_oracle_*.py.  Parity pins: every function below is pinned
except the accuracy experiments of the paper, which are out of scope.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# =============================================================================== Section 4.1 / Algorithm 1
def svd(W):
    """Thin SVD W = U diag(s) Vt (LAPACK)."""
    return np.linalg.svd(np.asarray(W, F64), full_matrices=False)


def truncate(U, s, Vt, r):
    """Keep the first r singular triplets: U[:, :r], s[:r], Vt[:r, :] (Algorithm 1, truncation steps)."""
    return U[:, :r], s[:r], Vt[:r, :]


def low_rank_weight(W, r):
    """W~ = U_r diag(s_r) Vt_r, the rank-r approximation the method substitutes for W.  Returns (W~, s_all)."""
    U, s, Vt = svd(W)
    Ur, sr, Vtr = truncate(U, s, Vt, r)
    return (Ur * sr) @ Vtr, s


def latent_factors(W, r):
    """Down-/up-projection pair with W~ = A @ B: A = U_r diag(s_r) (applied when a token is cached, so the
    singular values travel with the cached quantity as in Section 4.1) and B = Vt_r (applied at read)."""
    U, s, Vt = svd(W)
    Ur, sr, Vtr = truncate(U, s, Vt, r)
    return Ur * sr, Vtr, s


def rel_frobenius_error(M, M_hat):
    """epsilon = ||M - M^||_F / ||M||_F (Appendix B)."""
    M = np.asarray(M, F64)
    return np.linalg.norm(M - np.asarray(M_hat, F64), "fro") / np.linalg.norm(M, "fro")


def layer_ratio(d_c, n_kv_heads, head_dim):
    """rho = d_c / (h d) (Section 4.1, compression ratio)."""
    return d_c / (n_kv_heads * head_dim)


def overall_ratio(layer_ratios):
    """Model-level ratio = mean of the per-layer ratios (uncompressed layers count as 1)."""
    return float(np.mean(np.asarray(layer_ratios, F64)))


def kv_cache_elements(batch, seq_len, n_kv_heads, head_dim):
    """C_{k,v} = b N h d per layer, for one of K or V (Eq. 4)."""
    return batch * seq_len * n_kv_heads * head_dim


# =============================================================================== Section 4.2
def condition_number(sigma):
    """kappa = sigma_max / sigma_min (Eq. 10); +inf for a singular matrix."""
    sigma = np.asarray(sigma, F64)
    smin = sigma.min()
    return np.inf if smin == 0 else sigma.max() / smin


def cumulative_log_condition(kappa_k, kappa_v):
    """log kappa~_l, kappa~_l = prod_{j>=l} kappa(W_k^j) kappa(W_v^j) (Eq. 12), layers indexed 0..L-1."""
    logs = np.log(np.asarray(kappa_k, F64)) + np.log(np.asarray(kappa_v, F64))
    return np.cumsum(logs[::-1])[::-1]


def compression_dims(log_cum_kappa, d_max, d_min):
    """Real-valued d_c^l of Eq. (dc).  A constant profile (max == min) keeps d_max."""
    lk = np.asarray(log_cum_kappa, F64)
    hi, lo = lk.max(), lk.min()
    if hi == lo:
        return np.full(lk.shape, float(d_max))
    return d_max * (1.0 - (hi - lk) / (hi - lo) * (1.0 - d_min / d_max))


def round_dims(d_c, align, d_min, d_max):
    """Integer ranks: nearest multiple of `align` (ties away from zero), clamped to [d_min, d_max]."""
    q = np.floor(np.asarray(d_c, F64) / align + 0.5) * align
    return np.clip(q, d_min, d_max).astype(np.int64)


# =============================================================================== Appendix C (RoPE)
def rope_angles(pos, head_dim, base):
    """angle[p, i] = pos_p * base**(-2 i / d), i in [0, d/2)."""
    i = np.arange(head_dim // 2, dtype=F64)
    theta = F64(base) ** (-2.0 * i / head_dim)
    return np.asarray(pos, F64)[..., None] * theta


def apply_rope(x, pos, base):
    """Rotate x[..., d] at integer positions pos (broadcast over the leading axes of x except the last).

    Pair (i, i + d/2):  x'_i = x_i cos - x_{i+d/2} sin,  x'_{i+d/2} = x_{i+d/2} cos + x_i sin.
    """
    x = np.asarray(x, F64)
    d = x.shape[-1]
    ang = rope_angles(pos, d, base)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., : d // 2], x[..., d // 2:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


# =============================================================================== Eq. (1), Section 4.3
def softmax_rows(S):
    """Max-subtracted softmax over the last axis."""
    S = np.asarray(S, F64)
    E = np.exp(S - S.max(axis=-1, keepdims=True))
    return E / E.sum(axis=-1, keepdims=True)


def split_heads(M, n_heads, head_dim):
    """[N, n_heads*head_dim] -> [N, n_heads, head_dim]: head g owns columns g*d .. (g+1)*d."""
    return np.asarray(M, F64).reshape(M.shape[0], n_heads, head_dim)


def attention_weights(q, q_pos, K, k_pos, rope_base, scale=None):
    """P[h, j] for one query token: q[h_q, d] (un-rotated), K[N, h_kv, d] (un-rotated), positions given.

    Keys and the query are rotated here (the cache stores un-rotated quantities); query head h uses KV head
    h // G.
    """
    q = np.asarray(q, F64)
    h_q, d = q.shape
    N, h_kv, _ = K.shape
    G = h_q // h_kv
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    q_rot = apply_rope(q, np.full((h_q,), q_pos), rope_base)                  # [h_q, d]
    K_rot = apply_rope(K, np.asarray(k_pos)[:, None] * np.ones((1, h_kv)), rope_base)   # [N, h_kv, d]
    P = np.empty((h_q, N), F64)
    for h in range(h_q):
        P[h] = softmax_rows((K_rot[:, h // G, :] @ q_rot[h]) * scale)
    return P


def attention_decode(q, q_pos, K, V, k_pos, rope_base, scale=None):
    """out[h_q, d] = softmax(q_rot K_rot^T / sqrt(d)) V for one query token over N cached positions."""
    P = attention_weights(q, q_pos, K, k_pos, rope_base, scale)
    h_q = P.shape[0]
    G = h_q // K.shape[1]
    V = np.asarray(V, F64)
    return np.stack([P[h] @ V[:, h // G, :] for h in range(h_q)])


def attention_prefill(q, K, V, rope_base, scale=None, first_pos=0):
    """Causal attention for one sequence: token i (position first_pos + i) attends to tokens j <= i.

    q[T, h_q, d], K,V[T, h_kv, d] -> out[T, h_q, d].
    """
    q = np.asarray(q, F64)
    T, h_q, d = q.shape
    h_kv = K.shape[1]
    G = h_q // h_kv
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    pos = first_pos + np.arange(T)
    q_rot = apply_rope(q, pos[:, None] * np.ones((1, h_q)), rope_base)
    K_rot = apply_rope(K, pos[:, None] * np.ones((1, h_kv)), rope_base)
    V = np.asarray(V, F64)
    out = np.empty((T, h_q, d), F64)
    mask = np.tril(np.ones((T, T), bool))
    for h in range(h_q):
        S = (q_rot[:, h, :] @ K_rot[:, h // G, :].T) * scale
        S = np.where(mask, S, -np.inf)
        out[:, h, :] = softmax_rows(S) @ V[:, h // G, :]
    return out


# =============================================================================== the method end to end
def compressed_kv(X, W_k, W_v, r_k, r_v, n_kv_heads, head_dim):
    """K~ = X W~_k and V~ = X W~_v, reshaped to heads.  Returns (K~, V~, s_k, s_v)."""
    Wt_k, s_k = low_rank_weight(W_k, r_k)
    Wt_v, s_v = low_rank_weight(W_v, r_v)
    X = np.asarray(X, F64)
    return (split_heads(X @ Wt_k, n_kv_heads, head_dim), split_heads(X @ Wt_v, n_kv_heads, head_dim), s_k, s_v)


def lorc_decode(X_ctx, q, q_pos, W_k, W_v, r_k, r_v, n_kv_heads, head_dim, rope_base, scale=None):
    """One decode step of one sequence: context hidden states X_ctx[N, D] (token j at position j), query
    q[h_q, d] at position q_pos.  Rank-r K/V are materialised and fed to plain attention."""
    K, V, _, _ = compressed_kv(X_ctx, W_k, W_v, r_k, r_v, n_kv_heads, head_dim)
    return attention_decode(q, q_pos, K, V, np.arange(K.shape[0]), rope_base, scale)


def lorc_prefill(X, q, W_k, W_v, r_k, r_v, n_kv_heads, head_dim, rope_base, scale=None):
    """Causal prefill of one sequence under the rank-r model."""
    K, V, _, _ = compressed_kv(X, W_k, W_v, r_k, r_v, n_kv_heads, head_dim)
    return attention_prefill(q, K, V, rope_base, scale)


def lorc_decode_from_latents(C_k, C_v, B_k, B_v, q, q_pos, n_kv_heads, head_dim, rope_base, scale=None):
    """Same decode step written on the cached quantities: C_k[N, r_k], C_v[N, r_v] latents, K = C_k B_k,
    and the value up-projection applied after the weighted sum, (P C_v) B_v.  Equal to lorc_decode by
    associativity; exists so that the tests can tie the cached formulation to the materialised one and so
    that externally produced latents (e.g. read back from a device cache) can be evaluated."""
    C_k, C_v, B_k, B_v = (np.asarray(a, F64) for a in (C_k, C_v, B_k, B_v))
    K = split_heads(C_k @ B_k, n_kv_heads, head_dim)
    N = K.shape[0]
    P = attention_weights(q, q_pos, K, np.arange(N), rope_base, scale)
    h_q = P.shape[0]
    G = h_q // n_kv_heads
    o_lat = P @ C_v                                                  # [h_q, r_v]
    out = np.empty((h_q, head_dim), F64)
    for h in range(h_q):
        g = h // G
        out[h] = o_lat[h] @ B_v[:, g * head_dim:(g + 1) * head_dim]
    return out


def lorc_decode_latent_output(C_k, C_v, B_k, q, q_pos, n_kv_heads, head_dim, rope_base, scale=None):
    """Decode step that stops before the value up-projection (Section 4.1, Eq. 9: U^T can be absorbed into
    W_o): o_lat[h] = sum_j P[h, j] C_v[j], with P the attention weights of Eq. (1) on K = C_k B_k.  Then
    o_lat[h] @ B_v[:, head block of h] is the output of lorc_decode_from_latents."""
    N = C_k.shape[0]
    K = split_heads(np.asarray(C_k, F64) @ np.asarray(B_k, F64), n_kv_heads, head_dim)
    P = attention_weights(q, q_pos, K, np.arange(N), rope_base, scale)
    return P @ np.asarray(C_v, F64)



# =============================================================================== Section 4.1, Eq. (7)
# The key factor can be folded into the query projection when nothing position-dependent sits between q and k
# (no rotary embedding): q . (c B_k^g) = (B_k^g q) . c.  The functions below are that setting.
def attention_decode_plain(q, K, V, scale=None):
    """Eq. (1) for one query token without any positional rotation: out[h] = softmax(q[h] K_g^T * scale) V_g,
    q[h_q, d], K, V[N, h_kv, d], query head h uses KV head h // G."""
    q, K, V = (np.asarray(a, F64) for a in (q, K, V))
    h_q, d = q.shape
    G = h_q // K.shape[1]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    out = np.empty((h_q, d), F64)
    for h in range(h_q):
        out[h] = softmax_rows((K[:, h // G, :] @ q[h]) * scale) @ V[:, h // G, :]
    return out


def lorc_decode_plain(X_ctx, q, W_k, W_v, r_k, r_v, n_kv_heads, head_dim, scale=None):
    """One decode step of one sequence under the rank-r model with no positional rotation: rank-r K, V are
    materialised and fed to attention_decode_plain."""
    K, V, _, _ = compressed_kv(X_ctx, W_k, W_v, r_k, r_v, n_kv_heads, head_dim)
    return attention_decode_plain(q, K, V, scale)


def absorb_query(q, B_k, n_kv_heads, head_dim):
    """Eq. (7): the read-side key factor folded into the query.  q[h_q, d], B_k[r_k, n_kv_heads * d] ->
    q_lat[h_q, r_k] with q_lat[h] = B_k[:, head block of h // G] q[h], so that q_lat[h] . c = q[h] . (c B_k^g)."""
    q, B_k = np.asarray(q, F64), np.asarray(B_k, F64)
    h_q = q.shape[0]
    G = h_q // n_kv_heads
    return np.stack([B_k[:, (h // G) * head_dim:(h // G + 1) * head_dim] @ q[h] for h in range(h_q)])


def lorc_decode_absorbed(C_k, C_v, B_v, q_lat, n_kv_heads, head_dim, scale=None):
    """The same step written on the cached latents and an absorbed query: scores q_lat[h] . C_k[j] * scale
    (scale defaults to 1/sqrt(head_dim)), softmax over j, o_lat = P C_v, then the value up-projection."""
    C_k, C_v, B_v, q_lat = (np.asarray(a, F64) for a in (C_k, C_v, B_v, q_lat))
    h_q = q_lat.shape[0]
    G = h_q // n_kv_heads
    scale = 1.0 / np.sqrt(head_dim) if scale is None else scale
    out = np.empty((h_q, head_dim), F64)
    for h in range(h_q):
        o_lat = softmax_rows((C_k @ q_lat[h]) * scale) @ C_v
        out[h] = o_lat @ B_v[:, (h // G) * head_dim:(h // G + 1) * head_dim]
    return out


# =============================================================================== Section 5, Theorems 1 and 3
def truncation_error_constant(sigma, rank):
    """Theorem 1: ||x W - x W~||_2 <= sigma_{rank+1} ||x||_2.  sigma in decreasing order; 0 at full rank."""
    sigma = np.asarray(sigma, F64)
    return F64(sigma[rank]) if rank < sigma.shape[0] else F64(0.0)


def network_error_bound(sigmas, ranks, lipschitz=1.0):
    """Theorem 3: for an L-layer network x_i = phi(W_i x_{i-1}) with L_phi-Lipschitz phi, layer i truncated to rank
    k_i, the output error is bounded by  sum_i sigma^{(i)}_{k_i+1} L_phi^{L-i} prod_{j>i} ||W_j||_2,  with
    ||W_j||_2 = sigma^{(j)}_1.  As printed the bound carries no input norm: it is the bound for layer inputs of
    norm at most 1.  sigmas: one decreasing array per layer.  Returns (bound, terms[L])."""
    L = len(sigmas)
    terms = np.zeros(L, F64)
    for i in range(L):
        t = truncation_error_constant(sigmas[i], int(ranks[i])) * F64(lipschitz) ** (L - 1 - i)
        for j in range(i + 1, L):
            t *= F64(np.asarray(sigmas[j], F64)[0])
        terms[i] = t
    return F64(terms.sum()), terms
