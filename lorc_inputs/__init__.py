"""Seeded synthetic inputs for the LoRC hot path (weights, hidden states, queries, page tables).

This module only *generates data*: it holds none of the method's arithmetic (no SVD truncation, no
attention, no RoPE, no cache layout).  Both the CPU oracle's tests and the HIP path's tests/bench draw
their inputs from here so that the two sides see identical numbers.

Shapes follow the paper's model table (Table 3: LLaMA-3-8B 4096x1024, 32/8 heads, d=128; LLaMA-3-70B
8192x1024, 64/8 heads) and the benchmark configurations; trained weights are replaced by matrices with a
known power-law singular spectrum so that truncation errors have closed forms.
"""
from __future__ import annotations

import numpy as np

ALPHA = 0.7  # sigma_i proportional to i**-ALPHA


# ----------------------------------------------------------------------------- bf16 storage format
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even) and return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Values of x rounded to the bfloat16 grid, returned as float32 (exactly representable in bf16)."""
    return bf16_to_f32(bf16_bits(x)).reshape(np.shape(x))


# ----------------------------------------------------------------------------- weights
def power_law_spectrum(n: int, alpha: float = ALPHA) -> np.ndarray:
    """sigma_i = c * i**-alpha (i = 1..n), c chosen so that sum(sigma**2) == n."""
    i = np.arange(1, n + 1, dtype=np.float64)
    s = i ** (-alpha)
    return s * np.sqrt(n / np.sum(s * s))


def power_law_weight(rows: int, cols: int, seed: int, alpha: float = ALPHA):
    """W = P diag(sigma) Q^T (rows x cols, fp64) with Haar-like orthonormal P, Q and a power-law spectrum.

    ||W||_F^2 == cols, i.e. entries have variance 1/rows like N(0, 1/rows) initialisation, so x W has
    roughly unit-variance coordinates for x ~ N(0, I).  Returns (W, sigma).
    """
    k = min(rows, cols)
    rng = np.random.Generator(np.random.PCG64(seed))
    P, _ = np.linalg.qr(rng.standard_normal((rows, k)))
    Q, _ = np.linalg.qr(rng.standard_normal((cols, k)))
    sigma = power_law_spectrum(k, alpha)
    W = (P * sigma) @ Q.T
    return W, sigma


# ----------------------------------------------------------------------------- activations
def hidden_states(tokens: int, d_model: int, seed: int) -> np.ndarray:
    """x ~ N(0,1) i.i.d., rounded to the bf16 grid; float32 [tokens, d_model]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return bf16_round(rng.standard_normal((tokens, d_model), dtype=np.float32))


def queries(count: int, n_q_heads: int, head_dim: int, seed: int) -> np.ndarray:
    """q ~ N(0,1) per element, bf16 grid; float32 [count, n_q_heads, head_dim] (un-rotated)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return bf16_round(rng.standard_normal((count, n_q_heads, head_dim), dtype=np.float32))


def latent_samples(tokens: int, sigma_kept: np.ndarray, seed: int) -> np.ndarray:
    """Bench-only cache fill: c_j ~ N(0, sigma_j^2), the exact law of x (U_r Sigma_r) for x ~ N(0, I).

    Used where the hidden states themselves (tens of GB per layer) would not fit; float32 [tokens, r]
    on the bf16 grid.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    z = rng.standard_normal((tokens, sigma_kept.shape[0]), dtype=np.float32)
    return bf16_round(z * sigma_kept.astype(np.float32)[None, :])


# ----------------------------------------------------------------------------- paging
def block_table(n_seqs: int, pages_per_seq: int, pool_pages: int, seed: int) -> np.ndarray:
    """int32 [n_seqs, pages_per_seq]: a seeded random choice of distinct pool pages (non-contiguous)."""
    assert n_seqs * pages_per_seq <= pool_pages
    rng = np.random.Generator(np.random.PCG64(seed))
    perm = rng.permutation(pool_pages)[: n_seqs * pages_per_seq]
    return perm.astype(np.int32).reshape(n_seqs, pages_per_seq)


def rank_ramp(n_layers: int, r_first: int, r_last: int, align: int = 32) -> list[int]:
    """Per-layer ranks falling linearly from r_first (layer 0) to r_last (last layer), each rounded to the
    nearest multiple of `align` (ties away from zero)."""
    out = []
    for l in range(n_layers):
        t = l / (n_layers - 1) if n_layers > 1 else 0.0
        v = r_first + (r_last - r_first) * t
        out.append(int(align * np.floor(v / align + 0.5)))
    return out


# ----------------------------------------------------------------------------- named workloads
# Index = position in the benchmark's configuration list.
CONFIGS = {
    0: dict(name="tiny", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rank=32, batch=1,
            context=128, rope_base=10000.0, layers=1, seed=0),
    1: dict(name="llama3-8b-layer-decode", d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=512,
            batch=16, context=4096, rope_base=500000.0, layers=1, seed=1),
    2: dict(name="llama3-8b-stack-decode", d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
            rank_first=768, rank_last=384, batch=32, context=8192, rope_base=500000.0, layers=32, seed=2),
    3: dict(name="llama3-8b-prefill", d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank=512,
            batch=4, context=8192, rope_base=500000.0, layers=1, seed=3),
    4: dict(name="llama3-70b-share-decode", d_model=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, rank=512,
            batch=64, context=32768, rope_base=500000.0, layers=8, seed=4),
}
