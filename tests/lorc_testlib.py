"""Shared plumbing of the GPU parity tests: builds a seeded problem, drives the HIP library through its
Python binding, and evaluates the fp64 oracle on the same inputs.  No arithmetic of the method lives here
except the cache index formulas, which are retyped from the header's documentation on purpose (they are the
contract the bit-exact indexing tests check)."""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

import lorc_inputs as gen
from oracle import lorc_oracle as orc

PAGE = 64
TOL = 2e-2  # max |err| <= TOL * ||out||_inf  (bf16 storage, fp32 accumulation)


# --- documented page layout (include/lorc.h), retyped independently of the library --------------------
def k_index(r_k, slot, j):
    return ((slot // 32 * (r_k // 16) + j // 16) * 64 + slot % 32 + 32 * ((j % 16) // 8)) * 8 + j % 8


def v_index(r_k, slot, j):
    return 64 * r_k + (((j // 32) * 4 + slot // 16) * 64 + j % 32 + 32 * ((slot % 16) // 8)) * 8 + slot % 8


def page_gather_indices(r_k, r_v):
    """[64, r_k + r_v] element indices inside a page: row = slot, columns = K latents then V latents."""
    slot = np.arange(PAGE)[:, None]
    jk = np.arange(r_k)[None, :]
    jv = np.arange(r_v)[None, :]
    return np.concatenate([k_index(r_k, slot, jk), v_index(r_k, slot, jv)], axis=1)


@dataclass
class Problem:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rank_k: int
    rank_v: int
    rope_base: float
    ctx: list            # context length per sequence
    seed: int = 0
    W_k: np.ndarray = field(default=None, repr=False)
    W_v: np.ndarray = field(default=None, repr=False)
    X: list = field(default=None, repr=False)      # per sequence [N_s, D] float32 on the bf16 grid
    q: np.ndarray = field(default=None, repr=False)  # [b, h_q, d] float32 on the bf16 grid

    @property
    def n(self):
        return self.n_kv_heads * self.head_dim

    def build(self):
        self.W_k, _ = gen.power_law_weight(self.d_model, self.n, seed=1000 + 2 * self.seed)
        self.W_v, _ = gen.power_law_weight(self.d_model, self.n, seed=1001 + 2 * self.seed)
        self.X = [gen.hidden_states(N, self.d_model, seed=50000 + 97 * self.seed + s) for s, N in enumerate(self.ctx)]
        self.q = gen.queries(len(self.ctx), self.n_q_heads, self.head_dim, seed=90000 + self.seed)
        return self


def numpy_factors(W, rank):
    """Truncated SVD by LAPACK for shapes where the library's own host factorisation would take minutes:
    A = U_r Sigma_r, B = V_r^T (fp64), and the low-rank weight A B."""
    U, s, Vt = np.linalg.svd(W, full_matrices=False)
    A, B = U[:, :rank] * s[:rank], Vt[:rank]
    return A, B, A @ B


def oracle_decode(pb: Problem, seqs=None, q_pos=None, Wt=None):
    """fp64 oracle outputs [len(seqs), h_q, d] for the chosen sequences (default: all).

    Wt: optional (W~_k, W~_v), the rank-r weights when the caller has factored them already; an uncompressed
    layer (rank = n) uses the weights themselves."""
    seqs = range(len(pb.ctx)) if seqs is None else seqs
    if Wt is not None:
        Wt_k, Wt_v = Wt
    elif pb.rank_k == pb.n and pb.rank_v == pb.n:
        Wt_k, Wt_v = pb.W_k, pb.W_v
    else:
        Wt_k, _ = orc.low_rank_weight(pb.W_k, pb.rank_k)
        Wt_v, _ = orc.low_rank_weight(pb.W_v, pb.rank_v)
    outs = []
    for s in seqs:
        N = pb.ctx[s]
        if N == 0:
            outs.append(np.zeros((pb.n_q_heads, pb.head_dim)))
            continue
        X = pb.X[s].astype(np.float64)
        K = orc.split_heads(X @ Wt_k, pb.n_kv_heads, pb.head_dim)
        V = orc.split_heads(X @ Wt_v, pb.n_kv_heads, pb.head_dim)
        qp = N - 1 if q_pos is None else q_pos[s]
        outs.append(orc.attention_decode(pb.q[s].astype(np.float64), qp, K, V, np.arange(N), pb.rope_base))
    return np.stack(outs)


def oracle_prefill(pb: Problem, Q, seqs=None):
    """fp64 oracle of causal prefill: Q[s] is [N_s, h_q, d] (bf16 grid); returns a list of [N_s, h_q, d]."""
    seqs = range(len(pb.ctx)) if seqs is None else seqs
    if pb.rank_k == pb.n and pb.rank_v == pb.n:   # uncompressed layer: the weights themselves
        Wt_k, Wt_v = pb.W_k, pb.W_v
    else:
        Wt_k, _ = orc.low_rank_weight(pb.W_k, pb.rank_k)
        Wt_v, _ = orc.low_rank_weight(pb.W_v, pb.rank_v)
    outs = []
    for s in seqs:
        X = pb.X[s].astype(np.float64)
        K = orc.split_heads(X @ Wt_k, pb.n_kv_heads, pb.head_dim)
        V = orc.split_heads(X @ Wt_v, pb.n_kv_heads, pb.head_dim)
        outs.append(orc.attention_prefill(Q[s].astype(np.float64), K, V, pb.rope_base))
    return outs


class GpuLayer:
    """One layer's device state: packed factors, page pool, block table."""

    def __init__(self, pb: Problem, extra_pages=3, sentinel=0xFF, page_seed=7, max_pages=None, plain=False, factors=None):
        """plain: an uncompressed layer (rank = n, A = W, no read-side factors).  factors: (A_k, B_k, A_v, B_v)
        worked out by the caller instead of the library's host factorisation."""
        import torch
        import paper_2410_03111_amd as L
        self.L, self.torch, self.pb, self.plain = L, torch, pb, plain
        dev = torch.device("cuda:0")
        self.dev = dev
        self.desc = L.layer_desc(pb.d_model, pb.n_q_heads, pb.n_kv_heads, pb.head_dim, pb.rank_k, pb.rank_v, pb.rope_base)
        f = lambda a: torch.from_numpy(a.astype(np.float32)).to(dev).to(torch.bfloat16).contiguous()
        if plain:
            assert pb.rank_k == pb.n and pb.rank_v == pb.n
            self.A_k, self.A_v, self.B_k, self.B_v = pb.W_k, pb.W_v, None, None
            self.dA_k, self.dA_v, self.dB_k, self.dB_v = f(self.A_k), f(self.A_v), None, None
        else:
            if factors is not None:
                self.A_k, self.B_k, self.A_v, self.B_v = factors
            else:  # offline factorisation by the library itself (host), rounded once to bf16 on upload
                self.A_k, self.B_k, self.sigma_k, self.eps_k = L.factorize(pb.W_k, pb.rank_k)
                self.A_v, self.B_v, self.sigma_v, self.eps_v = L.factorize(pb.W_v, pb.rank_v)
            self.dA_k, self.dA_v, self.dB_k, self.dB_v = f(self.A_k), f(self.A_v), f(self.B_k), f(self.B_v)
        self.packed = L.pack_factors(self.desc, self.dA_k, self.dA_v, self.dB_k, self.dB_v)
        b = len(pb.ctx)
        self.max_pages = max_pages or max(1, max((N + PAGE - 1) // PAGE for N in pb.ctx))
        self.n_pages = b * self.max_pages + extra_pages
        self.block_table_np = gen.block_table(b, self.max_pages, self.n_pages, seed=page_seed)
        self.block_table = torch.from_numpy(self.block_table_np).to(dev)
        self.page_bytes = L.page_bytes(self.desc)
        self.sentinel = sentinel
        self.cache = torch.full((self.n_pages * self.page_bytes,), sentinel, dtype=torch.uint8, device=dev)

    def append_all(self):
        """Append every token of every sequence (token j of sequence s at position j) in one call."""
        torch, pb = self.torch, self.pb
        xs = [x for x in pb.X if x.shape[0] > 0]
        if not xs:
            return
        x = torch.from_numpy(np.concatenate(xs, axis=0)).to(self.dev).to(torch.bfloat16).contiguous()
        seq = np.concatenate([np.full(N, s, np.int32) for s, N in enumerate(pb.ctx)])
        pos = np.concatenate([np.arange(N, dtype=np.int32) for N in pb.ctx])
        self.L.append_latent(self.desc, x, self.packed, torch.from_numpy(seq).to(self.dev),
                             torch.from_numpy(pos).to(self.dev), self.block_table, self.cache)

    def decode(self, q_pos=None, ctx=None, max_ctx=None):
        torch, pb = self.torch, self.pb
        ctx = pb.ctx if ctx is None else ctx
        q = torch.from_numpy(pb.q).to(self.dev).to(torch.bfloat16).contiguous()
        qp = np.array([max(N - 1, 0) for N in ctx] if q_pos is None else q_pos, np.int32)
        fn = self.L.decode_attention_plain if self.plain else self.L.decode_attention
        out = fn(self.desc, q, torch.from_numpy(qp).to(self.dev),
                                      torch.from_numpy(np.array(ctx, np.int32)).to(self.dev),
                                      max(ctx) if max_ctx is None else max_ctx, self.packed, self.cache, self.block_table)
        torch.cuda.synchronize()
        return out.float().cpu().numpy().astype(np.float64)

    def prefill(self, Q):
        """Causal prefill over the cached prompts; Q[s] is [N_s, h_q, d] float32 on the bf16 grid."""
        torch, pb = self.torch, self.pb
        q = torch.from_numpy(np.concatenate(Q, axis=0)).to(self.dev).to(torch.bfloat16).contiguous()
        cu = np.concatenate([[0], np.cumsum(pb.ctx)]).astype(np.int32)
        out = self.L.prefill_attention(self.desc, q, torch.from_numpy(cu).to(self.dev), max(pb.ctx), self.packed,
                                       self.cache, self.block_table, plain=self.plain)
        torch.cuda.synchronize()
        o = out.float().cpu().numpy().astype(np.float64)
        return [o[cu[s]:cu[s + 1]] for s in range(len(pb.ctx))]

    def read_latents(self, s, N):
        """Latents of the first N positions of sequence s as stored: uint16 [N, r_k + r_v]."""
        pb = self.pb
        pool = self.cache.cpu().numpy().view(np.uint16).reshape(self.n_pages, -1)
        idx = page_gather_indices(pb.rank_k, pb.rank_v)
        rows = []
        for p in range((N + PAGE - 1) // PAGE):
            page = pool[self.block_table_np[s, p]]
            rows.append(page[idx])
        return np.concatenate(rows, axis=0)[:N]


def rel_err(got, ref):
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
