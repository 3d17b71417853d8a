"""lorc_append_latent on the GPU: values against the oracle's latents, and bit-exact page indexing."""
import numpy as np
import pytest

import lorc_inputs as gen
from oracle import lorc_oracle as orc
from lorc_testlib import GpuLayer, Problem, PAGE, page_gather_indices

pytestmark = pytest.mark.gpu


def _append_and_compare_pool(geom, ctx, density=1.0, seed=5):
    """Appends integer-valued tokens (a fraction `density` of them non-zero) and compares the whole pool, byte for
    byte, with the latents placed by the documented index formulas.  Returns (L, desc, idx) for further checks."""
    import torch
    import paper_2410_03111_amd as L
    D, h_kv, d, r_k, r_v = geom
    desc = L.layer_desc(D, 2 * h_kv, h_kv, d, r_k, r_v, 10000.0)
    rng = np.random.default_rng(seed)
    A_k = rng.integers(-1, 2, (D, r_k)).astype(np.float32)
    A_v = rng.integers(-1, 2, (D, r_v)).astype(np.float32)
    B = np.zeros((r_k, h_kv * d), np.float32)
    T = sum(ctx)
    X = (rng.integers(-1, 2, (T, D)) * (rng.random((T, D)) < density)).astype(np.float32)
    dev = torch.device("cuda:0")
    bf = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16).contiguous()
    packed = L.pack_factors(desc, bf(A_k), bf(A_v), bf(B), bf(np.zeros((r_v, h_kv * d), np.float32)))
    max_pages = (max(ctx) + PAGE - 1) // PAGE
    n_pages = len(ctx) * max_pages + 5
    bt = gen.block_table(len(ctx), max_pages, n_pages, seed=3)
    page_elems = L.page_bytes(desc) // 2
    sentinel = 0xABCD
    pool0 = np.full((n_pages, page_elems), sentinel, np.uint16)
    cache = torch.from_numpy(pool0.view(np.uint8).reshape(-1).copy()).to(dev)
    # tokens in shuffled order: the slot arrays, not the order in x, decide where a latent goes
    seq = np.concatenate([np.full(N, s, np.int32) for s, N in enumerate(ctx)])
    pos = np.concatenate([np.arange(N, dtype=np.int32) for N in ctx])
    perm = rng.permutation(T)
    L.append_latent(desc, bf(X[perm]), packed, torch.from_numpy(seq[perm]).to(dev), torch.from_numpy(pos[perm]).to(dev),
                    torch.from_numpy(bt).to(dev), cache)
    torch.cuda.synchronize()
    got = cache.cpu().numpy().view(np.uint16).reshape(n_pages, page_elems)
    expect = pool0.copy()
    lat = np.concatenate([X @ A_k, X @ A_v], axis=1)          # exact small integers
    assert np.max(np.abs(lat)) <= 256
    bits = gen.bf16_bits(lat.astype(np.float32))
    idx = page_gather_indices(r_k, r_v)
    pages = bt[seq, pos // PAGE]
    for t in range(T):
        expect[pages[t], idx[pos[t] % PAGE]] = bits[t]
    assert np.array_equal(got, expect)
    return L, desc, idx


@pytest.mark.parametrize("geom,ctx", [((128, 2, 64, 64, 32), [130, 1, 64, 77]),
                                      ((256, 4, 64, 256, 224), [4100, 1, 64, 77]),
                                      ((128, 2, 64, 64, 32), [8100, 1, 64, 77])],
                         ids=["272_tokens", "4242_tokens_wide", "8242_tokens"])
def test_indexing_is_bit_exact_with_integer_data(geom, ctx):
    """Integer-valued inputs make every latent exactly representable, so the pool can be compared byte for
    byte: each (sequence, position) must sit at its documented place and nothing else may change.  The
    cases go through the 64-row-tile, the 128-row-tile and the 256-row-tile kernel."""
    L, desc, idx = _append_and_compare_pool(geom, ctx)
    r_k, r_v = geom[3], geom[4]
    # the library's own index helpers agree with the documented formulas
    for slot, j in [(0, 0), (33, 17), (63, r_k - 1), (17, 40)]:
        assert L.cache_index_k(desc, slot, j) == idx[slot, j]
    for slot, j in [(0, 0), (33, 17), (63, r_v - 1)]:
        assert L.cache_index_v(desc, slot, j) == idx[slot, r_k + j]


@pytest.mark.parametrize("D", [64, 192, 640, 832])
@pytest.mark.parametrize("case", ["64_row_tile", "128_row_tile", "256_row_tile"])
def test_model_dimension_tails_are_bit_exact(D, case):
    """Model dimensions of 1, 3, 10 and 13 k-tiles: fewer k-tiles than a kernel keeps in flight, and counts that
    leave a remainder after its unrolled groups, for each of the three tiled kernels."""
    geom, ctx = {"64_row_tile": ((D, 2, 64, 64, 32), [100, 37]),
                 "128_row_tile": ((D, 4, 64, 256, 224), [4100, 1, 90]),
                 "256_row_tile": ((D, 2, 64, 64, 32), [8100, 1, 90])}[case]
    _append_and_compare_pool(geom, ctx, density=0.2, seed=D)


def test_out_of_range_slots_are_skipped():
    import torch
    import paper_2410_03111_amd as L
    D, r = 128, 32
    desc = L.layer_desc(D, 2, 2, 64, r, r, 10000.0)
    dev = torch.device("cuda:0")
    z = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device=dev)
    packed = L.pack_factors(desc, torch.ones(D, r, dtype=torch.bfloat16, device=dev), z(D, r), z(r, 128), z(r, 128))
    cache = torch.full((4 * L.page_bytes(desc),), 0x5A, dtype=torch.uint8, device=dev)
    bt = torch.tensor([[1, -1], [99, 2]], dtype=torch.int32, device=dev)   # -1 and 99 are not pages of the pool
    x = torch.ones(6, D, dtype=torch.bfloat16, device=dev)
    seq = torch.tensor([0, 0, 1, 1, 2, -1], dtype=torch.int32, device=dev)
    pos = torch.tensor([0, 64, 0, 64, 0, 0], dtype=torch.int32, device=dev)
    L.append_latent(desc, x, packed, seq, pos, bt, cache)
    torch.cuda.synchronize()
    pool = cache.cpu().numpy().reshape(4, -1)
    assert np.all(pool[0] == 0x5A) and np.all(pool[3] == 0x5A)
    assert np.sum(pool[1] != 0x5A) > 0 and np.sum(pool[2] != 0x5A) > 0     # (0,0) -> page 1, (1,64) -> page 2
    changed = (pool != 0x5A).sum()
    assert changed <= 2 * (2 * r) * 2                                       # two tokens' latents at most


@pytest.mark.parametrize("shape", [
    dict(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rank_k=32, rank_v=32, rope_base=10000.0, ctx=[128]),
    dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=96, rope_base=10000.0, ctx=[1, 77, 300]),
    dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=512, rank_v=512, rope_base=500000.0, ctx=[200, 513]),
    # above a thousand tokens in one call, with ragged token and latent-row tails (64- and 128-row-tile GEMM)
    dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=96, rank_v=64, rope_base=10000.0, ctx=[700, 1, 530]),
    dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=768, rank_v=384, rope_base=500000.0, ctx=[1700, 333]),
    # 8192 tokens and more in one call: the 256-row-tile GEMM of long prompts, same ragged tails
    dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=96, rank_v=64, rope_base=10000.0, ctx=[7900, 1, 530]),
])
def test_latents_match_oracle(shape):
    pb = Problem(seed=3, **shape).build()
    layer = GpuLayer(pb)
    layer.append_all()
    layer.torch.cuda.synchronize()
    A_k, _, s_k = orc.latent_factors(pb.W_k, pb.rank_k)
    A_v, _, s_v = orc.latent_factors(pb.W_v, pb.rank_v)
    # singular vectors are fixed up to sign: compare latents through quantities that do not depend on it
    for s, N in enumerate(pb.ctx):
        got = gen.bf16_to_f32(layer.read_latents(s, N)).astype(np.float64)
        X = pb.X[s].astype(np.float64)
        ref = np.concatenate([X @ A_k, X @ A_v], axis=1)
        scale = np.max(np.abs(ref))
        assert np.max(np.abs(np.abs(got) - np.abs(ref))) <= 1.5e-2 * scale
        # the K latent rebuilds the rank-r key: C_k B_k == X W~_k
        Wt_k, _ = orc.low_rank_weight(pb.W_k, pb.rank_k)
        K_ref = X @ Wt_k
        K_got = got[:, :pb.rank_k] @ layer.dB_k.float().cpu().numpy().astype(np.float64)
        assert np.max(np.abs(K_got - K_ref)) <= 2e-2 * np.max(np.abs(K_ref))
    # untouched pages keep the sentinel
    used = set(layer.block_table_np[s, p] for s, N in enumerate(pb.ctx) for p in range((N + PAGE - 1) // PAGE))
    pool = layer.cache.cpu().numpy().reshape(layer.n_pages, -1)
    for p in range(layer.n_pages):
        if p not in used:
            assert np.all(pool[p] == layer.sentinel)


@pytest.mark.parametrize("T", [1, 5, 16, 17, 32, 33, 64, 65, 100, 129, 200])
def test_small_batches_are_bit_exact(T):
    """The dot-product kernel of small batches (T <= 64, one pass per 16 tokens) and the 64-row-tile kernel just
    above it, with integer data: every latent must land bit-exact at its documented place, one call per batch size."""
    import torch
    import paper_2410_03111_amd as L
    D, h_kv, d, r_k, r_v = 256, 2, 64, 96, 32
    desc = L.layer_desc(D, 4, h_kv, d, r_k, r_v, 10000.0)
    rng = np.random.default_rng(100 + T)
    A_k = rng.integers(-1, 2, (D, r_k)).astype(np.float32)
    A_v = rng.integers(-1, 2, (D, r_v)).astype(np.float32)
    X = rng.integers(-1, 2, (T, D)).astype(np.float32)
    dev = torch.device("cuda:0")
    bf = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16).contiguous()
    z = np.zeros((r_k, h_kv * d), np.float32)
    packed = L.pack_factors(desc, bf(A_k), bf(A_v), bf(z), bf(np.zeros((r_v, h_kv * d), np.float32)))
    n_seqs, max_pages, n_pages = 4, 2, 11
    bt = gen.block_table(n_seqs, max_pages, n_pages, seed=T)
    page_elems = L.page_bytes(desc) // 2
    pool0 = np.full((n_pages, page_elems), 0xABCD, np.uint16)
    cache = torch.from_numpy(pool0.view(np.uint8).reshape(-1).copy()).to(dev)
    # distinct (sequence, position) pairs in random order
    pairs = rng.permutation(n_seqs * max_pages * PAGE)[:T]
    seq, pos = (pairs // (max_pages * PAGE)).astype(np.int32), (pairs % (max_pages * PAGE)).astype(np.int32)
    L.append_latent(desc, bf(X), packed, torch.from_numpy(seq).to(dev), torch.from_numpy(pos).to(dev),
                    torch.from_numpy(bt).to(dev), cache)
    torch.cuda.synchronize()
    got = cache.cpu().numpy().view(np.uint16).reshape(n_pages, page_elems)
    lat = np.concatenate([X @ A_k, X @ A_v], axis=1)
    assert np.max(np.abs(lat)) <= 256
    bits = gen.bf16_bits(lat.astype(np.float32))
    idx = page_gather_indices(r_k, r_v)
    expect = pool0.copy()
    for t in range(T):
        expect[bt[seq[t], pos[t] // PAGE], idx[pos[t] % PAGE]] = bits[t]
    assert np.array_equal(got, expect)


def test_decode_time_append_matches_oracle_on_the_8b_shape():
    """16 new tokens against the 4096 x 1024 down-projection (the call bench.py times): values against the fp64
    latents, through sign-free quantities."""
    pb = Problem(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=512, rank_v=512, rope_base=500000.0,
                 ctx=[1] * 16, seed=21).build()
    layer = GpuLayer(pb)
    layer.append_all()  # 16 tokens in one call, one per sequence
    layer.torch.cuda.synchronize()
    A_k, _, _ = orc.latent_factors(pb.W_k, pb.rank_k)
    A_v, _, _ = orc.latent_factors(pb.W_v, pb.rank_v)
    got = np.concatenate([gen.bf16_to_f32(layer.read_latents(s, 1)).astype(np.float64) for s in range(16)])
    X = np.concatenate(pb.X).astype(np.float64)
    ref = np.concatenate([X @ A_k, X @ A_v], axis=1)
    assert np.max(np.abs(np.abs(got) - np.abs(ref))) <= 1.5e-2 * np.max(np.abs(ref))
