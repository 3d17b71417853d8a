"""lorc_decode_attention on the GPU against the fp64 oracle (element by element)."""
import numpy as np
import pytest

from lorc_testlib import GpuLayer, Problem, TOL, oracle_decode, rel_err

pytestmark = pytest.mark.gpu

SHAPES = {
    "config0_tiny": dict(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rank_k=32, rank_v=32,
                         rope_base=10000.0, ctx=[128], seed=0),
    "ragged_mid": dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=96,
                       rope_base=10000.0, ctx=[1, 77, 300, 64, 129], seed=1),
    "d64_wide": dict(d_model=256, n_q_heads=16, n_kv_heads=4, head_dim=64, rank_k=160, rank_v=64,
                     rope_base=10000.0, ctx=[257, 31], seed=2),
    "llama8b_short": dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=512, rank_v=512,
                          rope_base=500000.0, ctx=[200, 513, 1100], seed=3),
    "rank_above_512": dict(d_model=1024, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=768, rank_v=640,
                           rope_base=500000.0, ctx=[333, 65], seed=4),
    "g8_two_query_blocks": dict(d_model=1024, n_q_heads=64, n_kv_heads=8, head_dim=128, rank_k=128, rank_v=128,
                                rope_base=500000.0, ctx=[190, 300], seed=5),
    # value rank far above the key rank: the split's output rows do not fit the K tile's LDS and are stored directly
    "narrow_k_wide_v": dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=32, rank_v=256,
                            rope_base=10000.0, ctx=[150, 64, 3], seed=6),
}


@pytest.mark.parametrize("name", list(SHAPES))
def test_decode_matches_oracle(name):
    pb = Problem(**SHAPES[name]).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = layer.decode()
    ref = oracle_decode(pb)
    assert got.shape == ref.shape
    assert np.all(np.isfinite(got))
    err = rel_err(got, ref)
    print(f"{name}: rel err {err:.3e}")
    assert err <= TOL


@pytest.mark.parametrize("name", ["llama8b_short", "rank_above_512"])  # group merge kernel / generic merge kernel
def test_latent_space_output_times_factor_equals_decode(name):
    """lorc_decode_attention_latent: its output times the library's own value up-projection factor is the
    oracle's decode output (the factor gauge is the library's, so the product is what can be compared)."""
    import torch
    pb = Problem(**SHAPES[name]).build()
    layer = GpuLayer(pb)
    layer.append_all()
    L = layer.L
    q = torch.from_numpy(pb.q).to(layer.dev).to(torch.bfloat16).contiguous()
    ctx = torch.tensor(pb.ctx, dtype=torch.int32, device=layer.dev)
    o_lat = L.decode_attention_latent(layer.desc, q, ctx - 1, ctx, max(pb.ctx), layer.packed, layer.cache, layer.block_table)
    torch.cuda.synchronize()
    assert tuple(o_lat.shape) == (len(pb.ctx), pb.n_q_heads, pb.rank_v)
    o_lat = o_lat.float().cpu().numpy().astype(np.float64)
    B_v = layer.dB_v.float().cpu().numpy().astype(np.float64)  # bf16 factor as uploaded
    G, d = pb.n_q_heads // pb.n_kv_heads, pb.head_dim
    got = np.stack([np.stack([o_lat[s, h] @ B_v[:, (h // G) * d:(h // G + 1) * d] for h in range(pb.n_q_heads)])
                    for s in range(len(pb.ctx))])
    ref = oracle_decode(pb)
    err = rel_err(got, ref)
    print(f"latent output x B_v: rel err {err:.3e}")
    assert err <= TOL
    # and it is the same attention as the full entry point
    full = layer.decode()
    assert rel_err(got, full) <= TOL


@pytest.mark.parametrize("ctx", [[2560], [9000, 70]], ids=["40_splits", "141_splits"])
def test_many_context_splits(ctx):
    """One long sequence spreads over many context splits: 40 exercises the second batch of partials in the
    group merge kernel, 141 is past its limit and takes the generic merge kernel."""
    pb = Problem(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=64, rope_base=10000.0,
                 ctx=ctx, seed=31).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = layer.decode()
    ref = oracle_decode(pb)
    err = rel_err(got, ref)
    print(f"ctx {ctx}: rel err {err:.3e}")
    assert err <= TOL
