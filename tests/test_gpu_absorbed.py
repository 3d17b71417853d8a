"""Decode without positional rotation, key factor folded into the query (Section 4.1, Eq. 7), through the C ABI:
lorc_decode_attention_absorbed against the fp64 oracle of the materialised rank-r model."""
import numpy as np
import pytest

from lorc_testlib import GpuLayer, Problem, TOL, rel_err
from oracle import lorc_oracle as orc

pytestmark = pytest.mark.gpu

SHAPES = {
    "config0_tiny": dict(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rank_k=32, rank_v=32, ctx=[128], seed=0),
    "ragged_mid": dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=96,
                       ctx=[1, 77, 300, 64, 129], seed=1),
    "d64_wide": dict(d_model=256, n_q_heads=16, n_kv_heads=4, head_dim=64, rank_k=160, rank_v=64, ctx=[257, 31], seed=2),
    "llama8b_short": dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=512, rank_v=512,
                          ctx=[200, 513, 1100], seed=3),
    "narrow_k_wide_v": dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=32, rank_v=256,
                            ctx=[150, 64, 3], seed=6),
    "one_kv_head_g32": dict(d_model=512, n_q_heads=32, n_kv_heads=1, head_dim=128, rank_k=128, rank_v=96, ctx=[100, 257], seed=7),
}


def run_absorbed(layer, ctx=None, max_ctx=None):
    """q_lat[s][h] = B_k^{g(h)} q[s][h] with the factors the layer was packed with, rounded to bf16 once."""
    torch, pb = layer.torch, layer.pb
    ctx = pb.ctx if ctx is None else ctx
    q_lat = np.stack([orc.absorb_query(pb.q[s].astype(np.float64), layer.B_k, pb.n_kv_heads, pb.head_dim)
                      for s in range(len(ctx))]).astype(np.float32)
    out = layer.L.decode_attention_absorbed(
        layer.desc, torch.from_numpy(q_lat).to(layer.dev).to(torch.bfloat16).contiguous(),
        torch.from_numpy(np.array(ctx, np.int32)).to(layer.dev), max_ctx or max(max(ctx), 1), layer.packed, layer.cache,
        layer.block_table)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


def oracle_plain(pb, seqs=None):
    seqs = range(len(pb.ctx)) if seqs is None else seqs
    outs = []
    for s in seqs:
        if pb.ctx[s] == 0:
            outs.append(np.zeros((pb.n_q_heads, pb.head_dim)))
            continue
        outs.append(orc.lorc_decode_plain(pb.X[s].astype(np.float64), pb.q[s].astype(np.float64), pb.W_k, pb.W_v,
                                          pb.rank_k, pb.rank_v, pb.n_kv_heads, pb.head_dim))
    return np.stack(outs)


@pytest.mark.parametrize("name", list(SHAPES))
def test_absorbed_decode_matches_oracle(name):
    pb = Problem(rope_base=10000.0, **SHAPES[name]).build()
    layer = GpuLayer(pb)   # pool pre-filled with 0xFF bytes: every slot that is not written is a bf16 NaN
    layer.append_all()
    got = run_absorbed(layer)
    ref = oracle_plain(pb)
    assert np.all(np.isfinite(got))
    err = rel_err(got, ref)
    print(f"{name}: rel err {err:.3e}")
    assert err <= TOL


def test_absorbed_decode_empty_and_shortened_contexts():
    pb = Problem(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=64, rope_base=10000.0,
                 ctx=[0, 200, 0, 190], seed=14).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = run_absorbed(layer)
    ref = oracle_plain(pb)
    assert np.all(got[0] == 0.0) and np.all(got[2] == 0.0)
    assert rel_err(got[[1, 3]], ref[[1, 3]]) <= TOL
    short = [0, 77, 0, 128]   # attends to a prefix of what is cached
    got = run_absorbed(layer, ctx=short, max_ctx=200)
    pb_short = Problem(**{**pb.__dict__, "ctx": short, "X": [x[:n] for x, n in zip(pb.X, short)]})
    assert rel_err(got[[1, 3]], oracle_plain(pb_short)[[1, 3]]) <= TOL


def test_absorbed_decode_many_splits_and_tiles():
    """Long contexts over few sequences: several tiles per workgroup and tens of splits per sequence."""
    pb = Problem(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=96, rank_v=64, rope_base=10000.0,
                 ctx=[9000, 2500], seed=15).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = run_absorbed(layer)
    assert rel_err(got, oracle_plain(pb)) <= TOL


# beyond the single streaming kernel (h_q <= 32, ranks <= 512): scores on the latents, values in column chunks, merge
LARGE = {
    "q64_g8_r512": dict(d_model=1024, n_q_heads=64, n_kv_heads=8, head_dim=128, rank_k=512, rank_v=512, ctx=[300, 70, 0], seed=21),
    "rk1024_rv768": dict(d_model=1024, n_q_heads=16, n_kv_heads=8, head_dim=128, rank_k=1024, rank_v=768, ctx=[200, 1], seed=22),
    "d64_mha_r1280_1056": dict(d_model=2048, n_q_heads=32, n_kv_heads=32, head_dim=64, rank_k=1280, rank_v=1056, ctx=[130], seed=23),
    "q40_rv544_long": dict(d_model=640, n_q_heads=40, n_kv_heads=5, head_dim=128, rank_k=96, rank_v=544, ctx=[2600, 64], seed=24),
}


@pytest.mark.parametrize("name", list(LARGE))
def test_absorbed_decode_large_shapes_match_oracle(name):
    pb = Problem(rope_base=10000.0, **LARGE[name]).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = run_absorbed(layer)
    ref = oracle_plain(pb)
    assert np.all(np.isfinite(got))
    for s, N in enumerate(pb.ctx):
        if N == 0:
            assert np.all(got[s] == 0.0)
    live = [s for s, N in enumerate(pb.ctx) if N > 0]
    err = rel_err(got[live], ref[live])
    print(f"{name}: rel err {err:.3e}")
    assert err <= TOL


def test_absorbed_decode_refuses_shapes_it_is_not_built_for():
    import paper_2410_03111_amd as L
    # value rank above what the merge kernel holds; the streaming kernel's own limits are covered by the three-launch path
    assert L.decode_absorbed_workspace_bytes(L.layer_desc(2560, 20, 20, 128, 512, 2304, 10000.0), 1, 64) == 0
    assert L.decode_absorbed_workspace_bytes(L.layer_desc(2560, 20, 20, 128, 2304, 2048, 10000.0), 1, 64) > 0
    assert L.decode_absorbed_workspace_bytes(L.layer_desc(1024, 64, 8, 128, 128, 128, 10000.0), 1, 64) > 0
