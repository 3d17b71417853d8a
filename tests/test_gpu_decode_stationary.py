"""Parity of the decode path on the shapes that take the split kernel with the key factor held in registers
(head_dim 128, an even number of KV heads, G <= 8, 384 < rank_k <= 512, rank_v <= 512): query-group sizes 1 .. 8, ranks
that are not a multiple of 128 (padded k-steps), ragged and empty contexts, many tiles per split, many splits, pages
that are not cached, shifted and long positions.  Model widths are small so that the fp64 oracle stays cheap."""
import numpy as np
import pytest

from lorc_testlib import GpuLayer, Problem, TOL, oracle_decode, rel_err

pytestmark = pytest.mark.gpu

SHAPES = {
    "g4_rank512": dict(n_q_heads=16, n_kv_heads=4, rank_k=512, rank_v=512, ctx=[700, 64, 1, 129]),
    "g8_rank448_416": dict(n_q_heads=32, n_kv_heads=4, rank_k=448, rank_v=416, ctx=[300, 1000]),
    "g1_rank416_v32": dict(n_q_heads=4, n_kv_heads=4, rank_k=416, rank_v=32, ctx=[200, 65]),
    "g2_rank480_empty_and_long": dict(n_q_heads=8, n_kv_heads=4, rank_k=480, rank_v=512, ctx=[0, 2500, 63]),
    "six_kv_heads_rank416": dict(n_q_heads=12, n_kv_heads=6, rank_k=416, rank_v=96, ctx=[1300]),
}


@pytest.mark.parametrize("name", list(SHAPES))
def test_stationary_shapes_match_oracle(name):
    shape = dict(SHAPES[name])
    n = shape["n_kv_heads"] * 128
    pb = Problem(d_model=max(512, n), head_dim=128, rope_base=500000.0, seed=61 + len(name), **shape).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = layer.decode()
    ref = oracle_decode(pb)
    assert np.all(np.isfinite(got))
    for s, N in enumerate(pb.ctx):
        if N == 0:
            assert np.all(got[s] == 0.0)
    live = [s for s, N in enumerate(pb.ctx) if N > 0]
    err = rel_err(got[live], ref[live])
    print(f"{name}: rel err {err:.3e}")
    assert err <= TOL


def test_stationary_unmapped_page_and_shifted_query_positions():
    import torch
    pb = Problem(d_model=512, n_q_heads=16, n_kv_heads=4, head_dim=128, rank_k=512, rank_v=448, rope_base=500000.0,
                 ctx=[330, 200], seed=71).build()
    layer = GpuLayer(pb)
    bt = layer.block_table_np.copy()
    bt[0, 1] = -1                      # positions 64 .. 127 of sequence 0
    bt[0, 4] = layer.n_pages + 9       # positions 256 .. 319
    bt[1, 0] = -7                      # the first tile of sequence 1
    layer.block_table_np = bt
    layer.block_table = torch.from_numpy(bt).to(layer.dev)
    layer.append_all()
    q_pos = [1000, 199]
    got = layer.decode(q_pos=q_pos)
    X = [x.copy() for x in pb.X]
    X[0][64:128] = 0.0
    X[0][256:320] = 0.0
    X[1][0:64] = 0.0
    ref = oracle_decode(Problem(**{**pb.__dict__, "X": X}), q_pos=q_pos)
    assert np.all(np.isfinite(got))
    err = rel_err(got, ref)
    print(f"unmapped pages, shifted query: rel err {err:.3e}")
    assert err <= TOL


def test_stationary_wide_batch_walks_many_tiles_per_workgroup():
    """A batch wide enough that the plan gives every workgroup a long walk (few context splits), ragged lengths."""
    ctx = [1500 - 37 * (s % 9) for s in range(48)]
    pb = Problem(d_model=512, n_q_heads=16, n_kv_heads=4, head_dim=128, rank_k=512, rank_v=512, rope_base=500000.0,
                 ctx=ctx, seed=74).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = layer.decode()
    sample = [0, 7, 23, 47]
    ref = oracle_decode(pb, seqs=sample)
    err = rel_err(got[sample], ref)
    print(f"wide batch: rel err {err:.3e}")
    assert np.all(np.isfinite(got)) and err <= TOL


def test_stationary_long_positions():
    """20000 positions of one sequence (many context splits of several tiles), angles up to 3e4 rad at base 500000."""
    pb = Problem(d_model=512, n_q_heads=16, n_kv_heads=4, head_dim=128, rank_k=448, rank_v=448, rope_base=500000.0,
                 ctx=[20000, 777], seed=72).build()
    layer = GpuLayer(pb)
    layer.append_all()
    q_pos = [33000, 776]
    got = layer.decode(q_pos=q_pos)
    ref = oracle_decode(pb, q_pos=q_pos)
    err = [rel_err(got[s], ref[s]) for s in range(2)]
    print(f"long walk: rel err {err[0]:.3e}, {err[1]:.3e}")
    assert max(err) <= TOL


def test_stationary_latent_output_matches_full_output():
    """The latent-space entry point shares the split kernel: o_lat B_v must reproduce the full output."""
    import torch
    pb = Problem(d_model=512, n_q_heads=16, n_kv_heads=4, head_dim=128, rank_k=512, rank_v=512, rope_base=10000.0,
                 ctx=[400, 100], seed=73).build()
    layer = GpuLayer(pb)
    layer.append_all()
    L, dev = layer.L, layer.dev
    q = torch.from_numpy(pb.q).to(dev).to(torch.bfloat16).contiguous()
    qp = torch.tensor([n - 1 for n in pb.ctx], dtype=torch.int32, device=dev)
    cl = torch.tensor(pb.ctx, dtype=torch.int32, device=dev)
    o_lat = L.decode_attention_latent(layer.desc, q, qp, cl, max(pb.ctx), layer.packed, layer.cache, layer.block_table)
    torch.cuda.synchronize()
    o_lat = o_lat.float().cpu().numpy().astype(np.float64)
    B_v = layer.dB_v.float().cpu().numpy().astype(np.float64)
    G, d = pb.n_q_heads // pb.n_kv_heads, pb.head_dim
    got = np.stack([np.stack([o_lat[s, h] @ B_v[:, (h // G) * d:(h // G + 1) * d] for h in range(pb.n_q_heads)])
                    for s in range(len(pb.ctx))])
    assert rel_err(got, oracle_decode(pb)) <= TOL
