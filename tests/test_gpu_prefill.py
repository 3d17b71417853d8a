"""lorc_prefill_attention on the GPU against the fp64 oracle, and its consistency with the decode path."""
import numpy as np
import pytest

import lorc_inputs as gen
from lorc_testlib import GpuLayer, Problem, TOL, oracle_prefill, rel_err

pytestmark = pytest.mark.gpu

SHAPES = {
    "tiny_d64": dict(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rank_k=32, rank_v=32,
                     rope_base=10000.0, ctx=[128], seed=10),
    "ragged_mid": dict(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=96,
                       rope_base=10000.0, ctx=[1, 70, 200, 64, 129], seed=11),
    "llama8b_short": dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=512, rank_v=512,
                          rope_base=500000.0, ctx=[300, 130], seed=12),
    # groupings that deal the workgroup's waves differently: one head x four query sub-blocks, and a group of three
    # (a pass of two heads, then a pass with one head and idle waves)
    "mha_ragged": dict(d_model=512, n_q_heads=4, n_kv_heads=4, head_dim=128, rank_k=96, rank_v=64,
                       rope_base=10000.0, ctx=[1, 33, 200, 290, 128], seed=14),
    "g3_d64": dict(d_model=256, n_q_heads=6, n_kv_heads=2, head_dim=64, rank_k=64, rank_v=32,
                   rope_base=10000.0, ctx=[97, 260], seed=15),
    "g8_rank768": dict(d_model=1024, n_q_heads=64, n_kv_heads=8, head_dim=128, rank_k=768, rank_v=640,
                       rope_base=500000.0, ctx=[150, 67], seed=13),
}


def make_queries(pb, seed):
    return [gen.queries(N, pb.n_q_heads, pb.head_dim, seed=seed + s) for s, N in enumerate(pb.ctx)]


@pytest.mark.parametrize("name", list(SHAPES))
def test_prefill_matches_oracle(name):
    pb = Problem(**SHAPES[name]).build()
    layer = GpuLayer(pb)
    layer.append_all()
    Q = make_queries(pb, 7000)
    got = layer.prefill(Q)
    ref = oracle_prefill(pb, Q)
    scale = max(np.max(np.abs(r)) for r in ref)
    worst = 0.0
    for g, r in zip(got, ref):
        assert g.shape == r.shape and np.all(np.isfinite(g))
        worst = max(worst, float(np.max(np.abs(g - r))) / scale)
    print(f"{name}: rel err {worst:.3e}")
    assert worst <= TOL


def test_last_prefill_row_equals_decode():
    """Row N-1 of the causal prefill is the decode step with ctx_len = N (same query)."""
    pb = Problem(**SHAPES["ragged_mid"]).build()
    layer = GpuLayer(pb)
    layer.append_all()
    Q = make_queries(pb, 7100)
    pb.q = np.stack([q[-1] for q in Q])
    pre = layer.prefill(Q)
    dec = layer.decode()
    last = np.stack([o[-1] for o in pre])
    assert rel_err(last, dec) <= 1e-2
