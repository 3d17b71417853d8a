"""A grid over the geometry the entry points accept -- head_dim, KV heads, group size, unequal K/V ranks up to the
full KV width -- each through append + decode + causal prefill (and the absorbed-query decode where it is built)
against the oracle.  Catches shapes that a launch plan refuses or mis-sizes."""
import itertools

import numpy as np
import pytest

import lorc_inputs as gen
from lorc_testlib import GpuLayer, Problem, TOL, oracle_decode, oracle_prefill, rel_err
from test_gpu_absorbed import oracle_plain, run_absorbed

pytestmark = pytest.mark.gpu

GRID = [(d, hkv, G, rk, rv)
        for d, (hkv, G), (rk, rv) in itertools.product((64, 128), ((1, 32), (2, 4), (8, 8), (8, 4), (2, 16)),
                                                       ((32, 1024), (640, 512), (1024, 32), (256, 160)))
        if hkv * G <= 64]


@pytest.mark.parametrize("d,hkv,G,rk,rv", GRID)
def test_geometry(d, hkv, G, rk, rv):
    n, hq = hkv * d, hkv * G
    rk, rv = min(rk, n), min(rv, n)   # a rank cannot exceed the KV width
    pb = Problem(d_model=max(256, n), n_q_heads=hq, n_kv_heads=hkv, head_dim=d, rank_k=rk, rank_v=rv, rope_base=10000.0,
                 ctx=[130, 70, 1], seed=d + hkv + G + rk).build()
    lay = GpuLayer(pb)
    lay.append_all()
    assert rel_err(lay.decode(), oracle_decode(pb)) <= TOL
    Q = [gen.queries(N, hq, d, seed=5 + i).astype(np.float32) for i, N in enumerate(pb.ctx)]
    for got, ref in zip(lay.prefill(Q), oracle_prefill(pb, Q)):
        assert rel_err(got, ref) <= TOL
    if hq <= 32 and rk <= 512 and rv <= 512:
        assert rel_err(run_absorbed(lay), oracle_plain(pb)) <= TOL
