"""Seeded random geometries -- group sizes that are not powers of two, unequal ranks, contexts on and around page
boundaries -- through append + decode + causal prefill (and the absorbed-query decode where it is built) against
the oracle.  Complements the fixed grid of test_gpu_shape_sweep.py."""
import numpy as np
import pytest

import lorc_inputs as gen
from lorc_testlib import GpuLayer, Problem, TOL, oracle_decode, oracle_prefill, rel_err
from test_gpu_absorbed import oracle_plain, run_absorbed

pytestmark = pytest.mark.gpu


def _draw(case):
    rng = np.random.default_rng(7000 + case)
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([g for g in (1, 2, 3, 4, 5, 8, 16, 32) if hkv * g <= 64]))
    n = hkv * d
    rk = 32 * int(rng.integers(1, min(n, 1024) // 32 + 1))
    rv = 32 * int(rng.integers(1, min(n, 1024) // 32 + 1))
    ctx = [int(rng.choice([1, 2, 31, 63, 64, 65, 127, 128, 129, int(rng.integers(1, 1500))]))
           for _ in range(int(rng.integers(1, 5)))]
    return d, hkv, G, rk, rv, ctx


@pytest.mark.parametrize("case", range(12))
def test_random_geometry(case):
    d, hkv, G, rk, rv, ctx = _draw(case)
    n, hq = hkv * d, hkv * G
    print(f"d {d} h_kv {hkv} G {G} r_k {rk} r_v {rv} ctx {ctx}", flush=True)
    pb = Problem(d_model=max(256, n), n_q_heads=hq, n_kv_heads=hkv, head_dim=d, rank_k=rk, rank_v=rv, rope_base=10000.0,
                 ctx=ctx, seed=600 + case).build()
    lay = GpuLayer(pb)
    lay.append_all()
    assert rel_err(lay.decode(), oracle_decode(pb)) <= TOL
    Q = [gen.queries(N, hq, d, seed=5 + i).astype(np.float32) for i, N in enumerate(pb.ctx)]
    for got, ref in zip(lay.prefill(Q), oracle_prefill(pb, Q)):
        assert rel_err(got, ref) <= TOL
    if hq <= 32 and rk <= 512 and rv <= 512:
        assert rel_err(run_absorbed(lay), oracle_plain(pb)) <= TOL
