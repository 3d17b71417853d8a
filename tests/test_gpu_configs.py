"""The benchmark configurations that bench.py does not time, as parity cases at their real layer shapes (reduced
batch and context): configs[2]'s progressive per-layer ranks and configs[4]'s 70B-shaped layer, each through
append + decode (+ a short causal prefill) against the oracle."""
import numpy as np
import pytest

import lorc_inputs as gen
from lorc_testlib import GpuLayer, Problem, TOL, oracle_decode, oracle_prefill, rel_err

pytestmark = pytest.mark.gpu


def config2_ranks():
    c = gen.CONFIGS[2]
    return gen.rank_ramp(c["layers"], c["rank_first"], c["rank_last"])


def test_config2_rank_ramp_has_the_stated_ends_and_mean():
    r = config2_ranks()
    assert r[0] == 768 and r[-1] == 384 and all(a >= b for a, b in zip(r, r[1:])) and all(x % 32 == 0 for x in r)
    assert abs(sum(r) / len(r) - 576) < 1e-9


@pytest.mark.parametrize("layer", [0, 15, 31])
def test_config2_layer_shapes(layer):
    c = gen.CONFIGS[2]
    r = config2_ranks()[layer]
    pb = Problem(d_model=c["d_model"], n_q_heads=c["n_q_heads"], n_kv_heads=c["n_kv_heads"], head_dim=c["head_dim"],
                 rank_k=r, rank_v=r, rope_base=c["rope_base"], ctx=[700, 129, 300], seed=c["seed"] * 100 + layer).build()
    lay = GpuLayer(pb)
    lay.append_all()
    err = rel_err(lay.decode(), oracle_decode(pb))
    print(f"config2 layer {layer} (rank {r}): rel err {err:.3e}")
    assert err <= TOL


def test_config4_layer_shape_decode_and_prefill():
    c = gen.CONFIGS[4]
    pb = Problem(d_model=c["d_model"], n_q_heads=c["n_q_heads"], n_kv_heads=c["n_kv_heads"], head_dim=c["head_dim"],
                 rank_k=c["rank"], rank_v=c["rank"], rope_base=c["rope_base"], ctx=[2100, 640], seed=c["seed"]).build()
    lay = GpuLayer(pb)
    lay.append_all()
    err = rel_err(lay.decode(), oracle_decode(pb))
    print(f"config4 shape decode: rel err {err:.3e}")
    assert err <= TOL
    # causal prefill of the shorter prompt over the same cache
    Q = [None, gen.queries(640, pb.n_q_heads, pb.head_dim, seed=4242).astype(np.float32)]
    pb1 = Problem(**{**pb.__dict__, "ctx": [640], "X": [pb.X[1]], "q": pb.q[1:2]})
    lay1 = GpuLayer(pb1)
    lay1.append_all()
    got = lay1.prefill([Q[1]])[0]
    ref = oracle_prefill(pb1, [Q[1]])[0]
    err = rel_err(got, ref)
    print(f"config4 shape prefill: rel err {err:.3e}")
    assert err <= TOL
