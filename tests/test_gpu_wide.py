"""Parity of the three-launch decode path (scores, values in column chunks, merge) against the fp64 oracle:
uncompressed layers (Algorithm 1's threshold, Section 6.2: the pages hold keys and values, no rebuild) and wide
compressed layers (ranks above 1024, Table 2's LLaMA-2-13B row: MHA, n = 5120 -> 2048).  Small model widths keep the
oracle cheap; one case runs the 13B layer shape itself with LAPACK factors."""
import numpy as np
import pytest

from lorc_testlib import GpuLayer, Problem, TOL, numpy_factors, oracle_decode, rel_err

pytestmark = pytest.mark.gpu


def _check(pb, layer, q_pos=None, ref=None, tag=""):
    got = layer.decode(q_pos=q_pos)
    ref = oracle_decode(pb, q_pos=q_pos) if ref is None else ref
    assert np.all(np.isfinite(got))
    for s, N in enumerate(pb.ctx):
        if N == 0:
            assert np.all(got[s] == 0.0)
    live = [s for s, N in enumerate(pb.ctx) if N > 0]
    err = rel_err(got[live], ref[live])
    print(f"{tag}: rel err {err:.3e}")
    assert err <= TOL
    return got


# ---------------------------------------------------------------------------------------------- uncompressed layers
PLAIN = {
    "gqa4_ragged_and_empty": dict(d_model=512, n_q_heads=8, n_kv_heads=2, ctx=[300, 64, 1, 0, 129]),
    "mha_five_heads": dict(d_model=640, n_q_heads=5, n_kv_heads=5, ctx=[200, 130]),
    "g8": dict(d_model=512, n_q_heads=16, n_kv_heads=2, ctx=[1000, 65]),
    "g32_one_kv_head": dict(d_model=256, n_q_heads=32, n_kv_heads=1, ctx=[190]),
    "many_splits": dict(d_model=256, n_q_heads=4, n_kv_heads=2, ctx=[9000]),
}


@pytest.mark.parametrize("name", list(PLAIN))
def test_uncompressed_layer_matches_oracle(name):
    shape = dict(PLAIN[name])
    n = shape["n_kv_heads"] * 128
    pb = Problem(head_dim=128, rank_k=n, rank_v=n, rope_base=500000.0, seed=101 + len(name), **shape).build()
    layer = GpuLayer(pb, plain=True)
    layer.append_all()
    _check(pb, layer, tag=f"uncompressed {name}")


def test_uncompressed_layer_caches_keys_and_values_themselves():
    """What an uncompressed layer stores is x W_k and x W_v (un-rotated), in the documented page tiling."""
    pb = Problem(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, rank_k=256, rank_v=256, rope_base=10000.0,
                 ctx=[100], seed=5).build()
    layer = GpuLayer(pb, plain=True)
    layer.append_all()
    import lorc_inputs as gen
    lat = gen.bf16_to_f32(layer.read_latents(0, 100)).astype(np.float64)
    X = pb.X[0].astype(np.float64)
    Wk = gen.bf16_round(pb.W_k.astype(np.float32)).astype(np.float64)
    Wv = gen.bf16_round(pb.W_v.astype(np.float32)).astype(np.float64)
    ref = np.concatenate([X @ Wk, X @ Wv], axis=1)
    assert np.max(np.abs(lat - ref)) <= 2.0 ** -7 * np.max(np.abs(ref))   # one bf16 rounding of an fp32 sum


def test_uncompressed_8b_shape_full_width():
    """The 8B layer shape left uncompressed (n = 1024, 32 query heads, 8 KV heads), several tiles per split."""
    pb = Problem(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=1024, rank_v=1024, rope_base=500000.0,
                 ctx=[700, 2100], seed=17).build()
    layer = GpuLayer(pb, plain=True)
    layer.append_all()
    _check(pb, layer, tag="uncompressed 8B shape")


def test_uncompressed_8b_shape_in_the_benchmark_launch_configuration():
    """Batch 16, context 4096 (the split plan bench.py's uncompressed_8b leg times); two sequences carry the full
    context and are checked against the oracle."""
    import paper_2410_03111_amd as L
    ctx = [4096, 100] + [64] * 5 + [4033] + [1] * 8
    pb = Problem(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=1024, rank_v=1024, rope_base=500000.0,
                 ctx=ctx, seed=29).build()
    layer = GpuLayer(pb, plain=True)
    layer.append_all()
    got = layer.decode()
    assert np.all(np.isfinite(got))
    sample = [0, 7, 1]
    ref = oracle_decode(pb, seqs=sample)
    err = [rel_err(got[s], ref[i]) for i, s in enumerate(sample)]
    print(f"uncompressed 8B shape, b 16 x ctx 4096: rel err {max(err):.3e}")
    assert max(err) <= TOL


def test_uncompressed_unmapped_page_shifted_and_long_positions():
    import torch
    pb = Problem(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, rank_k=256, rank_v=256, rope_base=500000.0,
                 ctx=[20010, 200], seed=23).build()
    layer = GpuLayer(pb, plain=True)
    bt = layer.block_table_np.copy()
    bt[0, 3] = -1                      # positions 192 .. 255 of sequence 0
    bt[1, 0] = layer.n_pages + 2       # the first tile of sequence 1
    layer.block_table_np = bt
    layer.block_table = torch.from_numpy(bt).to(layer.dev)
    layer.append_all()
    q_pos = [20009, 5000]
    X = [x.copy() for x in pb.X]
    X[0][192:256] = 0.0
    X[1][0:64] = 0.0
    ref = oracle_decode(Problem(**{**pb.__dict__, "X": X}), q_pos=q_pos)
    _check(pb, layer, q_pos=q_pos, ref=ref, tag="uncompressed, unmapped pages, positions to 20 k")


def test_plain_entry_point_refuses_a_compressed_desc():
    import paper_2410_03111_amd as L
    assert L.decode_plain_workspace_bytes(L.layer_desc(512, 8, 2, 128, 128, 256, 1e4), 1, 64) == 0
    assert L.decode_plain_workspace_bytes(L.layer_desc(512, 8, 2, 128, 256, 256, 1e4), 1, 64) > 0
    assert L.decode_plain_workspace_bytes(L.layer_desc(512, 8, 2, 128, 256, 256, 1e4), 1, 0) > 0


# ---------------------------------------------------------------------------------------------- wide compressed layers
WIDE = {
    # two rank parts (64 + 16 k-steps), three value chunks the last of which is a quarter full
    "mha12_r1280_1152": dict(d_model=1536, n_q_heads=12, n_kv_heads=12, rank_k=1280, rank_v=1152, ctx=[200, 70, 0, 1]),
    # query groups of two, ten KV heads (the third head group of the scores kernel is half empty)
    "gqa2_r1088": dict(d_model=1280, n_q_heads=20, n_kv_heads=10, rank_k=768, rank_v=1088, ctx=[330]),
    # one rank part kept in LDS for both passes, but more value columns than the single-pass kernels take
    "mha10_rk1024_rv1280": dict(d_model=1280, n_q_heads=10, n_kv_heads=10, rank_k=1024, rank_v=1280, ctx=[150, 600]),
    # three LDS parts (32 + 32 + 6 k-steps)
    "mha10_rk1120": dict(d_model=1280, n_q_heads=10, n_kv_heads=10, rank_k=1120, rank_v=1056, ctx=[260, 31]),
    # 64 query heads in groups of eight at rank 768: below the wide ranks, but two score blocks per wave
    "q64_g8_r768": dict(d_model=1024, n_q_heads=64, n_kv_heads=8, rank_k=768, rank_v=640, ctx=[700, 64, 0]),
}


@pytest.mark.parametrize("name", list(WIDE))
def test_wide_layer_matches_oracle(name):
    import paper_2410_03111_amd as L
    shape = dict(WIDE[name])
    pb = Problem(head_dim=128, rope_base=500000.0, seed=131 + len(name), **shape).build()
    layer = GpuLayer(pb)
    assert L.decode_plan_info(layer.desc, len(pb.ctx), max(pb.ctx))[0] == "wide_scores_kernel"
    layer.append_all()
    _check(pb, layer, tag=f"wide {name}")


def test_wide_layer_many_splits_unmapped_page_and_latent_output():
    import torch
    import paper_2410_03111_amd as L
    pb = Problem(d_model=1152, n_q_heads=9, n_kv_heads=9, head_dim=128, rank_k=1056, rank_v=1056, rope_base=500000.0,
                 ctx=[2600, 100], seed=37).build()
    layer = GpuLayer(pb)
    bt = layer.block_table_np.copy()
    bt[0, 2] = -1
    layer.block_table_np = bt
    layer.block_table = torch.from_numpy(bt).to(layer.dev)
    layer.append_all()
    q_pos = [3000, 99]
    X = [x.copy() for x in pb.X]
    X[0][128:192] = 0.0
    pbz = Problem(**{**pb.__dict__, "X": X})
    got = _check(pb, layer, q_pos=q_pos, ref=oracle_decode(pbz, q_pos=q_pos), tag="wide, 41 tiles, unmapped page")
    # the latent-space output (before B_v) times B_v is the same result
    q = torch.from_numpy(pb.q).to(layer.dev).to(torch.bfloat16).contiguous()
    lat = L.decode_attention_latent(layer.desc, q, torch.tensor(q_pos, dtype=torch.int32, device=layer.dev),
                                    torch.tensor(pb.ctx, dtype=torch.int32, device=layer.dev), max(pb.ctx), layer.packed,
                                    layer.cache, layer.block_table)
    torch.cuda.synchronize()
    lat = lat.float().cpu().numpy().astype(np.float64)                       # [b, h_q, r_v]
    Bv = layer.dB_v.float().cpu().numpy().astype(np.float64)                 # [r_v, n]
    up = np.stack([np.stack([lat[s, h] @ Bv[:, h * 128:(h + 1) * 128] for h in range(9)]) for s in range(2)])
    assert rel_err(up, got) <= 1e-2


@pytest.fixture(scope="module")
def factors_13b():
    """Table 2 / Table 3: 40 MHA heads of 128, n = D = 5120, keys and values compressed to rank 2048.  Weights of seed
    13 and their factors by LAPACK, once for the module (the library's host factorisation of a 5120 x 5120 matrix
    takes minutes, two LAPACK ones the better part of a minute)."""
    pb = Problem(d_model=5120, n_q_heads=40, n_kv_heads=40, head_dim=128, rank_k=2048, rank_v=2048, rope_base=10000.0,
                 ctx=[1], seed=13).build()
    A_k, B_k, Wt_k = numpy_factors(pb.W_k, 2048)
    A_v, B_v, Wt_v = numpy_factors(pb.W_v, 2048)
    return dict(factors=(A_k, B_k, A_v, B_v), Wt=(Wt_k, Wt_v))


def test_llama2_13b_layer_shape(factors_13b):
    """Two short sequences on the 13B layer shape."""
    import paper_2410_03111_amd as L
    pb = Problem(d_model=5120, n_q_heads=40, n_kv_heads=40, head_dim=128, rank_k=2048, rank_v=2048, rope_base=10000.0,
                 ctx=[150, 70], seed=13).build()
    layer = GpuLayer(pb, factors=factors_13b["factors"])
    assert L.decode_plan_info(layer.desc, 2, 150)[0] == "wide_scores_kernel"
    layer.append_all()
    _check(pb, layer, ref=oracle_decode(pb, Wt=factors_13b["Wt"]), tag="LLaMA-2-13B layer shape")


def test_llama2_13b_layer_shape_in_the_benchmark_launch_configuration(factors_13b):
    """Batch 16, context 4096 (the split plan and grids that bench.py's wide_13b leg times): two sequences carry the
    full context and are checked against the oracle, the other fourteen are short."""
    import paper_2410_03111_amd as L
    ctx = [4096, 37] + [64] * 6 + [4095] + [1] * 7
    pb = Problem(d_model=5120, n_q_heads=40, n_kv_heads=40, head_dim=128, rank_k=2048, rank_v=2048, rope_base=10000.0,
                 ctx=ctx, seed=13).build()
    layer = GpuLayer(pb, factors=factors_13b["factors"])
    name, ns, tps = L.decode_plan_info(layer.desc, 16, 4096)
    assert name == "wide_scores_kernel" and ns * tps >= 64
    layer.append_all()
    got = layer.decode()
    assert np.all(np.isfinite(got))
    sample = [0, 8, 1]
    ref = oracle_decode(pb, seqs=sample, Wt=factors_13b["Wt"])
    err = [rel_err(got[s], ref[i]) for i, s in enumerate(sample)]
    print(f"13B shape, b 16 x ctx 4096 ({ns} splits x {tps} tiles): rel err {max(err):.3e}")
    assert max(err) <= TOL


def test_llama2_13b_uncompressed_layer_shape():
    pb = Problem(d_model=5120, n_q_heads=40, n_kv_heads=40, head_dim=128, rank_k=5120, rank_v=5120, rope_base=10000.0,
                 ctx=[130, 64], seed=19).build()
    layer = GpuLayer(pb, plain=True)
    layer.append_all()
    _check(pb, layer, tag="LLaMA-2-13B layer shape, uncompressed")


# ---------------------------------------------------------------------------------------------- uncompressed layers, prefill
PLAIN_PREFILL = {
    "gqa4_ragged": dict(d_model=512, n_q_heads=8, n_kv_heads=2, ctx=[1, 70, 200, 64, 129]),
    "mha_three_heads": dict(d_model=384, n_q_heads=3, n_kv_heads=3, ctx=[150]),
    "8b_shape": dict(d_model=4096, n_q_heads=32, n_kv_heads=8, ctx=[300, 130]),
}


@pytest.mark.parametrize("name", list(PLAIN_PREFILL))
def test_uncompressed_layer_prefill_matches_oracle(name):
    import lorc_inputs as gen
    from lorc_testlib import oracle_prefill
    shape = dict(PLAIN_PREFILL[name])
    n = shape["n_kv_heads"] * 128
    pb = Problem(head_dim=128, rank_k=n, rank_v=n, rope_base=500000.0, seed=151 + len(name), **shape).build()
    layer = GpuLayer(pb, plain=True)
    layer.append_all()
    Q = [gen.queries(N, pb.n_q_heads, pb.head_dim, seed=7300 + s) for s, N in enumerate(pb.ctx)]
    got = layer.prefill(Q)
    ref = oracle_prefill(pb, Q)
    scale = max(np.max(np.abs(r)) for r in ref)
    worst = 0.0
    for g, r in zip(got, ref):
        assert g.shape == r.shape and np.all(np.isfinite(g))
        worst = max(worst, float(np.max(np.abs(g - r))) / scale)
    print(f"uncompressed prefill {name}: rel err {worst:.3e}")
    assert worst <= TOL
    # the last row of the causal prefill is the decode step over the same cache
    pb.q = np.stack([q[-1] for q in Q])
    dec = layer.decode()
    assert rel_err(np.stack([o[-1] for o in got]), dec) <= 1e-2


# ---------------------------------------------------------------------------------------------- wide layers, prefill
@pytest.mark.parametrize("name", ["mha12_r1280_1152", "gqa2_r1088"])
def test_wide_layer_prefill_matches_oracle(name):
    """Ranks above 1024: the prefill's rebuild launch walks the rank in parts too."""
    import lorc_inputs as gen
    from lorc_testlib import oracle_prefill
    shape = dict(WIDE[name])
    shape["ctx"] = [150, 70]
    pb = Problem(head_dim=128, rope_base=500000.0, seed=171 + len(name), **shape).build()
    layer = GpuLayer(pb)
    layer.append_all()
    Q = [gen.queries(N, pb.n_q_heads, pb.head_dim, seed=7400 + s) for s, N in enumerate(pb.ctx)]
    got = layer.prefill(Q)
    ref = oracle_prefill(pb, Q)
    scale = max(np.max(np.abs(r)) for r in ref)
    worst = max(float(np.max(np.abs(g - r))) / scale for g, r in zip(got, ref))
    print(f"wide prefill {name}: rel err {worst:.3e}")
    assert all(np.all(np.isfinite(g)) for g in got) and worst <= TOL


# ---------------------------------------------------------------------------------------------- edge cases of the three-launch paths
@pytest.mark.parametrize("plain", [True, False])
def test_three_launch_paths_with_empty_and_clamped_contexts(plain):
    """Every context empty with max_ctx = 0; then context lengths beyond max_ctx (clamped to it) and a negative one
    (treated as empty)."""
    import torch
    import paper_2410_03111_amd as L
    if plain:
        pb = Problem(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, rank_k=256, rank_v=256, rope_base=10000.0,
                     ctx=[200, 130, 64], seed=43).build()
    else:
        pb = Problem(d_model=1280, n_q_heads=10, n_kv_heads=10, head_dim=128, rank_k=1056, rank_v=1088, rope_base=10000.0,
                     ctx=[200, 130, 64], seed=44).build()
    layer = GpuLayer(pb, plain=plain)
    layer.append_all()
    got = layer.decode(ctx=[0, 0, 0], max_ctx=0)
    assert np.all(got == 0.0)
    # max_ctx 128: sequence 0 is clamped to its first 128 positions, sequence 1 likewise, sequence 2 is "negative" = empty
    got = layer.decode(q_pos=[127, 127, 0], ctx=[200, 1 << 30, -5], max_ctx=128)
    pb128 = Problem(**{**pb.__dict__, "ctx": [128, 128, 0], "X": [pb.X[0][:128], pb.X[1][:128], pb.X[2][:0]]})
    ref = oracle_decode(pb128, q_pos=[127, 127, 0])
    assert np.all(np.isfinite(got)) and np.all(got[2] == 0.0)
    assert rel_err(got[:2], ref[:2]) <= TOL
