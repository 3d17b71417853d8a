"""Edge cases of the device entry points, through the C ABI: degenerate contexts, shifted query positions, the
largest ranks and query groups the kernels are built for, the error paths that must refuse before launching, and
the full-size benchmark shapes checked on sampled outputs."""
import numpy as np
import pytest

from lorc_testlib import GpuLayer, Problem, TOL, oracle_decode, rel_err

pytestmark = pytest.mark.gpu


def test_empty_context_gives_zero_rows_and_leaves_others_intact():
    pb = Problem(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=64, rope_base=10000.0,
                 ctx=[0, 130, 0, 64], seed=11).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = layer.decode()
    ref = oracle_decode(pb)
    assert np.all(got[0] == 0.0) and np.all(got[2] == 0.0)
    assert rel_err(got[[1, 3]], ref[[1, 3]]) <= TOL


def test_all_contexts_empty():
    pb = Problem(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rank_k=32, rank_v=32, rope_base=10000.0,
                 ctx=[0, 0], seed=12).build()
    layer = GpuLayer(pb)
    got = layer.decode(max_ctx=0)
    assert np.all(got == 0.0)
    got = layer.decode(max_ctx=1)
    assert np.all(got == 0.0)


def test_query_position_is_independent_of_context_length():
    """The query is rotated at q_pos, the keys at their own positions: q_pos need not be ctx_len - 1."""
    pb = Problem(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=96, rank_v=64, rope_base=10000.0,
                 ctx=[150, 70], seed=13).build()
    layer = GpuLayer(pb)
    layer.append_all()
    q_pos = [400, 3]
    got = layer.decode(q_pos=q_pos)
    ref = oracle_decode(pb, q_pos=q_pos)
    assert rel_err(got, ref) <= TOL


def test_shorter_context_than_cached_ignores_the_tail():
    """ctx_len below what is cached attends to the prefix only (the tail stays in the pool, unused)."""
    pb = Problem(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=64, rope_base=10000.0,
                 ctx=[200, 190], seed=14).build()
    layer = GpuLayer(pb)
    layer.append_all()
    short = [77, 128]
    got = layer.decode(ctx=short)
    pb_short = Problem(**{**pb.__dict__, "ctx": short, "X": [x[:n] for x, n in zip(pb.X, short)]})
    ref = oracle_decode(pb_short)
    assert rel_err(got, ref) <= TOL


@pytest.mark.parametrize("shape", [
    dict(d_model=1024, n_q_heads=16, n_kv_heads=8, head_dim=128, rank_k=1024, rank_v=1024, ctx=[140, 65]),  # full rank
    dict(d_model=512, n_q_heads=32, n_kv_heads=1, head_dim=128, rank_k=128, rank_v=96, ctx=[100, 257]),     # G = 32
    dict(d_model=512, n_q_heads=64, n_kv_heads=2, head_dim=64, rank_k=128, rank_v=128, ctx=[90]),           # 64 heads, d 64
], ids=["rank1024_lossless", "one_kv_head_g32", "h64_d64"])
def test_largest_supported_shapes(shape):
    pb = Problem(rope_base=10000.0, seed=15, **shape).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = layer.decode()
    ref = oracle_decode(pb)
    err = rel_err(got, ref)
    print(f"rel err {err:.3e}")
    assert err <= TOL


def test_error_paths_refuse_before_launch():
    """Raw C-ABI calls with bad arguments return the documented codes and launch nothing."""
    import ctypes
    import torch
    import paper_2410_03111_amd as L
    dev = torch.device("cuda:0")
    desc = L.layer_desc(256, 4, 2, 64, 32, 32, 10000.0)
    pbytes = L.page_bytes(desc)
    z = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device=dev)
    packed = L.pack_factors(desc, z(256, 32), z(256, 32), z(32, 128), z(32, 128))
    cache = torch.zeros(4 * pbytes, dtype=torch.uint8, device=dev)
    bt = torch.zeros(1, 2, dtype=torch.int32, device=dev)
    q, out = z(1, 4, 64), z(1, 4, 64)
    qp = torch.zeros(1, dtype=torch.int32, device=dev)
    cl = torch.ones(1, dtype=torch.int32, device=dev)
    ws = torch.zeros(L.decode_workspace_bytes(desc, 1, 64), dtype=torch.uint8, device=dev)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())

    def raw(d, workspace=ws, ws_bytes=None, q_=q, b=1):
        return L._lib.lorc_decode_attention(ctypes.byref(d), ptr(q_) if q_ is not None else None, ptr(qp), ptr(cl), b, 64,
                                            ptr(packed), ptr(cache), ptr(bt), 2, 4, ptr(out), ptr(workspace),
                                            workspace.numel() if ws_bytes is None else ws_bytes, None)

    assert raw(desc) == L.OK
    assert raw(desc, ws_bytes=16) == L.EWORKSPACE
    assert raw(desc, q_=None) == L.EINVAL
    assert raw(desc, b=0) == L.EINVAL
    assert raw(L.layer_desc(256, 4, 2, 96, 32, 32, 10000.0)) == L.EUNSUPPORTED   # head_dim 96
    assert raw(L.layer_desc(256, 4, 2, 64, 40, 32, 10000.0)) == L.EUNSUPPORTED   # rank not a multiple of 32
    assert raw(L.layer_desc(256, 4, 2, 64, 256, 32, 10000.0)) == L.EINVAL        # rank above the KV width
    assert raw(L.layer_desc(256, 5, 2, 64, 32, 32, 10000.0)) == L.EINVAL         # 5 query heads over 2 KV heads
    assert L.strerror(L.EWORKSPACE) and L.strerror(L.EUNSUPPORTED) != L.strerror(L.EINVAL)
    torch.cuda.synchronize()
    # the binding turns a non-zero code into an exception that carries it
    with pytest.raises(L.LorcError) as e:
        L.decode_attention(desc, q, qp, cl, 64, packed, cache, bt, workspace=torch.zeros(16, dtype=torch.uint8, device=dev))
    assert e.value.code == L.EWORKSPACE


def test_prefill_refuses_sequences_beyond_its_32_bit_offsets():
    """One sequence's rebuilt keys must stay below 2 GiB; the check comes before anything is touched."""
    import ctypes
    import torch
    import paper_2410_03111_amd as L
    dev = torch.device("cuda:0")
    desc = L.layer_desc(4096, 32, 8, 128, 512, 512, 500000.0)   # h_kv d = 1024: 2 KiB of keys per position
    z = torch.zeros(64, dtype=torch.bfloat16, device=dev)
    i32 = torch.zeros(4, dtype=torch.int32, device=dev)
    ws = torch.zeros(256, dtype=torch.uint8, device=dev)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    long_seq = 1 << 20   # 2^20 positions x 2 KiB = 2 GiB
    rc = L._lib.lorc_prefill_attention(ctypes.byref(desc), ptr(z), ptr(i32), 1, long_seq, long_seq, ptr(z), ptr(z), ptr(i32),
                                       long_seq // 64, 4, ptr(z), ptr(ws), ws.numel(), None)
    assert rc == L.EUNSUPPORTED
    rc = L._lib.lorc_prefill_attention(ctypes.byref(desc), ptr(z), ptr(i32), 1, long_seq // 2, long_seq // 2, ptr(z), ptr(z), ptr(i32),
                                       long_seq // 128, 4, ptr(z), ptr(ws), ws.numel(), None)
    assert rc == L.EWORKSPACE   # within the limit: the next check (workspace size) is reached, nothing launched
    torch.cuda.synchronize()


def test_append_of_zero_tokens_is_a_no_op():
    import torch
    pb = Problem(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, rank_k=32, rank_v=32, rope_base=10000.0,
                 ctx=[10], seed=16).build()
    layer = GpuLayer(pb)
    before = layer.cache.clone()
    e = torch.zeros(0, dtype=torch.int32, device=layer.dev)
    x = torch.zeros(0, 256, dtype=torch.bfloat16, device=layer.dev)
    try:
        layer.L.append_latent(layer.desc, x, layer.packed, e, e, layer.block_table, layer.cache)
    except layer.L.LorcError as err:  # refusing an empty batch is also acceptable; it must not write
        assert err.code == layer.L.EINVAL
    torch.cuda.synchronize()
    assert torch.equal(before, layer.cache)


def test_unmapped_pages_inside_the_context_read_as_zero_latents():
    """A block-table entry that is negative or beyond the pool, for a page inside ctx_len: append skips its tokens,
    decode treats its positions as zero latents (key 0, value 0), which the oracle reproduces with zeroed hidden
    states.  Nothing outside the pool is touched either way."""
    import torch
    pb = Problem(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=96, rope_base=10000.0,
                 ctx=[300, 200], seed=17).build()
    layer = GpuLayer(pb)
    bt = layer.block_table_np.copy()
    bt[0, 2] = -1                      # positions 128 .. 191 of sequence 0
    bt[1, 0] = layer.n_pages + 5       # positions 0 .. 63 of sequence 1
    layer.block_table_np = bt
    layer.block_table = torch.from_numpy(bt).to(layer.dev)
    layer.append_all()
    got = layer.decode()
    X = [x.copy() for x in pb.X]
    X[0][128:192] = 0.0
    X[1][0:64] = 0.0
    ref = oracle_decode(Problem(**{**pb.__dict__, "X": X}))
    assert np.all(np.isfinite(got))
    err = rel_err(got, ref)
    print(f"unmapped pages: rel err {err:.3e}")
    assert err <= TOL


def test_rotary_decode_at_long_positions():
    """Key positions up to 32767 and query positions beyond them at RoPE base 500000 (the angle position * theta_0
    reaches 4e4 rad): one long and one shifted short sequence at a small model width, so that the fp64 oracle
    stays cheap.  The long context also walks many tiles per split and more than 64 splits."""
    pb = Problem(d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=64, rope_base=500000.0,
                 ctx=[32768, 1000], seed=18).build()
    layer = GpuLayer(pb)
    layer.append_all()
    q_pos = [32767, 40000]
    got = layer.decode(q_pos=q_pos)
    ref = oracle_decode(pb, q_pos=q_pos)
    err = [rel_err(got[s], ref[s]) for s in range(2)]
    print(f"long positions: rel err {err[0]:.3e} (ctx 32768), {err[1]:.3e} (q_pos 40000)")
    assert max(err) <= TOL


def test_stream_read_probe_folds_the_buffer():
    """The bandwidth probe reads every 16-byte element: its sink is written only by a thread whose XOR fold of
    what it read equals a magic word, so one planted element must reach it and an all-zero buffer must not."""
    import torch
    import paper_2410_03111_amd as L
    dev = torch.device("cuda:0")
    n_words = 1 << 22
    for plant in (0, 12345 * 4, n_words - 4):
        buf = torch.zeros(n_words, dtype=torch.int32, device=dev)
        buf[plant] = 0x9E3779B9 - (1 << 32)
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        L.stream_read_probe(buf, sink)
        torch.cuda.synchronize()
        assert int(sink.item()) & 0xFFFFFFFF == 0x9E3779B9
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    L.stream_read_probe(torch.zeros(n_words, dtype=torch.int32, device=dev), sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0


def test_mfma_rate_probe_accumulates_what_it_issues():
    """The matrix-core probe's sink holds, per thread, the sum of its 128 accumulators: 2048 * iters for operands of
    ones (each of the iters x 8 products adds k = 16 to 16 accumulators per lane), 0 for zeros; bad arguments are refused."""
    import torch
    import paper_2410_03111_amd as L
    dev = torch.device("cuda:0")
    wgs, iters = 24, 100
    sink = torch.full((256 * wgs,), -1.0, dtype=torch.float32, device=dev)
    L.mfma_rate_probe(sink, wgs, iters, operands=2)
    torch.cuda.synchronize()
    assert torch.all(sink == 2048.0 * iters)
    L.mfma_rate_probe(sink, wgs, iters, operands=1)
    torch.cuda.synchronize()
    assert torch.all(sink == 0.0)
    L.mfma_rate_probe(sink, wgs, iters, operands=0)
    torch.cuda.synchronize()
    assert torch.all(torch.isfinite(sink)) and float(sink.abs().max()) > 0.0
    for bad in (dict(workgroups=wgs + 1, iters=iters), dict(workgroups=0, iters=iters), dict(workgroups=wgs, iters=0),
                dict(workgroups=wgs, iters=iters, operands=3)):
        with pytest.raises(L.LorcError):
            L.mfma_rate_probe(sink, **bad)


# ---- full-size benchmark shapes, in the launch configuration bench.py times, checked on sampled outputs ----------
def test_config1_full_size_sampled_sequences():
    """configs[1] (8B shape, batch 16, context 4096): the same launch as bench.py (16 x 32 context splits); the
    oracle is evaluated for two of the sixteen sequences."""
    import lorc_inputs as gen
    c = gen.CONFIGS[1]
    pb = Problem(d_model=c["d_model"], n_q_heads=c["n_q_heads"], n_kv_heads=c["n_kv_heads"], head_dim=c["head_dim"],
                 rank_k=c["rank"], rank_v=c["rank"], rope_base=c["rope_base"], ctx=[c["context"]] * c["batch"],
                 seed=c["seed"]).build()
    layer = GpuLayer(pb)
    layer.append_all()
    got = layer.decode()
    assert np.all(np.isfinite(got))
    sample = [3, 12]
    ref = oracle_decode(pb, seqs=sample)
    err = rel_err(got[sample], ref)
    print(f"config1 full size, sequences {sample}: rel err {err:.3e}")
    assert err <= TOL


def test_config3_prefill_full_length_sampled_rows():
    """One configs[3] prompt (8192 tokens, rank 512): large-T append + causal prefill as bench.py launches them;
    sampled query rows against the oracle's decode at that position (the causal row i is decode with context
    i + 1), plus row-stochastic sanity on everything."""
    import lorc_inputs as gen
    from oracle import lorc_oracle as orc
    c = gen.CONFIGS[3]
    N = c["context"]
    pb = Problem(d_model=c["d_model"], n_q_heads=c["n_q_heads"], n_kv_heads=c["n_kv_heads"], head_dim=c["head_dim"],
                 rank_k=c["rank"], rank_v=c["rank"], rope_base=c["rope_base"], ctx=[N], seed=c["seed"]).build()
    Q = [gen.queries(N, pb.n_q_heads, pb.head_dim, seed=777).astype(np.float32)]
    layer = GpuLayer(pb)
    layer.append_all()
    got = layer.prefill(Q)[0]
    assert got.shape == (N, pb.n_q_heads, pb.head_dim) and np.all(np.isfinite(got))
    Wt_k, _ = orc.low_rank_weight(pb.W_k, pb.rank_k)
    Wt_v, _ = orc.low_rank_weight(pb.W_v, pb.rank_v)
    X = pb.X[0].astype(np.float64)
    K = orc.split_heads(X @ Wt_k, pb.n_kv_heads, pb.head_dim)
    V = orc.split_heads(X @ Wt_v, pb.n_kv_heads, pb.head_dim)
    rows = [0, 63, 64, 1000, 4095, 4096, 8191]
    worst = 0.0
    for i in rows:
        ref = orc.attention_decode(Q[0][i].astype(np.float64), i, K[: i + 1], V[: i + 1], np.arange(i + 1), pb.rope_base)
        worst = max(worst, rel_err(got[i], ref))
    print(f"config3 prompt, rows {rows}: worst rel err {worst:.3e}")
    assert worst <= TOL
    # property that holds at any size: an output row is a convex combination of value rows
    vmax = np.abs(V).max()
    assert np.abs(got).max() <= vmax * (1 + TOL)


def test_large_magnitudes_inside_the_documented_range():
    """Hidden states above the usual scale, far inside the fp16 range the header documents for rebuilt keys (6e4).
    x4: logits 16 times larger (a sharp softmax), parity to the usual tolerance.  x64: latents of a few hundred,
    rebuilt keys up to about 3e2, logits in the thousands -- the softmax is an argmax that the bf16 rounding of the
    latents alone can flip, so only what holds regardless is checked: finite outputs inside the hull of the values."""
    for rank in (512, 256):   # stationary and streaming split kernels
        base = Problem(d_model=512, n_q_heads=16, n_kv_heads=4, head_dim=128, rank_k=rank, rank_v=rank, rope_base=500000.0,
                       ctx=[300, 65], seed=77 + rank).build()
        for scale in (4.0, 64.0):
            pb = Problem(**{**base.__dict__, "X": [x * np.float32(scale) for x in base.X]})   # powers of two: still bf16
            layer = GpuLayer(pb)
            layer.append_all()
            got = layer.decode()
            assert np.all(np.isfinite(got))
            if scale == 4.0:
                err = rel_err(got, oracle_decode(pb))
                print(f"rank {rank}, x4 inputs: rel err {err:.3e}")
                assert err <= TOL
            else:
                from oracle import lorc_oracle as orc
                Wt_v, _ = orc.low_rank_weight(pb.W_v, rank)
                for s, N in enumerate(pb.ctx):
                    vmax = np.max(np.abs(pb.X[s].astype(np.float64) @ Wt_v))
                    assert np.max(np.abs(got[s])) <= 1.02 * vmax
