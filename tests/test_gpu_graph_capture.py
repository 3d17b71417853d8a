"""The device entry points only launch kernels once a device's one-time set-up has run, so a decode step (append of
the new token + decode attention without a workspace argument) can be recorded into a HIP graph.  The graph is
replayed several times with eager work and synchronisations between the replays, on changing inputs, and every
replay is checked against the eager call and the oracle."""
import ctypes

import numpy as np
import pytest

from lorc_testlib import GpuLayer, Problem, TOL, oracle_decode, rel_err

pytestmark = pytest.mark.gpu


def test_decode_step_replays_from_a_hip_graph():
    import torch
    import paper_2410_03111_amd as L
    pb = Problem(d_model=512, n_q_heads=16, n_kv_heads=4, head_dim=128, rank_k=512, rank_v=512, rope_base=500000.0,
                 ctx=[700, 129, 64], seed=91).build()
    layer = GpuLayer(pb)
    layer.append_all()                     # also the first device call: the one-time set-up happens here, eagerly
    dev, b = layer.dev, len(pb.ctx)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    q = torch.from_numpy(pb.q).to(dev).to(torch.bfloat16).contiguous()
    q_pos = torch.tensor([n - 1 for n in pb.ctx], dtype=torch.int32, device=dev)
    ctx = torch.tensor(pb.ctx, dtype=torch.int32, device=dev)
    # the step's append: the last token of every sequence again (same values: the cache does not change)
    x_last = torch.from_numpy(np.stack([pb.X[s][-1] for s in range(b)])).to(dev).to(torch.bfloat16).contiguous()
    slot_seq = torch.arange(b, dtype=torch.int32, device=dev)
    out = torch.zeros_like(q)
    max_ctx = max(pb.ctx)

    def step():
        L.append_latent(layer.desc, x_last, layer.packed, slot_seq, q_pos, layer.block_table, layer.cache)
        rc = L._lib.lorc_decode_attention_static(ctypes.byref(layer.desc), ptr(q), ptr(q_pos), ptr(ctx), b, max_ctx,
                                                 ptr(layer.packed), ptr(layer.cache), ptr(layer.block_table),
                                                 layer.max_pages, layer.n_pages, ptr(out),
                                                 ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == L.OK, L.strerror(rc)

    step()
    torch.cuda.synchronize()
    eager = out.float().cpu().numpy().astype(np.float64)
    assert rel_err(eager, oracle_decode(pb)) <= TOL

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    rng = np.random.default_rng(5)
    for rep in range(4):
        # eager work between the replays: new queries (replay must read them from the same buffers), a scrubbed output
        q_new = rng.standard_normal(pb.q.shape).astype(np.float32)
        q.copy_(torch.from_numpy(q_new).to(dev).to(torch.bfloat16))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = out.float().cpu().numpy().astype(np.float64)
        step()                                    # the same step eagerly
        torch.cuda.synchronize()
        ref = out.float().cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got)) and np.array_equal(got, ref), f"replay {rep}"
    pb2 = Problem(**{**pb.__dict__, "q": q.float().cpu().numpy()})
    assert rel_err(got, oracle_decode(pb2)) <= TOL
