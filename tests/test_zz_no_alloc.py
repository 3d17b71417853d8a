"""The entry point that allocates nothing (split partials in a fixed array inside the library's device code),
called through the C ABI and checked against lorc_decode_attention on the same inputs: two calls in a row on one
stream, the second on a smaller problem, so that whatever the first left in the shared array must not matter."""
import ctypes

import numpy as np
import pytest

from lorc_testlib import GpuLayer, Problem, TOL, oracle_decode, rel_err

pytestmark = pytest.mark.gpu


def _both(pb):
    import torch
    import paper_2410_03111_amd as L
    layer = GpuLayer(pb)
    layer.append_all()
    dev = layer.dev
    b = len(pb.ctx)
    q = torch.from_numpy(pb.q).to(dev).to(torch.bfloat16).contiguous()
    q_pos = torch.tensor([max(n - 1, 0) for n in pb.ctx], dtype=torch.int32, device=dev)
    ctx = torch.tensor(pb.ctx, dtype=torch.int32, device=dev)
    max_ctx = max(pb.ctx)
    ref_out = L.decode_attention(layer.desc, q, q_pos, ctx, max_ctx, layer.packed, layer.cache, layer.block_table)
    out = torch.full_like(q, float("nan"))
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = L._lib.lorc_decode_attention_static(ctypes.byref(layer.desc), ptr(q), ptr(q_pos), ptr(ctx), b, max_ctx,
                                             ptr(layer.packed), ptr(layer.cache), ptr(layer.block_table),
                                             layer.max_pages, layer.n_pages, ptr(out), None)
    assert rc == L.OK, L.strerror(rc)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), ref_out.float().cpu().numpy().astype(np.float64)


def test_static_workspace_entry_point_matches_the_workspace_one():
    import paper_2410_03111_amd as L
    big = Problem(d_model=1024, n_q_heads=32, n_kv_heads=8, head_dim=128, rank_k=256, rank_v=256, rope_base=500000.0,
                  ctx=[1500, 700, 64, 1301], seed=41).build()
    small = Problem(d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=128, rank_k=64, rank_v=96, rope_base=10000.0,
                    ctx=[130, 0, 77], seed=42).build()
    for pb in (big, small):   # second call: smaller input, same device array
        got, ref = _both(pb)
        assert np.all(np.isfinite(got))
        assert np.array_equal(got, ref)   # same kernels, same partials: bit-identical
        assert rel_err(got, oracle_decode(pb)) <= TOL
    # a problem whose partials exceed the array is refused, nothing launched
    import torch
    dev = torch.device("cuda:0")
    desc = L.layer_desc(8192, 64, 8, 128, 512, 512, 500000.0)
    huge_b = 4096
    assert L.decode_workspace_bytes(desc, huge_b, 64) > L.STATIC_WORKSPACE_BYTES
    z = torch.zeros(16, dtype=torch.uint8, device=dev)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = L._lib.lorc_decode_attention_static(ctypes.byref(desc), ptr(z), ptr(z), ptr(z), huge_b, 64, ptr(z), ptr(z),
                                             ptr(z), 1, 1, ptr(z), None)
    assert rc == L.EWORKSPACE
