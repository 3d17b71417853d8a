"""Thin Python binding of liblorc.so (C ABI in include/lorc.h): argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used for device memory and streams.
The library is built in-tree by `python paper_2410_03111_amd/build.py` (or __graft_entry__.build()); importing
this package without it raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liblorc.so")

PAGE_TOKENS = 64
OK, EINVAL, EUNSUPPORTED, ENOCONV, EWORKSPACE, EHIP = 0, -1, -2, -3, -4, -5


class LorcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class LayerDesc(ctypes.Structure):
    """Mirror of lorc_layer_desc."""
    _fields_ = [
        ("d_model", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("rank_k", ctypes.c_int32), ("rank_v", ctypes.c_int32),
        ("rope_base", ctypes.c_float), ("softmax_scale", ctypes.c_float), ("page_size", ctypes.c_int32),
    ]

    @property
    def n(self) -> int:
        return self.n_kv_heads * self.head_dim


def layer_desc(d_model, n_q_heads, n_kv_heads, head_dim, rank_k, rank_v, rope_base, softmax_scale=0.0,
               page_size=PAGE_TOKENS) -> LayerDesc:
    return LayerDesc(d_model, n_q_heads, n_kv_heads, head_dim, rank_k, rank_v, rope_base, softmax_scale, page_size)


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2410_03111_amd/build.py`")
    try:
        # torch bundles its own HIP runtime under the same soname; loading torch first makes this library
        # bind to that copy, so that stream handles and device pointers belong to one runtime
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(ctypes.c_double)
    dsc = ctypes.POINTER(LayerDesc)
    sig = {
        "lorc_strerror": (ctypes.c_char_p, [ctypes.c_int]),
        "lorc_factorize": (ctypes.c_int, [dp, i32, i32, i32, dp, dp, dp, dp]),
        "lorc_rank_schedule": (ctypes.c_int, [dp, dp, i32, i32, i32, i32, i32, ctypes.c_double, ctypes.POINTER(i32)]),
        "lorc_error_bound": (ctypes.c_int, [dp, ctypes.POINTER(i32), i32, i32, ctypes.c_double, dp, dp]),
        "lorc_packed_bytes": (sz, [dsc]),
        "lorc_pack_factors": (ctypes.c_int, [dsc, vp, vp, vp, vp, vp, vp]),
        "lorc_page_bytes": (sz, [dsc]),
        "lorc_cache_index_k": (ctypes.c_int64, [dsc, i32, i32]),
        "lorc_cache_index_v": (ctypes.c_int64, [dsc, i32, i32]),
        "lorc_append_latent": (ctypes.c_int, [dsc, vp, i32, vp, vp, vp, vp, i32, i32, i32, vp, vp]),
        "lorc_decode_workspace_bytes": (sz, [dsc, i32, i32]),
        "lorc_decode_plan_info": (ctypes.c_char_p, [dsc, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]),
        "lorc_decode_attention": (ctypes.c_int, [dsc, vp, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp]),
        "lorc_decode_plain_workspace_bytes": (sz, [dsc, i32, i32]),
        "lorc_decode_attention_plain": (ctypes.c_int, [dsc, vp, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp]),
        "lorc_decode_attention_static": (ctypes.c_int, [dsc, vp, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp, vp]),
        "lorc_decode_attention_latent": (ctypes.c_int, [dsc, vp, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp]),
        "lorc_decode_attention_timed": (ctypes.c_int, [dsc, vp, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp, vp, vp]),
        "lorc_decode_absorbed_workspace_bytes": (sz, [dsc, i32, i32]),
        "lorc_decode_attention_absorbed": (ctypes.c_int, [dsc, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp]),
        "lorc_decode_attention_absorbed_timed": (ctypes.c_int, [dsc, vp, vp, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp, vp, vp]),
        "lorc_prefill_workspace_bytes": (sz, [dsc, i32, i32]),
        "lorc_prefill_attention": (ctypes.c_int, [dsc, vp, vp, i32, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp]),
        "lorc_prefill_attention_plain": (ctypes.c_int, [dsc, vp, vp, i32, i32, i32, vp, vp, vp, i32, i32, vp, vp, sz, vp]),
        "lorc_stream_read_probe": (ctypes.c_int, [vp, sz, vp, vp]),
        "lorc_mfma_rate_probe": (ctypes.c_int, [vp, sz, i32, i32, i32, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = _load()
EXPORTS = ("lorc_strerror", "lorc_factorize", "lorc_rank_schedule", "lorc_error_bound", "lorc_packed_bytes", "lorc_pack_factors",
           "lorc_page_bytes", "lorc_cache_index_k", "lorc_cache_index_v", "lorc_append_latent",
           "lorc_decode_workspace_bytes", "lorc_decode_plan_info", "lorc_decode_attention", "lorc_decode_attention_timed",
           "lorc_decode_attention_latent", "lorc_decode_plain_workspace_bytes", "lorc_decode_attention_plain", "lorc_decode_attention_static", "lorc_decode_absorbed_workspace_bytes", "lorc_decode_attention_absorbed",
           "lorc_decode_attention_absorbed_timed",
           "lorc_prefill_workspace_bytes",
           "lorc_prefill_attention", "lorc_prefill_attention_plain", "lorc_stream_read_probe", "lorc_mfma_rate_probe")


def strerror(code: int) -> str:
    return _lib.lorc_strerror(code).decode()


def _check(code: int, where: str):
    if code != OK:
        raise LorcError(code, where)


def _ptr(t):
    return ctypes.c_void_p(None if t is None else t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of dtype {dtype}")
    return t


# ------------------------------------------------------------------------------------------------ host
def factorize(W, rank):
    """lorc_factorize on a numpy fp64 matrix [rows, cols]; returns (A, B, sigma, rel_frob_err)."""
    import numpy as np
    W = np.ascontiguousarray(W, dtype=np.float64)
    rows, cols = W.shape
    A = np.empty((rows, max(rank, 1)), np.float64)
    B = np.empty((max(rank, 1), cols), np.float64)
    sigma = np.empty(cols, np.float64)
    err = ctypes.c_double(0.0)
    dp = ctypes.POINTER(ctypes.c_double)
    _check(_lib.lorc_factorize(W.ctypes.data_as(dp), rows, cols, rank, A.ctypes.data_as(dp), B.ctypes.data_as(dp),
                               sigma.ctypes.data_as(dp), ctypes.byref(err)), "lorc_factorize")
    return A, B, sigma, err.value


def rank_schedule(sigma_k, sigma_v, d_max, d_min, align=32, log_threshold=0.0):
    import numpy as np
    sk = np.ascontiguousarray(sigma_k, dtype=np.float64)
    sv = np.ascontiguousarray(sigma_v, dtype=np.float64)
    L, n = sk.shape
    ranks = np.zeros(L, np.int32)
    dp = ctypes.POINTER(ctypes.c_double)
    _check(_lib.lorc_rank_schedule(sk.ctypes.data_as(dp), sv.ctypes.data_as(dp), L, n, d_max, d_min, align,
                                   float(log_threshold), ranks.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))),
           "lorc_rank_schedule")
    return ranks


def error_bound(sigma, ranks, lipschitz=1.0):
    """Theorem 3 bound of a layer chain: sigma [L, n] decreasing per layer, ranks [L] -> (bound, terms[L])."""
    import numpy as np
    sg = np.ascontiguousarray(sigma, dtype=np.float64)
    rk = np.ascontiguousarray(ranks, dtype=np.int32)
    L, n = sg.shape
    assert rk.shape == (L,)
    terms = np.zeros(L, np.float64)
    bound = ctypes.c_double()
    dp = ctypes.POINTER(ctypes.c_double)
    _check(_lib.lorc_error_bound(sg.ctypes.data_as(dp), rk.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), L, n,
                                 float(lipschitz), terms.ctypes.data_as(dp), ctypes.byref(bound)), "lorc_error_bound")
    return bound.value, terms


def page_bytes(desc: LayerDesc) -> int:
    return _lib.lorc_page_bytes(ctypes.byref(desc))


def packed_bytes(desc: LayerDesc) -> int:
    return _lib.lorc_packed_bytes(ctypes.byref(desc))


def cache_index_k(desc: LayerDesc, slot: int, j: int) -> int:
    return _lib.lorc_cache_index_k(ctypes.byref(desc), slot, j)


def cache_index_v(desc: LayerDesc, slot: int, j: int) -> int:
    return _lib.lorc_cache_index_v(ctypes.byref(desc), slot, j)


def decode_workspace_bytes(desc: LayerDesc, b: int, max_ctx: int) -> int:
    return _lib.lorc_decode_workspace_bytes(ctypes.byref(desc), b, max_ctx)


def decode_plan_info(desc: LayerDesc, b: int, max_ctx: int):
    """(split kernel name, context splits per sequence, 64-position tiles per split) of the decode launch."""
    ns, tps = ctypes.c_int32(0), ctypes.c_int32(0)
    name = _lib.lorc_decode_plan_info(ctypes.byref(desc), b, max_ctx, ctypes.byref(ns), ctypes.byref(tps))
    if name is None:
        raise LorcError(EUNSUPPORTED, "lorc_decode_plan_info")
    return name.decode(), ns.value, tps.value


def decode_absorbed_workspace_bytes(desc: LayerDesc, b: int, max_ctx: int) -> int:
    return _lib.lorc_decode_absorbed_workspace_bytes(ctypes.byref(desc), b, max_ctx)


def prefill_workspace_bytes(desc: LayerDesc, b: int, max_seqlen: int) -> int:
    return _lib.lorc_prefill_workspace_bytes(ctypes.byref(desc), b, max_seqlen)


# ------------------------------------------------------------------------------------------------ device
def pack_factors(desc: LayerDesc, A_k, A_v, B_k, B_v, packed=None):
    """A_k [D, r_k], A_v [D, r_v], B_k [r_k, n], B_v [r_v, n] bf16 CUDA tensors -> packed uint8 buffer.

    B_k = B_v = None packs an uncompressed layer (rank_k = rank_v = n, A = W)."""
    import torch
    for t, nm in ((A_k, "A_k"), (A_v, "A_v")) + (() if B_k is None and B_v is None else ((B_k, "B_k"), (B_v, "B_v"))):
        _dev(t, torch.bfloat16, nm)
    assert tuple(A_k.shape) == (desc.d_model, desc.rank_k) and tuple(A_v.shape) == (desc.d_model, desc.rank_v)
    if B_k is not None or B_v is not None:
        assert tuple(B_k.shape) == (desc.rank_k, desc.n) and tuple(B_v.shape) == (desc.rank_v, desc.n)
    nbytes = packed_bytes(desc)
    if nbytes == 0:
        raise LorcError(EUNSUPPORTED, "lorc_packed_bytes")
    if packed is None:
        packed = torch.empty(nbytes, dtype=torch.uint8, device=A_k.device)
    _check(_lib.lorc_pack_factors(ctypes.byref(desc), _ptr(A_k), _ptr(A_v), _ptr(B_k), _ptr(B_v), _ptr(packed),
                                  _stream()), "lorc_pack_factors")
    return packed


def append_latent(desc: LayerDesc, x, packed, slot_seq, slot_pos, block_table, cache):
    """x [T, D] bf16; slot_seq/slot_pos [T] int32; block_table [n_seqs, max_pages] int32; cache uint8 pool."""
    import torch
    _dev(x, torch.bfloat16, "x")
    _dev(slot_seq, torch.int32, "slot_seq")
    _dev(slot_pos, torch.int32, "slot_pos")
    _dev(block_table, torch.int32, "block_table")
    _dev(cache, torch.uint8, "cache")
    T = x.shape[0]
    assert x.shape[1] == desc.d_model and slot_seq.numel() == T and slot_pos.numel() == T
    n_seqs, max_pages = block_table.shape
    n_pages = cache.numel() // page_bytes(desc)
    _check(_lib.lorc_append_latent(ctypes.byref(desc), _ptr(x), T, _ptr(packed), _ptr(slot_seq), _ptr(slot_pos),
                                   _ptr(block_table), n_seqs, max_pages, n_pages, _ptr(cache), _stream()),
           "lorc_append_latent")


def decode_attention_latent(desc: LayerDesc, q, q_pos, ctx_len, max_ctx, packed, cache, block_table, out=None,
                            workspace=None):
    """Decode attention that stops in latent space: out [b, h_q, r_v] bf16 (see lorc_decode_attention_latent)."""
    import torch
    _dev(q, torch.bfloat16, "q")
    _dev(q_pos, torch.int32, "q_pos")
    _dev(ctx_len, torch.int32, "ctx_len")
    _dev(block_table, torch.int32, "block_table")
    _dev(cache, torch.uint8, "cache")
    b = q.shape[0]
    assert tuple(q.shape) == (b, desc.n_q_heads, desc.head_dim)
    n_seqs, max_pages = block_table.shape
    assert n_seqs >= b
    n_pages = cache.numel() // page_bytes(desc)
    need = decode_workspace_bytes(desc, b, max_ctx)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty(b, desc.n_q_heads, desc.rank_v, dtype=torch.bfloat16, device=q.device)
    _check(_lib.lorc_decode_attention_latent(ctypes.byref(desc), _ptr(q), _ptr(q_pos), _ptr(ctx_len), b, max_ctx,
                                             _ptr(packed), _ptr(cache), _ptr(block_table), max_pages, n_pages,
                                             _ptr(out), _ptr(workspace), workspace.numel(), _stream()),
           "lorc_decode_attention_latent")
    return out


def decode_attention(desc: LayerDesc, q, q_pos, ctx_len, max_ctx, packed, cache, block_table, out=None,
                     workspace=None, events=None):
    """q [b, h_q, d] bf16 (un-rotated); q_pos, ctx_len [b] int32 -> out [b, h_q, d] bf16.

    events: optional (begin, end) raw hipEvent_t handles recorded around the split kernel."""
    import torch
    _dev(q, torch.bfloat16, "q")
    _dev(q_pos, torch.int32, "q_pos")
    _dev(ctx_len, torch.int32, "ctx_len")
    _dev(block_table, torch.int32, "block_table")
    _dev(cache, torch.uint8, "cache")
    b = q.shape[0]
    assert tuple(q.shape) == (b, desc.n_q_heads, desc.head_dim)
    n_seqs, max_pages = block_table.shape
    assert n_seqs >= b
    n_pages = cache.numel() // page_bytes(desc)
    need = decode_workspace_bytes(desc, b, max_ctx)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty_like(q)
    args = (ctypes.byref(desc), _ptr(q), _ptr(q_pos), _ptr(ctx_len), b, max_ctx, _ptr(packed), _ptr(cache),
            _ptr(block_table), max_pages, n_pages, _ptr(out), _ptr(workspace), workspace.numel(), _stream())
    if events is None:
        _check(_lib.lorc_decode_attention(*args), "lorc_decode_attention")
    else:
        _check(_lib.lorc_decode_attention_timed(*args, ctypes.c_void_p(events[0]), ctypes.c_void_p(events[1])),
               "lorc_decode_attention_timed")
    return out


def decode_plain_workspace_bytes(desc: LayerDesc, b: int, max_ctx: int) -> int:
    return _lib.lorc_decode_plain_workspace_bytes(ctypes.byref(desc), b, max_ctx)


def decode_attention_plain(desc: LayerDesc, q, q_pos, ctx_len, max_ctx, packed, cache, block_table, out=None,
                           workspace=None):
    """Decode attention over an uncompressed layer (see lorc_decode_attention_plain): out [b, h_q, d] bf16."""
    import torch
    _dev(q, torch.bfloat16, "q")
    _dev(q_pos, torch.int32, "q_pos")
    _dev(ctx_len, torch.int32, "ctx_len")
    _dev(block_table, torch.int32, "block_table")
    _dev(cache, torch.uint8, "cache")
    b = q.shape[0]
    assert tuple(q.shape) == (b, desc.n_q_heads, desc.head_dim)
    n_seqs, max_pages = block_table.shape
    assert n_seqs >= b
    n_pages = cache.numel() // page_bytes(desc)
    need = decode_plain_workspace_bytes(desc, b, max_ctx)
    if need == 0:
        raise LorcError(EUNSUPPORTED, "lorc_decode_plain_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty_like(q)
    _check(_lib.lorc_decode_attention_plain(ctypes.byref(desc), _ptr(q), _ptr(q_pos), _ptr(ctx_len), b, max_ctx,
                                            _ptr(packed), _ptr(cache), _ptr(block_table), max_pages, n_pages,
                                            _ptr(out), _ptr(workspace), workspace.numel(), _stream()),
           "lorc_decode_attention_plain")
    return out


STATIC_WORKSPACE_BYTES = 32 << 20


def decode_attention_static(desc: LayerDesc, q, q_pos, ctx_len, max_ctx, packed, cache, block_table, out):
    """lorc_decode_attention_static: no workspace argument, nothing allocated (the caller passes `out`)."""
    import torch
    _dev(q, torch.bfloat16, "q")
    _dev(q_pos, torch.int32, "q_pos")
    _dev(ctx_len, torch.int32, "ctx_len")
    _dev(block_table, torch.int32, "block_table")
    _dev(cache, torch.uint8, "cache")
    _dev(out, torch.bfloat16, "out")
    b = q.shape[0]
    assert tuple(q.shape) == (b, desc.n_q_heads, desc.head_dim) and tuple(out.shape) == tuple(q.shape)
    n_seqs, max_pages = block_table.shape
    assert n_seqs >= b
    n_pages = cache.numel() // page_bytes(desc)
    _check(_lib.lorc_decode_attention_static(ctypes.byref(desc), _ptr(q), _ptr(q_pos), _ptr(ctx_len), b, max_ctx,
                                             _ptr(packed), _ptr(cache), _ptr(block_table), max_pages, n_pages,
                                             _ptr(out), _stream()), "lorc_decode_attention_static")
    return out


def decode_attention_absorbed(desc: LayerDesc, q_lat, ctx_len, max_ctx, packed, cache, block_table, out=None,
                              workspace=None, events=None):
    """No positional rotation, key factor folded into the query: q_lat [b, h_q, r_k] bf16 -> out [b, h_q, d] bf16.

    events: optional (begin, end) raw hipEvent_t handles recorded around the streaming kernel."""
    import torch
    _dev(q_lat, torch.bfloat16, "q_lat")
    _dev(ctx_len, torch.int32, "ctx_len")
    _dev(block_table, torch.int32, "block_table")
    _dev(cache, torch.uint8, "cache")
    b = q_lat.shape[0]
    assert tuple(q_lat.shape) == (b, desc.n_q_heads, desc.rank_k)
    n_seqs, max_pages = block_table.shape
    assert n_seqs >= b
    n_pages = cache.numel() // page_bytes(desc)
    need = decode_absorbed_workspace_bytes(desc, b, max_ctx)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q_lat.device)
    if out is None:
        out = torch.empty(b, desc.n_q_heads, desc.head_dim, dtype=torch.bfloat16, device=q_lat.device)
    args = (ctypes.byref(desc), _ptr(q_lat), _ptr(ctx_len), b, max_ctx, _ptr(packed), _ptr(cache), _ptr(block_table),
            max_pages, n_pages, _ptr(out), _ptr(workspace), workspace.numel(), _stream())
    if events is None:
        _check(_lib.lorc_decode_attention_absorbed(*args), "lorc_decode_attention_absorbed")
    else:
        _check(_lib.lorc_decode_attention_absorbed_timed(*args, ctypes.c_void_p(events[0]), ctypes.c_void_p(events[1])),
               "lorc_decode_attention_absorbed_timed")
    return out


def prefill_attention(desc: LayerDesc, q, cu_seqlens, max_seqlen, packed, cache, block_table, out=None,
                      workspace=None, plain=False):
    """q [total, h_q, d] bf16 packed over sequences; cu_seqlens [b+1] int32 -> out [total, h_q, d] bf16.

    plain: the layer is uncompressed (lorc_prefill_attention_plain)."""
    import torch
    _dev(q, torch.bfloat16, "q")
    _dev(cu_seqlens, torch.int32, "cu_seqlens")
    _dev(block_table, torch.int32, "block_table")
    _dev(cache, torch.uint8, "cache")
    total = q.shape[0]
    b = cu_seqlens.numel() - 1
    n_seqs, max_pages = block_table.shape
    n_pages = cache.numel() // page_bytes(desc)
    need = prefill_workspace_bytes(desc, b, max_seqlen)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty_like(q)
    fn, name = ((_lib.lorc_prefill_attention_plain, "lorc_prefill_attention_plain") if plain else
                (_lib.lorc_prefill_attention, "lorc_prefill_attention"))
    _check(fn(ctypes.byref(desc), _ptr(q), _ptr(cu_seqlens), b, total, max_seqlen, _ptr(packed), _ptr(cache),
              _ptr(block_table), max_pages, n_pages, _ptr(out), _ptr(workspace), workspace.numel(), _stream()), name)
    return out


def mfma_rate_probe(sink, workgroups: int, iters: int, operands: int = 0):
    """Launches the matrix-core rate probe (4 * workgroups * iters * 8 * 32768 flop); sink: float32, >= 256 * workgroups."""
    _check(_lib.lorc_mfma_rate_probe(_ptr(sink), sink.numel(), workgroups, iters, operands, _stream()), "lorc_mfma_rate_probe")


def stream_read_probe(src, sink):
    _check(_lib.lorc_stream_read_probe(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()),
           "lorc_stream_read_probe")
