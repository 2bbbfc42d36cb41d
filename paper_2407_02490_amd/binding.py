"""Thin ctypes binding over the C ABI of libminf (include/minf.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch is used for device memory and streams.  There is no CPU fallback: if
the shared library has not been built, importing the entry points raises.
"""
import ctypes
import os

import numpy as np
import torch

__all__ = [
    "lib", "MinfError", "VSIndex", "BSIndex", "alloc_vs_index", "alloc_bs_index",
    "vs_index_from_host", "bs_index_from_host",
    "minf_build_vs_index", "minf_build_vs_index_noalloc", "minf_vs_index_from_lines", "minf_build_bs_index", "minf_ashape_attn", "minf_vs_attn", "minf_vs_bs_attn",
    "minf_bs_attn", "minf_dense_attn", "minf_vs_cover_words",
    "minf_vs_index_workspace_bytes", "minf_bs_index_workspace_bytes",
]

BLOCK = 64
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libminf.so")
_lib = None


class MinfError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"minf status {status}: {msg}")
        self.status = status


class _QKV(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("o", ctypes.c_void_p),
                ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
                ("v_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3),
                ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("seq_len", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class _VSIndex(ctypes.Structure):
    _fields_ = [("v_idx", ctypes.c_void_p), ("s_idx", ctypes.c_void_p), ("cover", ctypes.c_void_p),
                ("cover_bits", ctypes.c_void_p), ("counts", ctypes.c_void_p),
                ("nv", ctypes.c_int32), ("ns", ctypes.c_int32), ("block", ctypes.c_int32),
                ("cover_words", ctypes.c_int32)]


class _BSIndex(ctypes.Structure):
    _fields_ = [("blk_idx", ctypes.c_void_p), ("blk_cnt", ctypes.c_void_p), ("order", ctypes.c_void_p),
                ("topk", ctypes.c_int32), ("block", ctypes.c_int32)]


def lib():
    """Load libminf.so (built in-tree by __graft_entry__.build()); fail loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                          "g.build()'` at the repository root (there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    i32, vp, sz = ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t
    pq, pi = ctypes.POINTER(_QKV), ctypes.POINTER(ctypes.c_int32)
    L.minf_status_string.restype = ctypes.c_char_p
    L.minf_status_string.argtypes = [ctypes.c_int]
    L.minf_vs_cover_words.restype = i32
    L.minf_vs_cover_words.argtypes = [i32]
    L.minf_vs_index_workspace_bytes.restype = sz
    L.minf_vs_index_workspace_bytes.argtypes = [pq, i32, i32]
    L.minf_bs_index_workspace_bytes.restype = sz
    L.minf_bs_index_workspace_bytes.argtypes = [pq, i32, i32]
    L.minf_build_vs_index.restype = ctypes.c_int
    L.minf_build_vs_index.argtypes = [pq, pi, i32, i32, i32, i32, i32, ctypes.POINTER(_VSIndex), vp, sz, vp]
    L.minf_build_vs_index_noalloc.restype = ctypes.c_int
    L.minf_build_vs_index_noalloc.argtypes = [pq, pi, i32, i32, i32, i32, i32, ctypes.POINTER(_VSIndex), vp]
    L.minf_vs_index_from_lines.restype = ctypes.c_int
    L.minf_vs_index_from_lines.argtypes = [i32, i32, ctypes.POINTER(_VSIndex), vp]
    L.minf_build_bs_index.restype = ctypes.c_int
    L.minf_build_bs_index.argtypes = [pq, pi, i32, i32, i32, ctypes.POINTER(_BSIndex), vp, sz, vp]
    L.minf_ashape_attn.restype = ctypes.c_int
    L.minf_ashape_attn.argtypes = [pq, pi, i32, i32, i32, vp]
    L.minf_dense_attn.restype = ctypes.c_int
    L.minf_dense_attn.argtypes = [pq, pi, i32, vp]
    L.minf_vs_attn.restype = ctypes.c_int
    L.minf_vs_attn.argtypes = [pq, pi, i32, ctypes.POINTER(_VSIndex), vp]
    L.minf_bs_attn.restype = ctypes.c_int
    L.minf_bs_attn.argtypes = [pq, pi, i32, ctypes.POINTER(_BSIndex), vp]
    L.minf_vs_bs_attn.restype = ctypes.c_int
    L.minf_vs_bs_attn.argtypes = [pq, pi, i32, ctypes.POINTER(_VSIndex), pi, i32, ctypes.POINTER(_BSIndex), vp]
    _lib = L
    return L


def _check(status):
    if status != 0:
        raise MinfError(status, lib().minf_status_string(status).decode())


def _strides4(t):
    """(batch, head, token) element strides of a [B, H, N, d] or [H, N, d] tensor."""
    if t.dim() == 3:
        return (0, t.stride(0), t.stride(1)), 1
    return (t.stride(0), t.stride(1), t.stride(2)), t.shape[0]


def _qkv(q, k, v=None, o=None, scale=0.0):
    for t in (q, k, v, o):
        if t is not None:
            assert t.dtype == torch.bfloat16 and t.stride(-1) == 1, "bf16, head_dim contiguous"
    x = _QKV()
    (qs, batch) = _strides4(q)
    x.q, x.k = q.data_ptr(), k.data_ptr()
    x.v = v.data_ptr() if v is not None else None
    x.o = o.data_ptr() if o is not None else None
    x.q_stride[:] = qs
    x.k_stride[:] = _strides4(k)[0]
    x.v_stride[:] = _strides4(v)[0] if v is not None else (0, 0, 0)
    x.o_stride[:] = _strides4(o)[0] if o is not None else (0, 0, 0)
    x.batch = batch
    x.n_q_heads, x.n_kv_heads = q.shape[-3], k.shape[-3]
    x.seq_len, x.head_dim = q.shape[-2], q.shape[-1]
    x.softmax_scale = float(scale)
    return x


def _heads(heads):
    n = len(heads)
    return (ctypes.c_int32 * n)(*[int(h) for h in heads]), n


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class VSIndex:
    """Device buffers of a Vertical-Slash index for `rows` heads (see minf_vs_index)."""

    def __init__(self, rows, nv, ns, seq_len, device):
        self.rows, self.nv, self.ns, self.seq_len = rows, nv, ns, seq_len
        self.cover_words = int(lib().minf_vs_cover_words(seq_len))
        kw = dict(dtype=torch.int32, device=device)
        self.v_idx = torch.empty(rows, nv, **kw)
        self.s_idx = torch.empty(rows, ns, **kw)
        self.cover = torch.empty(rows, ns, 2, **kw)
        self.cover_bits = torch.empty(rows, self.cover_words, **kw)
        self.counts = torch.zeros(rows, 4, **kw)

    def c_struct(self):
        s = _VSIndex()
        s.v_idx, s.s_idx, s.cover = self.v_idx.data_ptr(), self.s_idx.data_ptr(), self.cover.data_ptr()
        s.cover_bits, s.counts = self.cover_bits.data_ptr(), self.counts.data_ptr()
        s.nv, s.ns, s.block, s.cover_words = self.nv, self.ns, BLOCK, self.cover_words
        return s


class BSIndex:
    """Device buffers of a Block-Sparse index for `rows` heads (see minf_bs_index)."""

    def __init__(self, rows, n_blocks, topk, device, with_order=True):
        self.rows, self.n_blocks, self.topk = rows, n_blocks, topk
        self.blk_idx = torch.empty(rows, n_blocks, topk, dtype=torch.int32, device=device)
        self.blk_cnt = torch.empty(rows, n_blocks, dtype=torch.int32, device=device)
        self.order = torch.empty(rows, n_blocks, dtype=torch.int32, device=device) if with_order else None

    def c_struct(self):
        s = _BSIndex()
        s.blk_idx, s.blk_cnt = self.blk_idx.data_ptr(), self.blk_cnt.data_ptr()
        s.order = self.order.data_ptr() if self.order is not None else None
        s.topk, s.block = self.topk, BLOCK
        return s


def alloc_vs_index(rows, nv, ns, seq_len, device="cuda"):
    return VSIndex(rows, nv, ns, seq_len, device)


def alloc_bs_index(rows, seq_len, topk, device="cuda"):
    return BSIndex(rows, seq_len // BLOCK, topk, device)


def vs_index_from_host(v_lists, s_lists, seq_len, device="cuda", stream=None):
    """Index buffers filled from host lists of vertical positions and slash
    offsets (one pair per head, each ascending and distinct): the "static
    index" use of the attention call.  The lists are copied to the device as
    they are; minf_vs_index_from_lines builds the merged offset runs and the
    run bitmap there."""
    rows = len(v_lists)
    nv = max(1, max(len(v) for v in v_lists))
    ns = max(1, max(len(s) for s in s_lists))
    idx = VSIndex(rows, nv, ns, seq_len, device)
    v_idx = np.zeros((rows, nv), np.int32)
    s_idx = np.zeros((rows, ns), np.int32)
    counts = np.zeros((rows, 4), np.int32)
    for r in range(rows):
        v_idx[r, :len(v_lists[r])] = v_lists[r]
        s_idx[r, :len(s_lists[r])] = s_lists[r]
        counts[r, :2] = (len(v_lists[r]), len(s_lists[r]))
    idx.v_idx.copy_(torch.from_numpy(v_idx))
    idx.s_idx.copy_(torch.from_numpy(s_idx))
    idx.counts.copy_(torch.from_numpy(counts))
    minf_vs_index_from_lines(idx, stream=stream)
    return idx


def bs_index_from_host(blk_idx, blk_cnt, order=None, device="cuda"):
    """Index buffers from host arrays blk_idx [rows, NB, topk], blk_cnt [rows, NB] and,
    optionally, a processing order [rows, NB] (None: natural order)."""
    blk_idx = np.asarray(blk_idx, dtype=np.int32)
    blk_cnt = np.asarray(blk_cnt, dtype=np.int32)
    rows, NB, topk = blk_idx.shape
    idx = BSIndex(rows, NB, topk, device, with_order=order is not None)
    idx.blk_idx.copy_(torch.from_numpy(blk_idx))
    idx.blk_cnt.copy_(torch.from_numpy(blk_cnt))
    if order is not None:
        idx.order.copy_(torch.from_numpy(np.asarray(order, dtype=np.int32)))
    return idx


# ---------------------------------------------------------------- entry points
def minf_vs_cover_words(seq_len):
    return int(lib().minf_vs_cover_words(seq_len))


def minf_vs_index_workspace_bytes(q, k, n_heads, last_q=64):
    x = _qkv(q, k)
    return int(lib().minf_vs_index_workspace_bytes(ctypes.byref(x), n_heads, last_q))


def minf_bs_index_workspace_bytes(q, k, n_heads, topk=None):
    """topk=None: enough for any budget (the size of the unfused path)."""
    x = _qkv(q, k)
    return int(lib().minf_bs_index_workspace_bytes(ctypes.byref(x), n_heads, 2 ** 31 - 1 if topk is None else topk))


def minf_build_vs_index(q, k, heads, last_q, nv, ns, out, ws, block=BLOCK, scale=0.0, stream=None):
    x = _qkv(q, k, scale=scale)
    h, n = _heads(heads)
    s = out.c_struct()
    _check(lib().minf_build_vs_index(ctypes.byref(x), h, n, last_q, nv, ns, block, ctypes.byref(s),
                                     ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size(),
                                     _stream(stream)))


def minf_build_vs_index_noalloc(q, k, heads, last_q, nv, ns, out, block=BLOCK, scale=0.0, stream=None):
    x = _qkv(q, k, scale=scale)
    h, n = _heads(heads)
    s = out.c_struct()
    _check(lib().minf_build_vs_index_noalloc(ctypes.byref(x), h, n, last_q, nv, ns, block, ctypes.byref(s),
                                             _stream(stream)))


def minf_vs_index_from_lines(idx, stream=None):
    s = idx.c_struct()
    _check(lib().minf_vs_index_from_lines(idx.seq_len, idx.rows, ctypes.byref(s), _stream(stream)))


def minf_build_bs_index(q, k, heads, topk, out, ws, block=BLOCK, scale=0.0, stream=None):
    x = _qkv(q, k, scale=scale)
    h, n = _heads(heads)
    s = out.c_struct()
    _check(lib().minf_build_bs_index(ctypes.byref(x), h, n, block, topk, ctypes.byref(s),
                                     ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size(),
                                     _stream(stream)))


def minf_ashape_attn(q, k, v, o, heads, n_init, n_local, scale=0.0, stream=None):
    x = _qkv(q, k, v, o, scale)
    h, n = _heads(heads)
    _check(lib().minf_ashape_attn(ctypes.byref(x), h, n, n_init, n_local, _stream(stream)))


def minf_dense_attn(q, k, v, o, heads, scale=0.0, stream=None):
    x = _qkv(q, k, v, o, scale)
    h, n = _heads(heads)
    _check(lib().minf_dense_attn(ctypes.byref(x), h, n, _stream(stream)))


def minf_vs_attn(q, k, v, o, heads, idx, scale=0.0, stream=None):
    x = _qkv(q, k, v, o, scale)
    h, n = _heads(heads)
    s = idx.c_struct()
    _check(lib().minf_vs_attn(ctypes.byref(x), h, n, ctypes.byref(s), _stream(stream)))


def minf_bs_attn(q, k, v, o, heads, idx, scale=0.0, stream=None):
    x = _qkv(q, k, v, o, scale)
    h, n = _heads(heads)
    s = idx.c_struct()
    _check(lib().minf_bs_attn(ctypes.byref(x), h, n, ctypes.byref(s), _stream(stream)))


def minf_vs_bs_attn(q, k, v, o, vs_heads, vs_idx, bs_heads, bs_idx, scale=0.0, stream=None):
    x = _qkv(q, k, v, o, scale)
    hv, nv = _heads(vs_heads)
    hb, nb = _heads(bs_heads)
    sv, sb = vs_idx.c_struct(), bs_idx.c_struct()
    _check(lib().minf_vs_bs_attn(ctypes.byref(x), hv, nv, ctypes.byref(sv), hb, nb, ctypes.byref(sb), _stream(stream)))
