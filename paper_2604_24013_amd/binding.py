"""ctypes binding of ``libcommfuse.so`` -- argument marshalling only.

Every function here has the name of the C entry point it calls (minus the
``commfuse_`` prefix) and does nothing but turn torch tensors / Python numbers
into pointers and sizes.  There is no fallback: if the library has not been
built, loading raises.  PyTorch supplies device memory and streams only.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcommfuse.so")

CF_OK = 0
CF_ERR_INVALID_ARG, CF_ERR_NULL_PTR, CF_ERR_UNSUPPORTED, CF_ERR_MISALIGNED, CF_ERR_HIP = -1, -2, -3, -4, -5
CF_BF16, CF_F32 = 0, 1
CF_KIND_RS, CF_KIND_AG, CF_KIND_DP, CF_KIND_RS_PAIR, CF_KIND_DP_PAIR, CF_KIND_WGRAD_X, CF_KIND_WGRAD_G = 0, 1, 2, 3, 4, 5, 6
CF_W_KN, CF_W_NK = 0, 1
CF_NO_COPY, CF_NO_COMPUTE, CF_SERIAL, CF_POISON, CF_GRAPH, CF_FUSED_COPY, CF_DEVICE_WAIT = 1, 2, 4, 8, 16, 32, 64
CF_PERSISTENT = 128

KINDS = {"rs": CF_KIND_RS, "ag": CF_KIND_AG, "dp": CF_KIND_DP, "rs_pair": CF_KIND_RS_PAIR, "dp_pair": CF_KIND_DP_PAIR,
         "wgrad_x": CF_KIND_WGRAD_X, "wgrad_g": CF_KIND_WGRAD_G}
DTYPES = {"bf16": CF_BF16, "f32": CF_F32}

EXPORTS = [
    "commfuse_chunk_index", "commfuse_subslice_index", "commfuse_pair_partner", "commfuse_rs_pair_step", "commfuse_rs_pair_last_step", "commfuse_dp_pair_step", "commfuse_wgrad_step", "commfuse_attn_slice", "commfuse_attn_rs_step",
    "commfuse_run_attn_schedule", "commfuse_rs_step", "commfuse_rs_step_noalloc", "commfuse_ag_step", "commfuse_dp_reduce_step",
    "commfuse_run_schedule", "commfuse_last_error", "commfuse_workspace_bytes", "commfuse_set_workspace",
    "commfuse_device_status",
    "commfuse_destroy_cache", "commfuse_version",
]


class LayerDesc(ctypes.Structure):
    _fields_ = [
        ("p", ctypes.c_int32), ("rank", ctypes.c_int32),
        ("m_chunk", ctypes.c_int64), ("n", ctypes.c_int64), ("k", ctypes.c_int64),
        ("lda", ctypes.c_int64), ("ldw", ctypes.c_int64), ("ldo", ctypes.c_int64),
        ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("w_layout", ctypes.c_int32), ("m", ctypes.c_int32),
    ]


class Buffers(ctypes.Structure):
    _fields_ = [
        ("A_or_own_shard", ctypes.c_void_p), ("W", ctypes.c_void_p), ("O", ctypes.c_void_p),
        ("peer_stage", ctypes.POINTER(ctypes.c_void_p)),
        ("slot", ctypes.c_void_p * 2), ("send_slot", ctypes.c_void_p * 2),
        ("peer_sink", ctypes.POINTER(ctypes.c_void_p)),
        ("recv_each", ctypes.POINTER(ctypes.c_void_p)),
        ("send_each", ctypes.POINTER(ctypes.c_void_p)),
    ]


class AttnDesc(ctypes.Structure):
    _fields_ = [
        ("p", ctypes.c_int32), ("rank", ctypes.c_int32),
        ("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("seq", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("n", ctypes.c_int64), ("ldw", ctypes.c_int64), ("ldo", ctypes.c_int64),
        ("w_layout", ctypes.c_int32), ("scale", ctypes.c_float),
    ]


class AttnBuffers(ctypes.Structure):
    _fields_ = [
        ("Q", ctypes.c_void_p), ("K", ctypes.c_void_p), ("V", ctypes.c_void_p), ("Wo", ctypes.c_void_p),
        ("attn_out", ctypes.c_void_p), ("O", ctypes.c_void_p),
        ("peer_stage", ctypes.POINTER(ctypes.c_void_p)),
        ("slot", ctypes.c_void_p * 2), ("send_slot", ctypes.c_void_p * 2),
        ("peer_sink", ctypes.POINTER(ctypes.c_void_p)),
        ("recv_each", ctypes.POINTER(ctypes.c_void_p)),
        ("send_each", ctypes.POINTER(ctypes.c_void_p)),
    ]


class CommFuseError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"commfuse status {status}: {text}")
        self.status = status


_lib = None


def load():
    """Loads the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2604_24013_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.commfuse_chunk_index.argtypes = [i32, i32, i32, i32]
    lib.commfuse_chunk_index.restype = i32
    lib.commfuse_rs_step.argtypes = [ctypes.POINTER(LayerDesc), i32, vp, vp, vp, vp, vp]
    lib.commfuse_rs_step.restype = i32
    lib.commfuse_rs_step_noalloc.argtypes = [ctypes.POINTER(LayerDesc), i32, vp, vp, vp, vp, vp]
    lib.commfuse_rs_step_noalloc.restype = i32
    lib.commfuse_ag_step.argtypes = [ctypes.POINTER(LayerDesc), i32, vp, vp, vp, vp]
    lib.commfuse_ag_step.restype = i32
    lib.commfuse_dp_reduce_step.argtypes = [i32, i32, i32, vp, i64, vp, vp]
    lib.commfuse_dp_reduce_step.restype = i32
    lib.commfuse_subslice_index.argtypes = [i32, i32, i32, i32, i32]
    lib.commfuse_subslice_index.restype = i32
    lib.commfuse_pair_partner.argtypes = [i32, i32, i32]
    lib.commfuse_pair_partner.restype = i32
    lib.commfuse_rs_pair_step.argtypes = [ctypes.POINTER(LayerDesc), i32, vp, vp, vp, vp, vp, vp]
    lib.commfuse_rs_pair_step.restype = i32
    lib.commfuse_rs_pair_last_step.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, ctypes.POINTER(ctypes.c_void_p), vp, vp]
    lib.commfuse_rs_pair_last_step.restype = i32
    lib.commfuse_wgrad_step.argtypes = [ctypes.POINTER(LayerDesc), i32, vp, vp, vp, vp]
    lib.commfuse_wgrad_step.restype = i32
    lib.commfuse_attn_slice.argtypes = [ctypes.POINTER(AttnDesc), i32, vp, vp, vp, vp, vp]
    lib.commfuse_attn_slice.restype = i32
    lib.commfuse_attn_rs_step.argtypes = [ctypes.POINTER(AttnDesc), i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.commfuse_attn_rs_step.restype = i32
    lib.commfuse_run_attn_schedule.argtypes = [ctypes.POINTER(AttnDesc), ctypes.POINTER(AttnBuffers), vp, vp, ctypes.c_uint32]
    lib.commfuse_run_attn_schedule.restype = i32
    lib.commfuse_dp_pair_step.argtypes = [i32, i32, i32, vp, i64, vp, vp]
    lib.commfuse_dp_pair_step.restype = i32
    lib.commfuse_run_schedule.argtypes = [ctypes.POINTER(LayerDesc), i32, ctypes.POINTER(Buffers), vp, vp, ctypes.c_uint32]
    lib.commfuse_run_schedule.restype = i32
    lib.commfuse_last_error.argtypes = []
    lib.commfuse_last_error.restype = ctypes.c_char_p
    lib.commfuse_workspace_bytes.argtypes = [ctypes.POINTER(LayerDesc), i32]
    lib.commfuse_workspace_bytes.restype = ctypes.c_size_t
    lib.commfuse_set_workspace.argtypes = [vp, ctypes.c_size_t, vp]
    lib.commfuse_set_workspace.restype = i32
    lib.commfuse_device_status.argtypes = [vp]
    lib.commfuse_device_status.restype = i32
    lib.commfuse_destroy_cache.argtypes = []
    lib.commfuse_destroy_cache.restype = None
    lib.commfuse_version.argtypes = []
    lib.commfuse_version.restype = i32
    _lib = lib
    return lib


def last_error() -> str:
    return load().commfuse_last_error().decode()


def _check(status: int) -> None:
    if status != CF_OK:
        raise CommFuseError(status, last_error())


def _ptr(t) -> Optional[int]:
    """Device (or raw) pointer of a torch tensor, an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, int):
        return s or None
    return s.cuda_stream or None


def layer_desc(p: int, rank: int, m_chunk: int, n: int, k: int, in_dtype="bf16", out_dtype="f32",
               w_layout: int = CF_W_KN, lda: int = 0, ldw: int = 0, ldo: int = 0, m: int = 0) -> LayerDesc:
    d = LayerDesc()
    d.p, d.rank, d.m_chunk, d.n, d.k = p, rank, m_chunk, n, k
    d.lda, d.ldw, d.ldo = lda, ldw, ldo
    d.in_dtype = DTYPES[in_dtype] if isinstance(in_dtype, str) else in_dtype
    d.out_dtype = DTYPES[out_dtype] if isinstance(out_dtype, str) else out_dtype
    d.w_layout = w_layout
    d.m = m
    return d


def version() -> int:
    return load().commfuse_version()


def chunk_index(kind: int, p: int, rank: int, step: int) -> int:
    v = load().commfuse_chunk_index(kind, p, rank, step)
    if v < 0:
        raise CommFuseError(v, last_error())
    return v


def subslice_index(kind: int, p: int, m: int, rank: int, step: int) -> int:
    v = load().commfuse_subslice_index(kind, p, m, rank, step)
    if v < 0:
        raise CommFuseError(v, last_error())
    return v


def pair_partner(p: int, rank: int, round_: int) -> int:
    v = load().commfuse_pair_partner(p, rank, round_)
    if v < 0:
        raise CommFuseError(v, last_error())
    return v


def rs_pair_step(desc: LayerDesc, step: int, A, W, recv, acc, out, stream=None) -> None:
    _check(load().commfuse_rs_pair_step(ctypes.byref(desc), step, _ptr(A), _ptr(W), _ptr(recv), _ptr(acc), _ptr(out),
                                        _stream(stream)))


def rs_pair_last_step(desc: LayerDesc, A, W, recv_each: Sequence, out, stream=None) -> None:
    n = len(recv_each)
    table = (ctypes.c_void_p * max(n, 1))(*[_ptr(t) for t in recv_each])
    arg = ctypes.cast(table, ctypes.POINTER(ctypes.c_void_p)) if n else None
    _check(load().commfuse_rs_pair_last_step(ctypes.byref(desc), _ptr(A), _ptr(W), arg, _ptr(out), _stream(stream)))


def wgrad_step(desc: LayerDesc, step: int, left, right, dW, stream=None) -> None:
    _check(load().commfuse_wgrad_step(ctypes.byref(desc), step, _ptr(left), _ptr(right), _ptr(dW), _stream(stream)))


def attn_desc(p: int, rank: int, batch: int, heads: int, seq: int, head_dim: int, n: int, scale: float,
              w_layout: int = CF_W_KN, ldw: int = 0, ldo: int = 0) -> AttnDesc:
    d = AttnDesc()
    d.p, d.rank, d.batch, d.heads, d.seq, d.head_dim = p, rank, batch, heads, seq, head_dim
    d.n, d.ldw, d.ldo, d.w_layout, d.scale = n, ldw, ldo, w_layout, scale
    return d


def attn_slice(desc: AttnDesc, slice_: int, Q, K, V, attn_out, stream=None) -> None:
    _check(load().commfuse_attn_slice(ctypes.byref(desc), slice_, _ptr(Q), _ptr(K), _ptr(V), _ptr(attn_out), _stream(stream)))


def attn_rs_step(desc: AttnDesc, step: int, Q, K, V, Wo, recv, out, attn_out, stream=None) -> None:
    _check(load().commfuse_attn_rs_step(ctypes.byref(desc), step, _ptr(Q), _ptr(K), _ptr(V), _ptr(Wo), _ptr(recv),
                                        _ptr(out), _ptr(attn_out), _stream(stream)))


def _table(seq_):
    if seq_ is None or not len(seq_):
        return None, None
    t = (ctypes.c_void_p * len(seq_))(*[_ptr(x) for x in seq_])
    return ctypes.cast(t, ctypes.POINTER(ctypes.c_void_p)), t


def make_attn_buffers(Q, K, V, Wo, attn_out, O, peer_stage, slot, send_slot, peer_sink=None, recv_each=None,
                      send_each=None) -> AttnBuffers:
    b = AttnBuffers()
    b.Q, b.K, b.V, b.Wo, b.attn_out, b.O = _ptr(Q), _ptr(K), _ptr(V), _ptr(Wo), _ptr(attn_out), _ptr(O)
    b.peer_stage, b._k0 = _table(peer_stage)
    b.slot[0], b.slot[1] = _ptr(slot[0]), _ptr(slot[1])
    b.send_slot[0], b.send_slot[1] = _ptr(send_slot[0]), _ptr(send_slot[1])
    b.peer_sink, b._k1 = _table(peer_sink)
    b.recv_each, b._k2 = _table(recv_each)
    b.send_each, b._k3 = _table(send_each)
    return b


def run_attn_schedule(desc: AttnDesc, bufs: AttnBuffers, compute_stream, copy_stream, flags: int = 0) -> None:
    _check(load().commfuse_run_attn_schedule(ctypes.byref(desc), ctypes.byref(bufs), _stream(compute_stream),
                                             _stream(copy_stream), flags))


def dp_pair_step(p: int, rank: int, step: int, bucket, chunk_elems: int, recv, stream=None) -> None:
    _check(load().commfuse_dp_pair_step(p, rank, step, _ptr(bucket), chunk_elems, _ptr(recv), _stream(stream)))


def rs_step(desc: LayerDesc, step: int, A, W, recv, out, stream=None) -> None:
    _check(load().commfuse_rs_step(ctypes.byref(desc), step, _ptr(A), _ptr(W), _ptr(recv), _ptr(out), _stream(stream)))


def rs_step_noalloc(desc: LayerDesc, step: int, A, W, recv, out, stream=None) -> None:
    _check(load().commfuse_rs_step_noalloc(ctypes.byref(desc), step, _ptr(A), _ptr(W), _ptr(recv), _ptr(out),
                                           _stream(stream)))


def ag_step(desc: LayerDesc, step: int, shard, W, O, stream=None) -> None:
    _check(load().commfuse_ag_step(ctypes.byref(desc), step, _ptr(shard), _ptr(W), _ptr(O), _stream(stream)))


def dp_reduce_step(p: int, rank: int, step: int, bucket, chunk_elems: int, recv, stream=None) -> None:
    _check(load().commfuse_dp_reduce_step(p, rank, step, _ptr(bucket), chunk_elems, _ptr(recv), _stream(stream)))


def make_buffers(A_or_own_shard, W, O, peer_stage: Sequence, slot: Sequence, send_slot: Sequence = (None, None),
                 peer_sink: Optional[Sequence] = None, recv_each: Optional[Sequence] = None,
                 send_each: Optional[Sequence] = None) -> Buffers:
    """Fills a ``cf_buffers``.  The returned object keeps the pointer tables alive;
    the caller keeps the tensors alive."""
    b = Buffers()
    b.A_or_own_shard, b.W, b.O = _ptr(A_or_own_shard), _ptr(W), _ptr(O)
    n = len(peer_stage)
    stage = (ctypes.c_void_p * max(n, 1))(*[_ptr(t) for t in peer_stage])
    b.peer_stage = ctypes.cast(stage, ctypes.POINTER(ctypes.c_void_p)) if n else None
    b._stage_keepalive = stage
    b.slot[0], b.slot[1] = _ptr(slot[0]), _ptr(slot[1])
    b.send_slot[0], b.send_slot[1] = _ptr(send_slot[0]), _ptr(send_slot[1])
    if peer_sink is not None and len(peer_sink):
        sink = (ctypes.c_void_p * len(peer_sink))(*[_ptr(t) for t in peer_sink])
        b.peer_sink = ctypes.cast(sink, ctypes.POINTER(ctypes.c_void_p))
        b._sink_keepalive = sink
    else:
        b.peer_sink = None
    if recv_each is not None and len(recv_each):
        each = (ctypes.c_void_p * len(recv_each))(*[_ptr(t) for t in recv_each])
        b.recv_each = ctypes.cast(each, ctypes.POINTER(ctypes.c_void_p))
        b._each_keepalive = each
    else:
        b.recv_each = None
    b.send_each, b._send_each_keepalive = _table(send_each)
    return b


def run_schedule(desc: LayerDesc, kind: int, bufs: Buffers, compute_stream, copy_stream, flags: int = 0) -> None:
    _check(load().commfuse_run_schedule(ctypes.byref(desc), kind, ctypes.byref(bufs), _stream(compute_stream),
                                        _stream(copy_stream), flags))


def workspace_bytes(desc: LayerDesc, kind: int) -> int:
    return int(load().commfuse_workspace_bytes(ctypes.byref(desc), kind))


def set_workspace(buf, nbytes: int = 0, stream=None) -> None:
    """Registers (or, with ``None``, clears) the split-K workspace; ``buf`` is a device tensor or pointer."""
    if buf is not None and not isinstance(buf, int) and nbytes == 0:
        nbytes = buf.numel() * buf.element_size()
    _check(load().commfuse_set_workspace(_ptr(buf), nbytes, _stream(stream)))


def device_status(stream=None) -> None:
    """Synchronises ``stream``; raises if a kernel gave up a bounded device-side wait (CF_DEVICE_WAIT, or the
    pairwise reduce-scatter carrying its deliveries)."""
    _check(load().commfuse_device_status(_stream(stream)))


def destroy_cache() -> None:
    load().commfuse_destroy_cache()
