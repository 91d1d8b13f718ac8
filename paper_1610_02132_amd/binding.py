"""ctypes binding of libqsgd.so: same names as the C ABI (include/qsgd.h),
argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

CODE_SPARSE, CODE_DENSE, CODE_FIXED = 0, 1, 2
NORM_L2, NORM_MAX = 0, 1
QSGD_MAX_PEERS = 64

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = os.path.join(_HERE, "libqsgd.so")

EXPORTS = [
    "qsgd_version", "qsgd_strerror", "qsgd_max_encoded_bytes", "qsgd_workspace_bytes",
    "qsgd_encode", "qsgd_decode_accumulate", "qsgd_sgd_step", "qsgd_message_info",
    "qsgd_message_status", "qsgd_workspace_status", "qsgd_timing_enable",
    "qsgd_timing_reset", "qsgd_timing_get", "qsgd_copy_probe",
    "qsgd_layout_create", "qsgd_layout_destroy", "qsgd_layout_info",
    "qsgd_layout_max_encoded_bytes", "qsgd_layout_workspace_bytes", "qsgd_encode_layout",
    "qsgd_decode_accumulate_layout", "qsgd_sgd_step_layout", "qsgd_encode_slice",
    "qsgd_pipeline_create", "qsgd_pipeline_destroy", "qsgd_pipeline_step",
    "qsgd_copy_probe_words", "qsgd_encode_workspace_bytes",
    "qsgd_encode_static", "qsgd_static_scratch_bytes",
]


class QsgdError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {qsgd_strerror(code)} ({code})")
        self.code = code


class _Params(C.Structure):
    _fields_ = [("n", C.c_uint64), ("d", C.c_uint64), ("seed", C.c_uint64),
                ("s", C.c_uint32), ("code", C.c_uint32), ("norm", C.c_uint32),
                ("stream_id", C.c_uint32), ("iteration", C.c_uint32),
                ("reserved", C.c_uint32)]


@dataclass
class Params:
    """Mirror of struct qsgd_params."""
    n: int
    s: int
    d: int
    code: int = CODE_SPARSE
    norm: int = NORM_L2
    seed: int = 0
    stream_id: int = 0
    iteration: int = 0

    def c(self) -> _Params:
        return _Params(self.n, self.d, self.seed, self.s, self.code, self.norm,
                       self.stream_id, self.iteration, 0)


_lib = None


def lib_path() -> str:
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        raise ImportError(
            f"{_LIB} is missing: build it with `python -m paper_1610_02132_amd.build` "
            "(there is no CPU fallback)")
    L = C.CDLL(_LIB)
    vp, sz, PP = C.c_void_p, C.c_size_t, C.POINTER(_Params)
    L.qsgd_version.restype = C.c_int
    L.qsgd_strerror.argtypes = [C.c_int]
    L.qsgd_strerror.restype = C.c_char_p
    L.qsgd_max_encoded_bytes.argtypes = [PP]
    L.qsgd_max_encoded_bytes.restype = sz
    L.qsgd_workspace_bytes.argtypes = [PP, C.c_uint32]
    L.qsgd_workspace_bytes.restype = sz
    L.qsgd_encode.argtypes = [PP, vp, vp, sz, vp, sz, vp]
    L.qsgd_encode.restype = C.c_int
    L.qsgd_decode_accumulate.argtypes = [PP, vp, vp, C.c_uint32, vp, vp, sz, vp]
    L.qsgd_decode_accumulate.restype = C.c_int
    L.qsgd_sgd_step.argtypes = [PP, vp, vp, C.c_uint32, C.c_float, vp, vp, sz, vp]
    L.qsgd_sgd_step.restype = C.c_int
    L.qsgd_message_info.argtypes = [vp, PP, C.POINTER(C.c_uint64)]
    L.qsgd_message_info.restype = C.c_int
    L.qsgd_message_status.argtypes = [vp, C.POINTER(C.c_uint64), vp]
    L.qsgd_message_status.restype = C.c_int
    L.qsgd_workspace_status.argtypes = [vp, vp]
    L.qsgd_workspace_status.restype = C.c_int
    L.qsgd_timing_enable.argtypes = [C.c_int]
    L.qsgd_timing_enable.restype = C.c_int
    L.qsgd_timing_reset.restype = C.c_int
    L.qsgd_timing_get.argtypes = [C.c_char_p, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    L.qsgd_timing_get.restype = C.c_int
    L.qsgd_copy_probe.argtypes = [vp, vp, sz, vp]
    L.qsgd_copy_probe.restype = C.c_int
    L.qsgd_copy_probe_words.argtypes = [vp, vp, sz, vp]
    L.qsgd_copy_probe_words.restype = C.c_int
    L.qsgd_encode_workspace_bytes.argtypes = [PP, sz]
    L.qsgd_encode_workspace_bytes.restype = sz
    L.qsgd_encode_static.argtypes = [PP, vp, vp, sz, vp]
    L.qsgd_encode_static.restype = C.c_int
    L.qsgd_static_scratch_bytes.restype = sz
    u64p = C.POINTER(C.c_uint64)
    L.qsgd_layout_create.argtypes = [u64p, u64p, C.c_uint32, C.c_uint64, C.c_uint64,
                                     C.POINTER(vp)]
    L.qsgd_layout_create.restype = C.c_int
    L.qsgd_layout_destroy.argtypes = [vp]
    L.qsgd_layout_destroy.restype = None
    L.qsgd_layout_info.argtypes = [vp, u64p, u64p, u64p]
    L.qsgd_layout_info.restype = C.c_int
    L.qsgd_layout_max_encoded_bytes.argtypes = [PP, vp]
    L.qsgd_layout_max_encoded_bytes.restype = sz
    L.qsgd_layout_workspace_bytes.argtypes = [PP, vp, C.c_uint32]
    L.qsgd_layout_workspace_bytes.restype = sz
    L.qsgd_encode_layout.argtypes = [PP, vp, vp, vp, sz, vp, sz, vp]
    L.qsgd_encode_layout.restype = C.c_int
    L.qsgd_decode_accumulate_layout.argtypes = [PP, vp, vp, vp, C.c_uint32, vp, vp, sz, vp]
    L.qsgd_decode_accumulate_layout.restype = C.c_int
    L.qsgd_sgd_step_layout.argtypes = [PP, vp, vp, vp, C.c_uint32, C.c_float, vp, vp, sz, vp]
    L.qsgd_sgd_step_layout.restype = C.c_int
    L.qsgd_encode_slice.argtypes = [PP, C.c_uint64, vp, vp, sz, vp, sz, vp]
    L.qsgd_encode_slice.restype = C.c_int
    L.qsgd_pipeline_create.argtypes = [C.POINTER(vp)]
    L.qsgd_pipeline_create.restype = C.c_int
    L.qsgd_pipeline_destroy.argtypes = [vp]
    L.qsgd_pipeline_destroy.restype = None
    L.qsgd_pipeline_step.argtypes = [vp, PP, C.c_uint64, vp, C.c_uint32, C.c_float, vp, vp, sz,
                                     vp, vp, sz, vp]
    L.qsgd_pipeline_step.restype = C.c_int
    _lib = L
    return L


def _stream(stream):
    """A torch.cuda.Stream, a raw handle (int) or None (torch's current stream)."""
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def _dev(t, what: str):
    if t is None:
        return C.c_void_p(0), 0
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous device tensor")
    return C.c_void_p(t.data_ptr()), t.numel() * t.element_size()


def qsgd_version() -> int:
    return int(_load().qsgd_version())


def qsgd_strerror(err: int) -> str:
    return _load().qsgd_strerror(err).decode()


def qsgd_max_encoded_bytes(p: Params) -> int:
    cp = p.c()
    return int(_load().qsgd_max_encoded_bytes(C.byref(cp)))


def qsgd_workspace_bytes(p: Params, K: int) -> int:
    cp = p.c()
    return int(_load().qsgd_workspace_bytes(C.byref(cp), K))


def qsgd_encode(p: Params, g, msg, workspace, stream=None) -> None:
    """Queues Encode(g) -> msg (device byte/word tensor) on the stream."""
    if g.dtype.itemsize != 4 or not g.dtype.is_floating_point:
        raise ValueError("g must be float32")
    if g.numel() != p.n:
        raise ValueError("g has the wrong length")
    gp, _ = _dev(g, "g")
    mp, mbytes = _dev(msg, "msg")
    wp, wbytes = _dev(workspace, "workspace")
    cp = p.c()
    rc = _load().qsgd_encode(C.byref(cp), gp, mp, mbytes, wp, wbytes, _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_encode")


def _msgs(msgs, msg_bytes):
    K = len(msgs)
    ptrs = (C.c_void_p * K)()
    sizes = (C.c_size_t * K)()
    for k, m in enumerate(msgs):
        p, nbytes = _dev(m, "message")
        ptrs[k] = p.value
        sizes[k] = nbytes if msg_bytes is None else min(nbytes, int(msg_bytes[k]))
    return ptrs, sizes, K


def qsgd_decode_accumulate(p: Params, msgs, acc, workspace, msg_bytes=None, stream=None) -> None:
    """Queues acc += sum_k Decode(msgs[k])."""
    if acc.numel() != p.n or acc.dtype.itemsize != 4:
        raise ValueError("acc must hold n float32")
    ptrs, sizes, K = _msgs(msgs, msg_bytes)
    ap, _ = _dev(acc, "acc")
    wp, wbytes = _dev(workspace, "workspace")
    cp = p.c()
    rc = _load().qsgd_decode_accumulate(C.byref(cp), ptrs, sizes, K, ap, wp, wbytes,
                                        _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_decode_accumulate")


def qsgd_sgd_step(p: Params, msgs, eta: float, x, workspace, msg_bytes=None, stream=None) -> None:
    """Queues x -= (eta/K) * sum_k Decode(msgs[k])."""
    if x.numel() != p.n or x.dtype.itemsize != 4:
        raise ValueError("x must hold n float32")
    ptrs, sizes, K = _msgs(msgs, msg_bytes)
    xp, _ = _dev(x, "x")
    wp, wbytes = _dev(workspace, "workspace")
    cp = p.c()
    rc = _load().qsgd_sgd_step(C.byref(cp), ptrs, sizes, K, C.c_float(eta), xp, wp, wbytes,
                               _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_sgd_step")


def qsgd_message_info(header_host: bytes):
    """(status, Params, total_bytes) from a host copy of the first 64 bytes of a message."""
    buf = C.create_string_buffer(bytes(header_host[:64]), 64)
    cp = _Params()
    total = C.c_uint64(0)
    rc = _load().qsgd_message_info(buf, C.byref(cp), C.byref(total))
    p = Params(n=cp.n, s=cp.s, d=cp.d, code=cp.code, norm=cp.norm, seed=0,
               stream_id=cp.stream_id, iteration=cp.iteration)
    return int(rc), p, int(total.value)


def qsgd_message_status(msg, stream=None):
    """Waits for the stream; returns (status, total_bytes) of a device message."""
    mp, _ = _dev(msg, "msg")
    total = C.c_uint64(0)
    rc = _load().qsgd_message_status(mp, C.byref(total), _stream(stream))
    return int(rc), int(total.value)


def qsgd_workspace_status(workspace, stream=None) -> int:
    wp, _ = _dev(workspace, "workspace")
    return int(_load().qsgd_workspace_status(wp, _stream(stream)))


def qsgd_timing_enable(on: bool) -> None:
    _load().qsgd_timing_enable(1 if on else 0)


def qsgd_timing_reset() -> None:
    _load().qsgd_timing_reset()


def qsgd_timing_get(prefix: str):
    """(total milliseconds, launches) of the kernels whose name starts with prefix."""
    ms = C.c_double(0.0)
    cnt = C.c_uint64(0)
    rc = _load().qsgd_timing_get(prefix.encode(), C.byref(ms), C.byref(cnt))
    if rc:
        raise QsgdError(rc, "qsgd_timing_get")
    return float(ms.value), int(cnt.value)


def qsgd_copy_probe(dst, src, stream=None) -> None:
    """Plain device copy of src into dst (same byte size, a multiple of 16)."""
    dp, db = _dev(dst, "dst")
    sp, sb = _dev(src, "src")
    if db != sb:
        raise ValueError("dst and src differ in size")
    rc = _load().qsgd_copy_probe(dp, sp, sb, _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_copy_probe")


def qsgd_copy_probe_words(dst, src, stream=None) -> None:
    """The same copy with one 4-byte load and store per lane."""
    dp, db = _dev(dst, "dst")
    sp, sb = _dev(src, "src")
    if db != sb:
        raise ValueError("dst and src differ in size")
    rc = _load().qsgd_copy_probe_words(dp, sp, sb, _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_copy_probe_words")


def qsgd_encode_static(p: Params, g, msg, stream=None) -> None:
    """qsgd_encode with the library's built-in scratch instead of a workspace."""
    if g.dtype.itemsize != 4 or not g.dtype.is_floating_point or g.numel() != p.n:
        raise ValueError("g must hold n float32")
    gp, _ = _dev(g, "g")
    mp, mbytes = _dev(msg, "msg")
    cp = p.c()
    rc = _load().qsgd_encode_static(C.byref(cp), gp, mp, mbytes, _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_encode_static")


def qsgd_static_scratch_bytes() -> int:
    return int(_load().qsgd_static_scratch_bytes())


def qsgd_encode_workspace_bytes(p: Params, msg_capacity: int) -> int:
    cp = p.c()
    return int(_load().qsgd_encode_workspace_bytes(C.byref(cp), msg_capacity))


class Layout:
    """Handle of a qsgd_layout: tensors = [(offset, size), ...] in elements of the arena."""

    def __init__(self, tensors, d: int, bypass_below: int):
        T = len(tensors)
        offs = (C.c_uint64 * max(T, 1))(*[int(t[0]) for t in tensors])
        sizes = (C.c_uint64 * max(T, 1))(*[int(t[1]) for t in tensors])
        h = C.c_void_p(0)
        rc = _load().qsgd_layout_create(offs, sizes, T, d, bypass_below, C.byref(h))
        if rc:
            raise QsgdError(rc, "qsgd_layout_create")
        self.handle = h
        self.d = d
        self.bypass_below = bypass_below
        self.tensors = [(int(t[0]), int(t[1])) for t in tensors]

    def close(self) -> None:
        if self.handle:
            _load().qsgd_layout_destroy(self.handle)
            self.handle = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def qsgd_layout_info(layout: Layout):
    """(buckets, raw values, extent of the arena the tensors use)."""
    nb, raw, ext = C.c_uint64(0), C.c_uint64(0), C.c_uint64(0)
    rc = _load().qsgd_layout_info(layout.handle, C.byref(nb), C.byref(raw), C.byref(ext))
    if rc:
        raise QsgdError(rc, "qsgd_layout_info")
    return int(nb.value), int(raw.value), int(ext.value)


def qsgd_layout_max_encoded_bytes(p: Params, layout: Layout) -> int:
    cp = p.c()
    return int(_load().qsgd_layout_max_encoded_bytes(C.byref(cp), layout.handle))


def qsgd_layout_workspace_bytes(p: Params, layout: Layout, K: int) -> int:
    cp = p.c()
    return int(_load().qsgd_layout_workspace_bytes(C.byref(cp), layout.handle, K))


def qsgd_encode_layout(p: Params, layout: Layout, g, msg, workspace, stream=None) -> None:
    """Queues the tensor-aware Encode of the arena g -> msg."""
    if g.dtype.itemsize != 4 or not g.dtype.is_floating_point or g.numel() != p.n:
        raise ValueError("g must hold n float32")
    gp, _ = _dev(g, "g")
    mp, mbytes = _dev(msg, "msg")
    wp, wbytes = _dev(workspace, "workspace")
    cp = p.c()
    rc = _load().qsgd_encode_layout(C.byref(cp), layout.handle, gp, mp, mbytes, wp, wbytes,
                                    _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_encode_layout")


def qsgd_decode_accumulate_layout(p: Params, layout: Layout, msgs, acc, workspace, msg_bytes=None,
                                  stream=None) -> None:
    if acc.numel() != p.n or acc.dtype.itemsize != 4:
        raise ValueError("acc must hold n float32")
    ptrs, sizes, K = _msgs(msgs, msg_bytes)
    ap, _ = _dev(acc, "acc")
    wp, wbytes = _dev(workspace, "workspace")
    cp = p.c()
    rc = _load().qsgd_decode_accumulate_layout(C.byref(cp), layout.handle, ptrs, sizes, K, ap, wp,
                                               wbytes, _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_decode_accumulate_layout")


def qsgd_sgd_step_layout(p: Params, layout: Layout, msgs, eta: float, x, workspace, msg_bytes=None,
                         stream=None) -> None:
    if x.numel() != p.n or x.dtype.itemsize != 4:
        raise ValueError("x must hold n float32")
    ptrs, sizes, K = _msgs(msgs, msg_bytes)
    xp, _ = _dev(x, "x")
    wp, wbytes = _dev(workspace, "workspace")
    cp = p.c()
    rc = _load().qsgd_sgd_step_layout(C.byref(cp), layout.handle, ptrs, sizes, K, C.c_float(eta),
                                      xp, wp, wbytes, _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_sgd_step_layout")


def qsgd_encode_slice(p: Params, index_base: int, g, msg, workspace, stream=None) -> None:
    """Encode of the p.n values in g with the draws of positions index_base.. of a longer vector."""
    if g.dtype.itemsize != 4 or not g.dtype.is_floating_point or g.numel() != p.n:
        raise ValueError("g must hold n float32")
    gp, _ = _dev(g, "g")
    mp, mbytes = _dev(msg, "msg")
    wp, wbytes = _dev(workspace, "workspace")
    cp = p.c()
    rc = _load().qsgd_encode_slice(C.byref(cp), index_base, gp, mp, mbytes, wp, wbytes,
                                   _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_encode_slice")


class Pipeline:
    """Handle of a qsgd_pipeline (two internal streams and their events)."""

    def __init__(self):
        h = C.c_void_p(0)
        rc = _load().qsgd_pipeline_create(C.byref(h))
        if rc:
            raise QsgdError(rc, "qsgd_pipeline_create")
        self.handle = h

    def close(self) -> None:
        if self.handle:
            _load().qsgd_pipeline_destroy(self.handle)
            self.handle = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def qsgd_pipeline_step(pipe: Pipeline, p: Params, chunk_elems: int, grads, eta: float, x, msgs,
                       enc_workspace, dec_workspace, stream=None) -> None:
    """Queues the double-buffered pass: grads = K device gradients of n values, msgs = 2*K
    message buffers of equal size (two sets used alternately)."""
    K = len(grads)
    if len(msgs) != 2 * K:
        raise ValueError("msgs must hold 2*K buffers")
    if x.numel() != p.n or any(g.numel() != p.n for g in grads):
        raise ValueError("x and the gradients must hold n float32")
    gptr = (C.c_void_p * K)(*[_dev(g, "g")[0].value for g in grads])
    mptr = (C.c_void_p * (2 * K))()
    cap = None
    for i, m in enumerate(msgs):
        mp, nbytes = _dev(m, "message")
        mptr[i] = mp.value
        cap = nbytes if cap is None else min(cap, nbytes)
    xp, _ = _dev(x, "x")
    ep, ebytes = _dev(enc_workspace, "enc_workspace")
    dp, dbytes = _dev(dec_workspace, "dec_workspace")
    cp = p.c()
    rc = _load().qsgd_pipeline_step(pipe.handle, C.byref(cp), chunk_elems, gptr, K, C.c_float(eta),
                                    xp, mptr, cap, ep, dp, min(ebytes, dbytes), _stream(stream))
    if rc:
        raise QsgdError(rc, "qsgd_pipeline_step")
