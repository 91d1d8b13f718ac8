"""ctypes front end of the QSGD CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this.
It loads ``libqsgd_oracle.so`` built from ``qsgd_oracle.c`` (plain C, gcc) and
exposes its functions on numpy arrays.  Nothing here computes: every step of
the method is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libqsgd_oracle.so")
_SRC = [os.path.join(_HERE, f) for f in ("qsgd_oracle.c", "qsgd_oracle.h")]

CODE_SPARSE, CODE_DENSE, CODE_FIXED = 0, 1, 2
NORM_L2, NORM_MAX = 0, 1
OK, ERR_INVALID_ARG, ERR_CAPACITY, ERR_CORRUPT = 0, -1, -2, -3


def build(force: bool = False) -> str:
    """Compile the oracle if the library is missing or older than its source."""
    stale = force or not os.path.exists(_SO) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRC)
    if stale:
        subprocess.check_call(["sh", os.path.join(_HERE, "build.sh")])
    return _SO


class _Params(C.Structure):
    _fields_ = [("n", C.c_uint64), ("d", C.c_uint64), ("seed", C.c_uint64),
                ("s", C.c_uint32), ("code", C.c_uint32), ("norm", C.c_uint32),
                ("stream_id", C.c_uint32), ("iteration", C.c_uint32),
                ("reserved", C.c_uint32)]


@dataclass
class Params:
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


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, u64p, sz = C.c_void_p, C.POINTER(C.c_uint64), C.c_size_t
        PP = C.POINTER(_Params)
        L.qo_philox4x32_10.argtypes = [vp, vp, vp]
        L.qo_philox4x32_10.restype = None
        L.qo_draw.argtypes = [PP, C.c_uint64]
        L.qo_draw.restype = C.c_float
        L.qo_omega_len.argtypes = [C.c_uint64]
        L.qo_omega_len.restype = C.c_uint32
        L.qo_omega_string.argtypes = [C.c_uint64, C.c_char_p, sz]
        L.qo_omega_string.restype = C.c_uint32
        L.qo_omega_decode_string.argtypes = [C.c_char_p, sz, u64p]
        L.qo_omega_decode_string.restype = C.c_uint32
        L.qo_omega_roundtrip_failures.argtypes = [C.c_uint64, C.c_uint64]
        L.qo_omega_roundtrip_failures.restype = C.c_uint64
        L.qo_bucket_size.argtypes = [PP]
        L.qo_bucket_size.restype = C.c_uint64
        L.qo_num_buckets.argtypes = [PP]
        L.qo_num_buckets.restype = C.c_uint64
        L.qo_fixed_field_bits.argtypes = [C.c_uint32]
        L.qo_fixed_field_bits.restype = C.c_uint32
        L.qo_quantize.argtypes = [PP, vp, vp, vp, vp, vp, vp, vp]
        L.qo_quantize.restype = C.c_int
        L.qo_quantize_slice.argtypes = [PP, vp, C.c_uint64, vp, vp, vp, vp, vp, vp]
        L.qo_quantize_slice.restype = C.c_int
        L.qo_max_encoded_bytes.argtypes = [PP]
        L.qo_max_encoded_bytes.restype = sz
        L.qo_encode.argtypes = [PP, vp, vp, sz, C.POINTER(sz)]
        L.qo_encode.restype = C.c_int
        L.qo_encode_with_draws.argtypes = [PP, vp, vp, vp, sz, C.POINTER(sz)]
        L.qo_encode_with_draws.restype = C.c_int
        L.qo_encode_slice.argtypes = [PP, vp, C.c_uint64, vp, sz, C.POINTER(sz)]
        L.qo_encode_slice.restype = C.c_int
        L.qo_encode_bucket.argtypes = [PP, vp, C.c_uint64, C.c_uint64, vp, sz]
        L.qo_encode_bucket.restype = C.c_int64
        L.qo_message_info.argtypes = [vp, sz, PP, u64p]
        L.qo_message_info.restype = C.c_int
        L.qo_decode_tuple.argtypes = [vp, sz, vp, vp, vp]
        L.qo_decode_tuple.restype = C.c_int
        L.qo_decode.argtypes = [vp, sz, vp]
        L.qo_decode.restype = C.c_int
        L.qo_decode_accumulate.argtypes = [vp, vp, C.c_uint32, vp]
        L.qo_decode_accumulate.restype = C.c_int
        L.qo_sgd_step.argtypes = [vp, vp, C.c_uint32, C.c_float, vp]
        L.qo_sgd_step.restype = C.c_int
        L.qo_sgd_step_buckets.argtypes = [vp, vp, C.c_uint32, C.c_float, vp, C.c_uint64, C.c_uint64]
        L.qo_sgd_step_buckets.restype = C.c_int
        L.qo_bucket_extent.argtypes = [vp, sz, C.c_uint64, u64p, u64p]
        L.qo_bucket_extent.restype = C.c_int
        L.qo_payload_offset.argtypes = [vp, sz, u64p]
        L.qo_payload_offset.restype = C.c_int
        u32 = C.c_uint32
        L.qo_layout_counts.argtypes = [PP, vp, u32, C.c_uint64, u64p, u64p]
        L.qo_layout_counts.restype = C.c_int
        L.qo_layout_max_encoded_bytes.argtypes = [PP, vp, u32, C.c_uint64]
        L.qo_layout_max_encoded_bytes.restype = sz
        L.qo_encode_layout.argtypes = [PP, vp, u32, C.c_uint64, vp, vp, sz, C.POINTER(sz)]
        L.qo_encode_layout.restype = C.c_int
        L.qo_decode_layout.argtypes = [vp, u32, C.c_uint64, vp, sz, vp]
        L.qo_decode_layout.restype = C.c_int
        L.qo_decode_accumulate_layout.argtypes = [vp, u32, C.c_uint64, vp, vp, u32, vp]
        L.qo_decode_accumulate_layout.restype = C.c_int
        L.qo_sgd_step_layout.argtypes = [vp, u32, C.c_uint64, vp, vp, u32, C.c_float, vp]
        L.qo_sgd_step_layout.restype = C.c_int
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: oracle error {code}")
        self.code = code


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise OracleError(rc, what)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().qo_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def draw(p: Params, index: int) -> float:
    cp = p.c()
    return float(lib().qo_draw(C.byref(cp), index))


def omega_len(k: int) -> int:
    return int(lib().qo_omega_len(k))


def omega_string(k: int) -> str:
    buf = C.create_string_buffer(300)
    n = lib().qo_omega_string(k, buf, 300)
    return buf.value.decode()[:n]


def omega_decode_string(bits: str):
    """Returns (value, characters consumed); consumed == 0 means malformed."""
    k = C.c_uint64(0)
    b = bits.encode()
    used = lib().qo_omega_decode_string(b, len(b), C.byref(k))
    return int(k.value), int(used)


def omega_roundtrip_failures(lo: int, hi: int) -> int:
    return int(lib().qo_omega_roundtrip_failures(lo, hi))


def bucket_size(p: Params) -> int:
    cp = p.c()
    return int(lib().qo_bucket_size(C.byref(cp)))


def num_buckets(p: Params) -> int:
    cp = p.c()
    return int(lib().qo_num_buckets(C.byref(cp)))


def fixed_field_bits(s: int) -> int:
    return int(lib().qo_fixed_field_bits(s))


def quantize(p: Params, g, u=None, want_draws: bool = False, index_offset: int = 0):
    """Q_s per bucket.  Returns dict(levels, neg, norms[, u, p]).  index_offset: position
    of g[0] in a longer vector (it selects the draws)."""
    g = _f32(g)
    assert g.size == p.n
    nb = num_buckets(p)
    levels = np.zeros(max(p.n, 1), dtype=np.uint32)
    neg = np.zeros(max(p.n, 1), dtype=np.uint8)
    norms = np.zeros(max(nb, 1), dtype=np.float32)
    u_in = None if u is None else _f32(u)
    u_out = np.zeros(max(p.n, 1), dtype=np.float32) if want_draws else None
    p_out = np.zeros(max(p.n, 1), dtype=np.float32) if want_draws else None
    cp = p.c()
    _chk(lib().qo_quantize_slice(C.byref(cp), _ptr(g), index_offset, _ptr(u_in), _ptr(levels),
                                 _ptr(neg), _ptr(norms), _ptr(u_out), _ptr(p_out)), "quantize")
    out = dict(levels=levels[:p.n], neg=neg[:p.n], norms=norms[:nb])
    if want_draws:
        out["u"] = u_out[:p.n]
        out["p"] = p_out[:p.n]
    return out


def max_encoded_bytes(p: Params) -> int:
    cp = p.c()
    return int(lib().qo_max_encoded_bytes(C.byref(cp)))


def encode(p: Params, g, u=None, capacity: int | None = None) -> np.ndarray:
    """Encode(g) -> message as a uint32 array trimmed to its used length."""
    g = _f32(g)
    assert g.size == p.n
    cap = max_encoded_bytes(p) if capacity is None else capacity
    msg = np.zeros((cap + 3) // 4, dtype=np.uint32)
    used = C.c_size_t(0)
    cp = p.c()
    if u is None:
        rc = lib().qo_encode(C.byref(cp), _ptr(g), _ptr(msg), cap, C.byref(used))
    else:
        u = _f32(u)
        rc = lib().qo_encode_with_draws(C.byref(cp), _ptr(g), _ptr(u), _ptr(msg), cap,
                                        C.byref(used))
    _chk(rc, "encode")
    return msg[: used.value // 4].copy()


def encode_slice(p: Params, g, index_offset: int) -> np.ndarray:
    """Message of a slice (p.n elements) of a longer vector, drawn at global indices."""
    g = _f32(g)
    assert g.size == p.n
    cap = max_encoded_bytes(p)
    msg = np.zeros((cap + 3) // 4, dtype=np.uint32)
    used = C.c_size_t(0)
    cp = p.c()
    _chk(lib().qo_encode_slice(C.byref(cp), _ptr(g), index_offset, _ptr(msg), cap,
                               C.byref(used)), "encode_slice")
    return msg[: used.value // 4].copy()


def encode_bucket(p: Params, v, first_index: int) -> np.ndarray:
    """The string of ONE bucket holding the elements v (global index of v[0] given)."""
    v = _f32(v)
    q = Params(n=v.size, s=p.s, d=max(v.size, 1), code=p.code, norm=p.norm)
    cap_words = max_encoded_bytes(q) // 4 + 4
    words = np.zeros(cap_words, dtype=np.uint32)
    cp = p.c()
    nw = lib().qo_encode_bucket(C.byref(cp), _ptr(v), v.size, first_index, _ptr(words),
                                cap_words)
    if nw < 0:
        raise OracleError(int(nw), "encode_bucket")
    return words[:nw].copy()


def message_info(msg: np.ndarray):
    """Returns (Params as stored in the header, total bytes)."""
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    cp = _Params()
    total = C.c_uint64(0)
    _chk(lib().qo_message_info(_ptr(msg), msg.nbytes, C.byref(cp), C.byref(total)),
         "message_info")
    return (Params(n=cp.n, s=cp.s, d=cp.d, code=cp.code, norm=cp.norm, seed=0,
                   stream_id=cp.stream_id, iteration=cp.iteration), int(total.value))


def decode_tuple(msg: np.ndarray):
    """Decode -> dict(levels, neg, norms) (the tuple of Sec. 3.1)."""
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    p, _ = message_info(msg)
    nb = num_buckets(p)
    levels = np.zeros(max(p.n, 1), dtype=np.uint32)
    neg = np.zeros(max(p.n, 1), dtype=np.uint8)
    norms = np.zeros(max(nb, 1), dtype=np.float32)
    _chk(lib().qo_decode_tuple(_ptr(msg), msg.nbytes, _ptr(levels), _ptr(neg),
                               _ptr(norms)), "decode_tuple")
    return dict(levels=levels[:p.n], neg=neg[:p.n], norms=norms[:nb])


def decode(msg: np.ndarray) -> np.ndarray:
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    p, _ = message_info(msg)
    out = np.zeros(max(p.n, 1), dtype=np.float32)
    _chk(lib().qo_decode(_ptr(msg), msg.nbytes, _ptr(out)), "decode")
    return out[:p.n]


def _msg_arrays(msgs):
    msgs = [np.ascontiguousarray(m, dtype=np.uint32) for m in msgs]
    ptrs = (C.c_void_p * len(msgs))(*[m.ctypes.data for m in msgs])
    sizes = (C.c_size_t * len(msgs))(*[m.nbytes for m in msgs])
    return msgs, ptrs, sizes


def decode_accumulate(msgs, acc) -> np.ndarray:
    keep, ptrs, sizes = _msg_arrays(msgs)
    acc = _f32(acc).copy()
    _chk(lib().qo_decode_accumulate(ptrs, sizes, len(keep), _ptr(acc)),
         "decode_accumulate")
    return acc


def sgd_step(msgs, eta: float, x) -> np.ndarray:
    keep, ptrs, sizes = _msg_arrays(msgs)
    x = _f32(x).copy()
    _chk(lib().qo_sgd_step(ptrs, sizes, len(keep), C.c_float(eta), _ptr(x)), "sgd_step")
    return x


def sgd_step_buckets(msgs, eta: float, x, bucket_begin: int, bucket_count: int) -> np.ndarray:
    """The step on the coordinates of a run of buckets; x holds exactly those coordinates.
    `msgs` may be a prepared (arrays, pointers, sizes) triple from prepare_messages()."""
    keep, ptrs, sizes = msgs if isinstance(msgs, tuple) else _msg_arrays(msgs)
    x = _f32(x).copy()
    _chk(lib().qo_sgd_step_buckets(ptrs, sizes, len(keep), C.c_float(eta), _ptr(x),
                                   bucket_begin, bucket_count), "sgd_step_buckets")
    return x


def prepare_messages(msgs):
    """Pointer and size arrays of a list of messages, for repeated calls on the same list."""
    return _msg_arrays(msgs)


def bucket_extent(msg: np.ndarray, b: int):
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    off, cnt = C.c_uint64(0), C.c_uint64(0)
    _chk(lib().qo_bucket_extent(_ptr(msg), msg.nbytes, b, C.byref(off), C.byref(cnt)),
         "bucket_extent")
    return int(off.value), int(cnt.value)


def payload_offset_words(msg: np.ndarray) -> int:
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    off = C.c_uint64(0)
    _chk(lib().qo_payload_offset(_ptr(msg), msg.nbytes, C.byref(off)), "payload_offset")
    return int(off.value) // 4


def bucket_words(msg: np.ndarray, b: int) -> np.ndarray:
    off, cnt = bucket_extent(msg, b)
    base = payload_offset_words(msg)
    return np.asarray(msg[base + off: base + off + cnt])


# ---- tensor-aware messages: tensors = [(offset, size), ...] inside an arena of p.n floats ----

def _tensors(tensors) -> np.ndarray:
    t = np.ascontiguousarray(np.asarray(tensors, dtype=np.uint64).reshape(-1, 2))
    return t


def layout_counts(p: Params, tensors, bypass_below: int):
    """(number of quantization buckets, number of raw fp32 values)."""
    t = _tensors(tensors)
    nb, raw = C.c_uint64(0), C.c_uint64(0)
    cp = p.c()
    _chk(lib().qo_layout_counts(C.byref(cp), _ptr(t), len(t), bypass_below, C.byref(nb),
                                C.byref(raw)), "layout_counts")
    return int(nb.value), int(raw.value)


def encode_layout(p: Params, tensors, bypass_below: int, arena,
                  capacity: int | None = None) -> np.ndarray:
    t = _tensors(tensors)
    arena = _f32(arena)
    assert arena.size == p.n
    cp = p.c()
    cap = int(lib().qo_layout_max_encoded_bytes(C.byref(cp), _ptr(t), len(t), bypass_below)) \
        if capacity is None else capacity
    msg = np.zeros((cap + 3) // 4, dtype=np.uint32)
    used = C.c_size_t(0)
    _chk(lib().qo_encode_layout(C.byref(cp), _ptr(t), len(t), bypass_below, _ptr(arena),
                                _ptr(msg), cap, C.byref(used)), "encode_layout")
    return msg[: used.value // 4].copy()


def decode_layout(tensors, bypass_below: int, msg, n: int) -> np.ndarray:
    t = _tensors(tensors)
    msg = np.ascontiguousarray(msg, dtype=np.uint32)
    out = np.zeros(max(n, 1), dtype=np.float32)
    _chk(lib().qo_decode_layout(_ptr(t), len(t), bypass_below, _ptr(msg), msg.nbytes, _ptr(out)),
         "decode_layout")
    return out[:n]


def decode_accumulate_layout(tensors, bypass_below: int, msgs, acc) -> np.ndarray:
    t = _tensors(tensors)
    keep, ptrs, sizes = _msg_arrays(msgs)
    acc = _f32(acc).copy()
    _chk(lib().qo_decode_accumulate_layout(_ptr(t), len(t), bypass_below, ptrs, sizes, len(keep),
                                           _ptr(acc)), "decode_accumulate_layout")
    return acc


def sgd_step_layout(tensors, bypass_below: int, msgs, eta: float, x) -> np.ndarray:
    t = _tensors(tensors)
    keep, ptrs, sizes = _msg_arrays(msgs)
    x = _f32(x).copy()
    _chk(lib().qo_sgd_step_layout(_ptr(t), len(t), bypass_below, ptrs, sizes, len(keep),
                                  C.c_float(eta), _ptr(x)), "sgd_step_layout")
    return x
