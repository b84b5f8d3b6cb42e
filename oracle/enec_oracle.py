"""ctypes front end of the plain-C ENEC oracle (oracle/enec_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by the cpu_baseline leg of bench.py.  The GPU library never imports it.

`build()` compiles the C file with gcc into oracle/libenec_oracle.so; the
wrappers below only marshal numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "enec_oracle.c")
_LIB = os.path.join(_HERE, "libenec_oracle.so")

OK, E_ARG, E_DTYPE, E_BLOCK, E_PARAMS, E_CAPACITY, E_RANGE, E_FORMAT = range(8)
BF16, FP16, FP32 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle.  -ffp-contract=off keeps Eq. 4 in plain IEEE double."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        u8p, u16p, u64p = C.POINTER(C.c_uint8), C.POINTER(C.c_uint16), C.POINTER(C.c_uint64)
        L.orc_hh_pack.restype = C.c_size_t
        L.orc_hh_pack.argtypes = [u16p, C.c_size_t, C.c_int, u8p]
        L.orc_hh_unpack.restype = C.c_size_t
        L.orc_hh_unpack.argtypes = [u8p, C.c_size_t, C.c_int, u16p]
        for f in (L.orc_transform, L.orc_inverse_transform):
            f.restype = C.c_uint
            f.argtypes = [C.c_uint, C.c_uint, C.c_uint]
        L.orc_in_range.restype = C.c_int
        L.orc_in_range.argtypes = [C.c_uint, C.c_uint, C.c_uint]
        L.orc_width_for.restype = C.c_uint
        L.orc_width_for.argtypes = [C.c_uint, C.c_uint, C.c_uint]
        L.orc_histogram.restype = None
        L.orc_histogram.argtypes = [u16p, C.c_size_t, u64p]
        L.orc_tune_hist.restype = None
        L.orc_tune_hist.argtypes = [u64p, u8p, u64p, C.POINTER(C.c_double)]
        L.orc_tune.restype = None
        L.orc_tune.argtypes = [u16p, C.c_size_t, u8p, u64p, C.POINTER(C.c_double)]
        L.orc_default_block.restype = C.c_uint32
        L.orc_default_block.argtypes = [C.c_size_t]
        L.orc_num_blocks.restype = C.c_size_t
        L.orc_num_blocks.argtypes = [C.c_size_t, C.c_uint32]
        L.orc_payload_base.restype = C.c_size_t
        L.orc_payload_base.argtypes = [C.c_size_t, C.c_uint32]
        L.orc_compress_bound.restype = C.c_size_t
        L.orc_compress_bound.argtypes = [C.c_size_t, C.c_uint32]
        L.orc_compress.restype = C.c_int
        L.orc_compress.argtypes = [u16p, C.c_size_t, C.c_uint32, u8p, u8p, C.c_size_t,
                                   C.POINTER(C.c_size_t)]
        L.orc_stream_info.restype = C.c_int
        L.orc_stream_info.argtypes = [u8p, u8p, u64p, C.POINTER(C.c_uint32), u64p,
                                      C.POINTER(C.c_uint32)]
        L.orc_decompress.restype = C.c_int
        L.orc_decompress.argtypes = [u8p, C.c_size_t, u16p, C.c_size_t]
        L.orc_in_range_e.restype = C.c_int
        L.orc_in_range_e.argtypes = [C.c_uint] * 4
        L.orc_inverse_transform_e.restype = C.c_uint
        L.orc_inverse_transform_e.argtypes = [C.c_uint] * 4
        L.orc_width_for_e.restype = C.c_uint
        L.orc_width_for_e.argtypes = [C.c_uint] * 4
        L.orc_exp_bits.restype = C.c_uint
        L.orc_exp_bits.argtypes = [C.c_int]
        L.orc_histogram_dt.restype = None
        L.orc_histogram_dt.argtypes = [C.c_void_p, C.c_size_t, C.c_int, u64p]
        L.orc_tune_hist_e.restype = None
        L.orc_tune_hist_e.argtypes = [u64p, C.c_uint, u8p, u64p, C.POINTER(C.c_double)]
        L.orc_tune_hist_groups.restype = None
        L.orc_tune_hist_groups.argtypes = [u64p, C.c_uint, C.c_uint, u8p, u64p, C.POINTER(C.c_double)]
        L.orc_table_end.restype = C.c_size_t
        L.orc_table_end.argtypes = [C.c_size_t, C.c_uint32]
        L.orc_payload_base_dt.restype = C.c_size_t
        L.orc_payload_base_dt.argtypes = [C.c_size_t, C.c_uint32, C.c_int]
        L.orc_compress_bound_dt.restype = C.c_size_t
        L.orc_compress_bound_dt.argtypes = [C.c_size_t, C.c_uint32, C.c_int]
        L.orc_compress_dt.restype = C.c_int
        L.orc_compress_dt.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_uint32, u8p, u8p, C.c_size_t,
                                      C.POINTER(C.c_size_t)]
        L.orc_stream_info_dt.restype = C.c_int
        L.orc_stream_info_dt.argtypes = [u8p, u8p, u64p, C.POINTER(C.c_uint32), u64p,
                                         C.POINTER(C.c_uint32), C.POINTER(C.c_int)]
        L.orc_decompress_dt.restype = C.c_int
        L.orc_decompress_dt.argtypes = [u8p, C.c_size_t, C.c_void_p, C.c_size_t]
        L.orc_tuple_table_bytes.restype = C.c_size_t
        L.orc_tuple_table_bytes.argtypes = [C.c_size_t, C.c_uint32]
        L.orc_payload_base_pb.restype = C.c_size_t
        L.orc_payload_base_pb.argtypes = [C.c_size_t, C.c_uint32, C.c_int]
        L.orc_compress_bound_pb.restype = C.c_size_t
        L.orc_compress_bound_pb.argtypes = [C.c_size_t, C.c_uint32, C.c_int]
        L.orc_compress_pb.restype = C.c_int
        L.orc_compress_pb.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_uint32, C.c_uint, u8p, C.c_size_t,
                                      C.POINTER(C.c_size_t)]
        L.orc_stream_per_block.restype = C.c_int
        L.orc_stream_per_block.argtypes = [u8p]
        _lib = L
    return _lib


def _p(arr, ctype):
    return arr.ctypes.data_as(C.POINTER(ctype))


def _u16(w) -> np.ndarray:
    w = np.ascontiguousarray(w)
    assert w.dtype == np.uint16, "bf16 values are passed as their uint16 bit patterns"
    return w.reshape(-1)


def _words(w, dtype: int) -> np.ndarray:
    """Elements as their bit patterns: uint16 for bf16 / fp16, uint32 for fp32."""
    w = np.ascontiguousarray(w)
    want = np.uint32 if dtype == FP32 else np.uint16
    assert w.dtype == want, f"dtype {dtype} takes {want.__name__} bit patterns"
    return w.reshape(-1)


def hh_pack(values, a: int) -> np.ndarray:
    v = np.ascontiguousarray(values, dtype=np.uint16)
    out = np.zeros(2 * v.size + 2, dtype=np.uint8)
    n = lib().orc_hh_pack(_p(v, C.c_uint16), v.size, a, _p(out, C.c_uint8))
    return out[:n].copy()


def hh_unpack(stream, N: int, a: int) -> np.ndarray:
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    out = np.zeros(N, dtype=np.uint16)
    lib().orc_hh_unpack(_p(s, C.c_uint8), N, a, _p(out, C.c_uint16))
    return out


def transform(x: int, b: int, n: int) -> int:
    return int(lib().orc_transform(x, b, n))


def inverse_transform(y: int, b: int, n: int) -> int:
    return int(lib().orc_inverse_transform(y, b, n))


def in_range(x: int, b: int, n: int) -> bool:
    return bool(lib().orc_in_range(x, b, n))


def width_for(b: int, l: int, h: int) -> int:
    return int(lib().orc_width_for(b, l, h))


def exp_bits(dtype: int) -> int:
    return int(lib().orc_exp_bits(dtype))


def in_range_e(x: int, b: int, n: int, E: int) -> bool:
    return bool(lib().orc_in_range_e(x, b, n, E))


def inverse_transform_e(y: int, b: int, n: int, E: int) -> int:
    return int(lib().orc_inverse_transform_e(y, b, n, E))


def width_for_e(b: int, l: int, h: int, E: int) -> int:
    return int(lib().orc_width_for_e(b, l, h, E))


def histogram(w, dtype: int = BF16) -> np.ndarray:
    w = _words(w, dtype)
    hist = np.zeros(256, dtype=np.uint64)
    lib().orc_histogram_dt(w.ctypes.data, w.size, dtype, _p(hist, C.c_uint64))
    return hist


def tune_hist(hist, E: int = 8):
    """-> ((b, n, m, L), D_integer, B_exp); E = width of the exponent field"""
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    params = np.zeros(4, dtype=np.uint8)
    D = C.c_uint64(0)
    bexp = C.c_double(0)
    lib().orc_tune_hist_e(_p(hist, C.c_uint64), E, _p(params, C.c_uint8), C.byref(D), C.byref(bexp))
    return tuple(int(v) for v in params), int(D.value), float(bexp.value)


def tune_hist_groups(hist, E: int = 8, lengths=(8, 16, 32)):
    """Eq. 4 with the group length searched jointly with m -> ((b, n, m, L), D_integer, B_exp)"""
    hist = np.ascontiguousarray(hist, dtype=np.uint64)
    params = np.zeros(4, dtype=np.uint8)
    D = C.c_uint64(0)
    bexp = C.c_double(0)
    mask = 0
    for v in lengths:
        mask |= int(v)
    lib().orc_tune_hist_groups(_p(hist, C.c_uint64), E, mask, _p(params, C.c_uint8), C.byref(D), C.byref(bexp))
    return tuple(int(v) for v in params), int(D.value), float(bexp.value)


def tune(w, dtype: int = BF16, lengths=None):
    """-> (b, n, m, L) for a tensor of bit patterns; L = 16 unless a set of group lengths is given."""
    if lengths is None:
        return tune_hist(histogram(w, dtype), exp_bits(dtype))[0]
    return tune_hist_groups(histogram(w, dtype), exp_bits(dtype), lengths)[0]


SAMPLE_CHUNK = 4096


def sample(w, every: int, dtype: int = BF16) -> np.ndarray:
    """The elements a sampled tuner looks at: index e with (e // 4096) % every == 0, in order."""
    w = _words(w, dtype)
    e = np.arange(w.size, dtype=np.int64)
    return w[(e // SAMPLE_CHUNK) % every == 0]


def compress_sampled(w, every: int, B: int = 16384, dtype: int = BF16):
    """Sec. V-E on the sample, then the codec; if an exponent the sample missed is out of range, once more
    with n = width of the exponent field, where the transform is a bijection (Sec. V-C).
    -> (tuple used, status, stream)"""
    w = _words(w, dtype)
    prm = tune(sample(w, every, dtype), dtype)
    rc, s = compress(w, prm, B, dtype=dtype)
    if rc == E_RANGE:
        prm = (prm[0], exp_bits(dtype), prm[2], prm[3])
        rc, s = compress(w, prm, B, dtype=dtype)
    return prm, rc, s


def default_block(n_elems: int) -> int:
    return int(lib().orc_default_block(n_elems))


def num_blocks(n_elems: int, B: int) -> int:
    return int(lib().orc_num_blocks(n_elems, B))


def table_end(n_elems: int, B: int) -> int:
    return int(lib().orc_table_end(n_elems, B))


def payload_base(n_elems: int, B: int, dtype: int = BF16) -> int:
    return int(lib().orc_payload_base_dt(n_elems, B, dtype))


def compress_bound(n_elems: int, B: int, dtype: int = BF16) -> int:
    return int(lib().orc_compress_bound_dt(n_elems, B, dtype))


def compress(w, params, B: int = 16384, capacity: int | None = None, dtype: int = BF16):
    """-> (status, stream bytes as uint8 array).  On E_RANGE the array holds everything before the payloads."""
    w = _words(w, dtype)
    cap = compress_bound(w.size, B, dtype) if capacity is None else capacity
    out = np.zeros(max(cap, 1), dtype=np.uint8)
    prm = np.asarray(params, dtype=np.uint8)
    nbytes = C.c_size_t(0)
    rc = lib().orc_compress_dt(w.ctypes.data, w.size, dtype, B, _p(prm, C.c_uint8), _p(out, C.c_uint8),
                               cap, C.byref(nbytes))
    if rc == OK:
        return rc, out[:nbytes.value].copy()
    if rc == E_RANGE:
        return rc, out[:payload_base(w.size, B, dtype)].copy()
    return rc, None


def payload_base_pb(n_elems: int, B: int, dtype: int = BF16) -> int:
    return int(lib().orc_payload_base_pb(n_elems, B, dtype))


def compress_bound_pb(n_elems: int, B: int, dtype: int = BF16) -> int:
    return int(lib().orc_compress_bound_pb(n_elems, B, dtype))


def compress_per_block(w, B: int = 16384, dtype: int = BF16, L: int = 16):
    """One tuned (b, n, m) per data block -> (status, stream bytes as uint8 array)."""
    w = _words(w, dtype)
    cap = compress_bound_pb(w.size, B, dtype)
    out = np.zeros(max(cap, 1), dtype=np.uint8)
    nbytes = C.c_size_t(0)
    rc = lib().orc_compress_pb(w.ctypes.data, w.size, dtype, B, L, _p(out, C.c_uint8), cap, C.byref(nbytes))
    return rc, (out[:nbytes.value].copy() if rc == OK else None)


def block_tuples(stream) -> list:
    """The (b, n, m) of every data block of a stream that carries one tuple per block."""
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    info = stream_info(s)
    assert info["per_block"]
    nb = num_blocks(info["n_elems"], info["block_size"])
    at = table_end(info["n_elems"], info["block_size"])
    return [tuple(int(v) for v in s[at + 4 * k:at + 4 * k + 3]) for k in range(nb)]


def stream_info(stream) -> dict:
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    params = np.zeros(4, dtype=np.uint8)
    n = C.c_uint64(0)
    B = C.c_uint32(0)
    total = C.c_uint64(0)
    status = C.c_uint32(0)
    dt = C.c_int(0)
    rc = lib().orc_stream_info_dt(_p(s, C.c_uint8), _p(params, C.c_uint8), C.byref(n), C.byref(B),
                                  C.byref(total), C.byref(status), C.byref(dt))
    return dict(rc=rc, params=tuple(int(v) for v in params), n_elems=int(n.value),
                block_size=int(B.value), total_bytes=int(total.value), status=int(status.value),
                dtype=int(dt.value), per_block=bool(s.size > 40 and lib().orc_stream_per_block(_p(s, C.c_uint8))))


def decompress(stream, n_elems: int):
    """-> (status, array of bit patterns: uint32 if the header says fp32, else uint16)"""
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    fp32 = s.size > 6 and int(s[6]) == FP32
    out = np.zeros(n_elems, dtype=np.uint32 if fp32 else np.uint16)
    rc = lib().orc_decompress_dt(_p(s, C.c_uint8), s.size, out.ctypes.data, n_elems)
    return rc, out
