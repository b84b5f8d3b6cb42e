"""Thin Python binding of libenec's C ABI (include/enec.h).

Argument marshalling only: every step of the codec runs in the library's HIP kernels.
PyTorch is used for device memory and streams, nothing else.  There is no CPU fallback:
if libenec.so has not been built, or there is no GPU, the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libenec.so")

OK, E_ARG, E_DTYPE, E_BLOCK, E_PARAMS, E_CAPACITY, E_RANGE, E_FORMAT, E_HIP = range(9)
BF16, FP16, FP32 = 0, 1, 2
HEADER_BYTES = 64

EXPORTS = [
    "enec_version", "enec_strerror", "enec_default_block_size", "enec_compress_bound",
    "enec_workspace_bytes", "enec_workspace_init", "enec_compress", "enec_decompress",
    "enec_decompress_with_header", "enec_tune", "enec_tune_histogram", "enec_stream_info",
    "enec_copy", "enec_compress_batch", "enec_decompress_batch", "enec_tune_histogram_groups",
    "enec_tune_sampled", "enec_compress_sampled", "enec_compress_bound_per_block", "enec_compress_per_block", "enec_compress_per_block_batch",
    "enec_tune_batch", "enec_compress_static", "enec_pipeline_create", "enec_pipeline_destroy",
    "enec_pipeline_prefetch", "enec_pipeline_prefetch_from_host", "enec_pipeline_acquire", "enec_pipeline_release",
    "enec_pipeline_trace",
]


class TuneItem(C.Structure):
    _fields_ = [("src", C.c_void_p), ("n_elems", C.c_size_t)]


class Params(C.Structure):
    _fields_ = [("b", C.c_uint8), ("n", C.c_uint8), ("m", C.c_uint8), ("L", C.c_uint8)]

    def astuple(self):
        return (self.b, self.n, self.m, self.L)


class CompressItem(C.Structure):
    _fields_ = [("src", C.c_void_p), ("n_elems", C.c_size_t), ("block_size", C.c_uint32),
                ("params", C.POINTER(Params)), ("out", C.c_void_p), ("out_capacity", C.c_size_t),
                ("out_bytes", C.c_void_p)]


class DecompressItem(C.Structure):
    _fields_ = [("src", C.c_void_p), ("in_bytes", C.c_size_t), ("host_header", C.c_void_p),
                ("out", C.c_void_p), ("n_elems", C.c_size_t), ("status", C.c_void_p)]


class PerBlockItem(C.Structure):
    _fields_ = [("src", C.c_void_p), ("n_elems", C.c_size_t), ("block_size", C.c_uint32), ("out", C.c_void_p),
                ("out_capacity", C.c_size_t), ("out_bytes", C.c_void_p)]


class OffloadItem(C.Structure):
    _fields_ = [("host_stream", C.c_void_p), ("stream_bytes", C.c_size_t), ("out", C.c_void_p),
                ("n_elems", C.c_size_t), ("status", C.c_void_p)]


class EnecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None


def lib():
    """Loads libenec.so (built in-tree by paper_2604_03298_amd.build) or raises."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2604_03298_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, sz, u32, u64p = C.c_void_p, C.c_size_t, C.c_uint32, C.POINTER(C.c_uint64)
        L.enec_version.restype = u32
        L.enec_version.argtypes = []
        L.enec_strerror.restype = C.c_char_p
        L.enec_strerror.argtypes = [C.c_int]
        L.enec_default_block_size.restype = u32
        L.enec_default_block_size.argtypes = [sz]
        L.enec_compress_bound.restype = sz
        L.enec_compress_bound.argtypes = [sz, C.c_int, u32]
        L.enec_workspace_bytes.restype = sz
        L.enec_workspace_bytes.argtypes = [sz, u32]
        L.enec_workspace_init.restype = C.c_int
        L.enec_workspace_init.argtypes = [vp, sz, vp]
        L.enec_compress.restype = C.c_int
        L.enec_compress.argtypes = [vp, sz, C.c_int, u32, C.POINTER(Params), vp, sz, vp, vp, sz, vp]
        L.enec_compress_static.restype = C.c_int
        L.enec_compress_static.argtypes = [vp, sz, C.c_int, u32, C.POINTER(Params), vp, sz, vp, vp]
        L.enec_decompress.restype = C.c_int
        L.enec_decompress.argtypes = [vp, sz, vp, sz, vp]
        L.enec_decompress_with_header.restype = C.c_int
        L.enec_decompress_with_header.argtypes = [vp, sz, vp, vp, sz, vp, vp]
        L.enec_tune.restype = C.c_int
        L.enec_tune.argtypes = [vp, sz, C.c_int, C.POINTER(Params), u64p, vp, sz, vp]
        L.enec_compress_bound_per_block.restype = sz
        L.enec_compress_bound_per_block.argtypes = [sz, C.c_int, C.c_uint32]
        L.enec_compress_per_block.restype = C.c_int
        L.enec_compress_per_block.argtypes = [vp, sz, C.c_int, C.c_uint32, C.c_uint32, vp, sz, vp, vp, sz, vp]
        L.enec_compress_per_block_batch.restype = C.c_int
        L.enec_compress_per_block_batch.argtypes = [C.POINTER(PerBlockItem), sz, C.c_int, C.c_uint32, vp, sz, vp]
        L.enec_tune_batch.restype = C.c_int
        L.enec_tune_batch.argtypes = [C.POINTER(TuneItem), sz, C.c_int, C.c_uint32, C.POINTER(Params), u64p, vp, sz, vp]
        L.enec_tune_sampled.restype = C.c_int
        L.enec_tune_sampled.argtypes = [vp, sz, C.c_int, C.c_uint32, C.POINTER(Params), u64p, vp, sz, vp]
        L.enec_compress_sampled.restype = C.c_int
        L.enec_compress_sampled.argtypes = [vp, sz, C.c_int, C.c_uint32, C.c_uint32, C.POINTER(Params), vp, sz,
                                            vp, sz, vp]
        L.enec_tune_histogram.restype = C.c_int
        L.enec_tune_histogram.argtypes = [u64p, C.c_int, C.POINTER(Params)]
        L.enec_tune_histogram_groups.restype = C.c_int
        L.enec_tune_histogram_groups.argtypes = [u64p, C.c_int, u32, u32, C.POINTER(Params)]
        L.enec_stream_info.restype = C.c_int
        L.enec_stream_info.argtypes = [vp, C.POINTER(Params), u64p, C.POINTER(u32), u64p,
                                       C.POINTER(C.c_int), C.POINTER(u32)]
        L.enec_copy.restype = C.c_int
        L.enec_copy.argtypes = [vp, vp, sz, vp]
        L.enec_compress_batch.restype = C.c_int
        L.enec_compress_batch.argtypes = [C.POINTER(CompressItem), sz, C.c_int, vp, sz, vp]
        L.enec_decompress_batch.restype = C.c_int
        L.enec_decompress_batch.argtypes = [C.POINTER(DecompressItem), sz, vp]
        L.enec_pipeline_create.restype = C.c_int
        L.enec_pipeline_create.argtypes = [C.POINTER(vp), u32, vp, vp, vp, sz, C.c_int]
        L.enec_pipeline_destroy.restype = None
        L.enec_pipeline_destroy.argtypes = [vp]
        L.enec_pipeline_prefetch.restype = C.c_int
        L.enec_pipeline_prefetch.argtypes = [vp, u32, C.POINTER(DecompressItem), sz]
        L.enec_pipeline_prefetch_from_host.restype = C.c_int
        L.enec_pipeline_prefetch_from_host.argtypes = [vp, u32, C.POINTER(OffloadItem), sz]
        L.enec_pipeline_acquire.restype = C.c_int
        L.enec_pipeline_acquire.argtypes = [vp, u32, vp]
        L.enec_pipeline_release.restype = C.c_int
        L.enec_pipeline_release.argtypes = [vp, u32, vp]
        L.enec_pipeline_trace.restype = C.c_int
        L.enec_pipeline_trace.argtypes = [vp, C.POINTER(C.c_float), sz, C.POINTER(sz)]
        _lib = L
    return _lib


def _check(rc: int, where: str):
    if rc != OK:
        raise EnecError(rc, where)


def _stream_handle(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _params(p) -> Params:
    return p if isinstance(p, Params) else Params(*[int(v) for v in p])


def dtype_of(t, dtype=None) -> int:
    """The library's dtype code for a torch tensor: float16 -> FP16, 4-byte elements -> FP32,
    any other 2-byte element (bfloat16, or int16 / uint16 bit patterns) -> BF16, unless given."""
    if dtype is not None:
        return int(dtype)
    import torch
    if getattr(t, "dtype", None) == torch.float16:
        return FP16
    return FP32 if hasattr(t, "element_size") and t.element_size() == 4 else BF16


# ---- host-only entry points -------------------------------------------------------
def version() -> int:
    return int(lib().enec_version())


def strerror(status: int) -> str:
    return lib().enec_strerror(int(status)).decode()


def default_block_size(n_elems: int) -> int:
    return int(lib().enec_default_block_size(n_elems))


def compress_bound(n_elems: int, dtype: int = BF16, block_size: int = 0) -> int:
    return int(lib().enec_compress_bound(n_elems, dtype, block_size))


def workspace_bytes(n_elems: int, block_size: int = 0) -> int:
    return int(lib().enec_workspace_bytes(n_elems, block_size))


def tune_histogram(hist, dtype: int = BF16, lengths=None, block_size: int = 0) -> tuple:
    """(b, n, m, L) from a 256-bin exponent histogram; L = 16 unless candidate group lengths are given (the
    library leaves out those that block_size, 0 = 16384, does not admit)."""
    h = np.ascontiguousarray(hist, dtype=np.uint64)
    assert h.size == 256
    p = Params()
    if lengths is None:
        _check(lib().enec_tune_histogram(h.ctypes.data_as(C.POINTER(C.c_uint64)), dtype, C.byref(p)),
               "enec_tune_histogram")
    else:
        mask = 0
        for v in lengths:
            mask |= int(v)
        _check(lib().enec_tune_histogram_groups(h.ctypes.data_as(C.POINTER(C.c_uint64)), dtype, mask, block_size,
                                                C.byref(p)),
               "enec_tune_histogram_groups")
    return p.astuple()


def stream_info(header) -> dict:
    """header: bytes / numpy uint8 array holding at least the first 64 bytes of a stream."""
    buf = np.frombuffer(bytes(header[:HEADER_BYTES]), dtype=np.uint8).copy()
    p, n, B, total = Params(), C.c_uint64(0), C.c_uint32(0), C.c_uint64(0)
    dtype, status = C.c_int(0), C.c_uint32(0)
    rc = lib().enec_stream_info(buf.ctypes.data, C.byref(p), C.byref(n), C.byref(B), C.byref(total),
                                C.byref(dtype), C.byref(status))
    return dict(rc=rc, params=p.astuple(), n_elems=int(n.value), block_size=int(B.value),
                total_bytes=int(total.value), dtype=int(dtype.value), status=int(status.value),
                per_block=bool(rc == OK and buf[40] == 1))      # header byte 40: one tuple per data block


# ---- device entry points (torch tensors carry the pointers) ------------------------
def workspace_init(workspace, stream=None):
    _check(lib().enec_workspace_init(C.c_void_p(workspace.data_ptr()),
                                     workspace.numel() * workspace.element_size(),
                                     _stream_handle(stream)), "enec_workspace_init")


def new_workspace(n_elems: int, block_size: int = 0, device="cuda", stream=None):
    """Allocates (torch) and zeroes (library fill kernel) a workspace for tensors up to n_elems."""
    import torch
    ws = torch.empty(workspace_bytes(n_elems, block_size), dtype=torch.uint8, device=device)
    workspace_init(ws, stream)
    return ws


def compress(src, params, out, workspace, block_size: int = 0, out_bytes=None, stream=None,
             n_elems: int | None = None, dtype: int | None = None) -> int:
    """Enqueues enec_compress.  src: device tensor of 2- or 4-byte elements (dtype: see dtype_of);
    params: (b, n, m, L) or None (tune first); out: device uint8 tensor of >= compress_bound bytes;
    out_bytes: None or a device / pinned-host tensor with room for one u64.  Returns the status
    code (range errors are reported through the stream header, not here)."""
    n = src.numel() if n_elems is None else n_elems
    dt = dtype_of(src, dtype)
    assert src.element_size() == (4 if dt == FP32 else 2)
    pp = C.byref(_params(params)) if params is not None else None
    ob = C.c_void_p(out_bytes.data_ptr()) if out_bytes is not None else None
    return int(lib().enec_compress(
        C.c_void_p(src.data_ptr()), n, dt, block_size, pp, C.c_void_p(out.data_ptr()),
        out.numel() * out.element_size(), ob, C.c_void_p(workspace.data_ptr()),
        workspace.numel() * workspace.element_size(), _stream_handle(stream)))


STATIC_SCRATCH_BYTES = 1 << 20


def compress_static(src, params, out, block_size: int = 0, out_bytes=None, stream=None,
                    n_elems: int | None = None, dtype: int | None = None) -> int:
    """Enqueues enec_compress_static: enec_compress on the library's own scratch array (no workspace,
    no allocation); params must be given."""
    n = src.numel() if n_elems is None else n_elems
    dt = dtype_of(src, dtype)
    pp = C.byref(_params(params)) if params is not None else None
    ob = C.c_void_p(out_bytes.data_ptr()) if out_bytes is not None else None
    return int(lib().enec_compress_static(
        C.c_void_p(src.data_ptr()), n, dt, block_size, pp, C.c_void_p(out.data_ptr()),
        out.numel() * out.element_size(), ob, _stream_handle(stream)))


def compress_bound_per_block(n_elems: int, dtype: int = BF16, block_size: int = 0) -> int:
    return int(lib().enec_compress_bound_per_block(n_elems, dtype, block_size))


def compress_per_block(src, out, workspace, block_size: int = 0, out_bytes=None, stream=None,
                       n_elems: int | None = None, dtype: int | None = None, group_length: int = 0) -> int:
    """Enqueues enec_compress_per_block: every data block is coded with the tuple tuned on its own
    exponents.  out: device uint8 tensor of >= compress_bound_per_block bytes."""
    n = src.numel() if n_elems is None else n_elems
    dt = dtype_of(src, dtype)
    ob = C.c_void_p(out_bytes.data_ptr()) if out_bytes is not None else None
    return int(lib().enec_compress_per_block(
        C.c_void_p(src.data_ptr()), n, dt, block_size, group_length, C.c_void_p(out.data_ptr()),
        out.numel() * out.element_size(), ob, C.c_void_p(workspace.data_ptr()),
        workspace.numel() * workspace.element_size(), _stream_handle(stream)))


def compress_per_block_batch(srcs, outs, workspace, out_bytes=None, stream=None, dtype: int | None = None,
                             block_sizes=None, group_length: int = 0) -> int:
    """Enqueues enec_compress_per_block_batch: the tensors of one block size share a launch.  out_bytes: None or
    one device int64 tensor (or None) per tensor; block_sizes: None (defaults) or one block size per tensor."""
    n = len(srcs)
    items = (PerBlockItem * max(n, 1))()
    for i in range(n):
        items[i].src = srcs[i].data_ptr()
        items[i].n_elems = srcs[i].numel()
        items[i].block_size = block_sizes[i] if block_sizes is not None else 0
        items[i].out = outs[i].data_ptr()
        items[i].out_capacity = outs[i].numel() * outs[i].element_size()
        ob = out_bytes[i] if out_bytes is not None else None
        items[i].out_bytes = ob.data_ptr() if ob is not None else None
    dt = dtype_of(srcs[0], dtype) if n else (BF16 if dtype is None else dtype)
    return int(lib().enec_compress_per_block_batch(items, n, dt, group_length, C.c_void_p(workspace.data_ptr()),
                                                   workspace.numel() * workspace.element_size(), _stream_handle(stream)))


def decompress(stream_buf, out, n_elems: int | None = None, stream=None) -> int:
    n = out.numel() if n_elems is None else n_elems
    return int(lib().enec_decompress(C.c_void_p(stream_buf.data_ptr()),
                                     stream_buf.numel() * stream_buf.element_size(),
                                     C.c_void_p(out.data_ptr()), n, _stream_handle(stream)))


def decompress_with_header(stream_buf, host_header, out, n_elems: int | None = None, stream=None, status=None) -> int:
    """status: None, or a device / pinned-host int32 tensor holding 0; the kernel stores E_FORMAT there if it
    leaves a data block undecoded."""
    n = out.numel() if n_elems is None else n_elems
    hdr = np.frombuffer(bytes(host_header[:HEADER_BYTES]), dtype=np.uint8).copy()
    return int(lib().enec_decompress_with_header(
        C.c_void_p(stream_buf.data_ptr()), stream_buf.numel() * stream_buf.element_size(),
        hdr.ctypes.data, C.c_void_p(out.data_ptr()), n,
        C.c_void_p(status.data_ptr()) if status is not None else None, _stream_handle(stream)))


def compress_batch(srcs, params, outs, workspace, block_sizes=None, out_bytes=None, stream=None,
                   dtype: int | None = None) -> int:
    """Enqueues enec_compress_batch.  srcs / outs: lists of device tensors (one element format for
    all, see dtype_of); params: list of (b, n, m, L) or None per tensor; out_bytes: None or a list
    of one-u64 device-accessible tensors."""
    n = len(srcs)
    dt = dtype_of(srcs[0], dtype) if n else BF16
    keep = [_params(p) if p is not None else None for p in params]
    items = (CompressItem * n)()
    for i in range(n):
        items[i].src = srcs[i].data_ptr()
        items[i].n_elems = srcs[i].numel()
        items[i].block_size = block_sizes[i] if block_sizes else 0
        items[i].params = C.pointer(keep[i]) if keep[i] is not None else None
        items[i].out = outs[i].data_ptr()
        items[i].out_capacity = outs[i].numel() * outs[i].element_size()
        items[i].out_bytes = out_bytes[i].data_ptr() if out_bytes is not None else None
    return int(lib().enec_compress_batch(items, n, dt, C.c_void_p(workspace.data_ptr()),
                                         workspace.numel() * workspace.element_size(),
                                         _stream_handle(stream)))


def make_decompress_items(stream_bufs, host_headers, outs, statuses=None):
    """Builds the item array for decompress_batch once (it can be reused for repeated calls).
    statuses: None or one device-accessible int32 tensor (holding 0) per stream.  Returns (items, keepalive)."""
    n = len(stream_bufs)
    hdrs = [np.frombuffer(bytes(h[:HEADER_BYTES]), dtype=np.uint8).copy() for h in host_headers]
    items = (DecompressItem * n)()
    for i in range(n):
        items[i].src = stream_bufs[i].data_ptr()
        items[i].in_bytes = stream_bufs[i].numel() * stream_bufs[i].element_size()
        items[i].host_header = hdrs[i].ctypes.data
        items[i].out = outs[i].data_ptr()
        items[i].n_elems = outs[i].numel()
        items[i].status = statuses[i].data_ptr() if statuses is not None else None
    return items, hdrs


def decompress_batch(stream_bufs, host_headers, outs, stream=None, items=None, statuses=None) -> int:
    keep = None
    if items is None:
        items, keep = make_decompress_items(stream_bufs, host_headers, outs, statuses)
    return int(lib().enec_decompress_batch(items, len(items), _stream_handle(stream)))


def tune(src, workspace, stream=None, want_histogram: bool = False, dtype: int | None = None, lengths=None,
         block_size: int = 0):
    """-> (b, n, m, L) [, histogram]; synchronous.  lengths: candidate group lengths for Eq. 4's joint
    search of (m, L), e.g. (8, 16, 32); None keeps the paper's L = 16.  block_size: the data-block size the
    tensor will be compressed with (0 = the default for its length)."""
    p = Params()
    hist = np.zeros(256, dtype=np.uint64)
    dt = dtype_of(src, dtype)
    _check(lib().enec_tune(C.c_void_p(src.data_ptr()), src.numel(), dt, C.byref(p),
                           hist.ctypes.data_as(C.POINTER(C.c_uint64)),
                           C.c_void_p(workspace.data_ptr()),
                           workspace.numel() * workspace.element_size(), _stream_handle(stream)),
           "enec_tune")
    prm = p.astuple() if lengths is None else tune_histogram(hist, dt, lengths,
                                                             block_size or default_block_size(src.numel()))
    return (prm, hist) if want_histogram else prm


def tune_batch(srcs, workspace, every: int = 1, stream=None, dtype: int | None = None, want_histograms: bool = False):
    """[(b, n, m, 16), ...] for a list of device tensors of one element format; one wait per sixteen tensors."""
    n = len(srcs)
    items = (TuneItem * n)()
    for i, s in enumerate(srcs):
        items[i].src = s.data_ptr()
        items[i].n_elems = s.numel()
    out = (Params * n)()
    hist = np.zeros((n, 256), dtype=np.uint64)
    dt = dtype_of(srcs[0], dtype) if n else BF16
    _check(lib().enec_tune_batch(items, n, dt, every, out, hist.ctypes.data_as(C.POINTER(C.c_uint64)),
                                 C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size(),
                                 _stream_handle(stream)), "enec_tune_batch")
    prm = [out[i].astuple() for i in range(n)]
    return (prm, hist) if want_histograms else prm


def tune_sampled(src, every: int, workspace, stream=None, dtype: int | None = None, want_histogram: bool = False):
    """(b, n, m, 16) from the exponents of every `every`-th chunk of 4096 elements; synchronous."""
    p = Params()
    hist = np.zeros(256, dtype=np.uint64)
    _check(lib().enec_tune_sampled(C.c_void_p(src.data_ptr()), src.numel(), dtype_of(src, dtype), every,
                                   C.byref(p), hist.ctypes.data_as(C.POINTER(C.c_uint64)),
                                   C.c_void_p(workspace.data_ptr()),
                                   workspace.numel() * workspace.element_size(), _stream_handle(stream)),
           "enec_tune_sampled")
    return (p.astuple(), hist) if want_histogram else p.astuple()


def compress_sampled(src, every: int, out, workspace, block_size: int = 0, stream=None,
                     dtype: int | None = None):
    """Tunes on a sample, compresses, and compresses again with the full exponent width if the sample
    missed an exponent.  Synchronous.  -> (status, tuple of the stream in `out`)."""
    p = Params()
    rc = int(lib().enec_compress_sampled(
        C.c_void_p(src.data_ptr()), src.numel(), dtype_of(src, dtype), block_size, every, C.byref(p),
        C.c_void_p(out.data_ptr()), out.numel() * out.element_size(), C.c_void_p(workspace.data_ptr()),
        workspace.numel() * workspace.element_size(), _stream_handle(stream)))
    return rc, p.astuple()


def copy(dst, src, nbytes: int | None = None, stream=None) -> int:
    nb = src.numel() * src.element_size() if nbytes is None else nbytes
    return int(lib().enec_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nb,
                               _stream_handle(stream)))


class Pipeline:
    """Handle of an enec_pipeline (include/enec.h): layer-wise decompression on a side stream, ordered
    against the consumer's stream with events; optionally fed from pinned host memory through a staging
    buffer.  Marshals arguments only."""

    def __init__(self, n_slots: int, decompress_stream, copy_stream=None, staging=None, trace: bool = False):
        self._h = C.c_void_p()
        self._keep = (decompress_stream, copy_stream, staging)
        _check(lib().enec_pipeline_create(
            C.byref(self._h), n_slots, C.c_void_p(decompress_stream.cuda_stream),
            C.c_void_p(copy_stream.cuda_stream) if copy_stream is not None else None,
            C.c_void_p(staging.data_ptr()) if staging is not None else None,
            staging.numel() * staging.element_size() if staging is not None else 0, int(trace)),
            "enec_pipeline_create")

    def close(self):
        if self._h:
            lib().enec_pipeline_destroy(self._h)
            self._h = C.c_void_p()

    __del__ = close

    def prefetch(self, slot: int, items) -> int:
        """items: the array make_decompress_items returns (device streams)."""
        return int(lib().enec_pipeline_prefetch(self._h, slot, items, len(items)))

    def prefetch_from_host(self, slot: int, host_streams, outs) -> int:
        """host_streams: pinned uint8 tensors, each one whole stream; outs: device tensors."""
        n = len(host_streams)
        items = (OffloadItem * n)()
        for i in range(n):
            items[i].host_stream = host_streams[i].data_ptr()
            items[i].stream_bytes = host_streams[i].numel()
            items[i].out = outs[i].data_ptr()
            items[i].n_elems = outs[i].numel()
            items[i].status = None
        return int(lib().enec_pipeline_prefetch_from_host(self._h, slot, items, n))

    def acquire(self, slot: int, consumer_stream=None) -> int:
        return int(lib().enec_pipeline_acquire(self._h, slot, _stream_handle(consumer_stream)))

    def release(self, slot: int, consumer_stream=None) -> int:
        return int(lib().enec_pipeline_release(self._h, slot, _stream_handle(consumer_stream)))

    def trace(self, max_steps: int = 4096):
        """Waits for the recorded steps; -> array (steps, 4) of milliseconds: copy start, copy end,
        decompression start, decompression end (-1 where a step had no copy)."""
        ms = np.zeros((max_steps, 4), dtype=np.float32)
        n = C.c_size_t(0)
        _check(lib().enec_pipeline_trace(self._h, ms.ctypes.data_as(C.POINTER(C.c_float)), max_steps, C.byref(n)),
               "enec_pipeline_trace")
        return ms[:min(int(n.value), max_steps)].copy()
