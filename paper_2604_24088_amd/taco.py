"""Thin ctypes binding of the C ABI in include/taco.h (libtaco_hip.so).

Argument marshalling only: every step of the operator runs in the HIP kernels.  PyTorch
supplies device memory and the stream.  There is no CPU fallback: if the library is not
built or cannot be loaded, the first call raises.

Function names follow the C entry points (taco_compress, taco_decompress,
taco_decompress_sum, ...).  Tensors: bf16 input/output as torch.bfloat16, payload as
torch.uint8 (E4M3 codes), scales as torch.float32 of shape [n_blocks, 2] = {alpha, s}.
"""
import ctypes
import os
from typing import Optional, Sequence

import torch

from . import build as _build

TACO_MAX_K = 16
TACO_MAX_BATCH = 32
TACO_MAX_BATCH_PAYLOADS = 128
TACO_FORMAT_E4M3, TACO_FORMAT_E5M2, TACO_FORMAT_INT8 = 0, 1, 2
TACO_MODE_RESCALE, TACO_MODE_ROTATE, TACO_MODE_POSTSCALE, TACO_MODE_FULL = 1, 2, 4, 7
TACO_IMPL_AUTO, TACO_IMPL_BUTTERFLY, TACO_IMPL_MFMA = 0, 1, 2
TACO_LAYOUT_SPLIT, TACO_LAYOUT_INTERLEAVED = 0, 1

# every symbol include/taco.h declares, then those of include/taco_debug.h
EXPORTS = ("taco_default_params", "taco_payload_bytes", "taco_scales_bytes", "taco_compress", "taco_decompress",
           "taco_decompress_sum", "taco_decompress_sum_compress", "taco_compress_batch", "taco_decompress_sum_batch",
           "taco_decompress_sum_compress_batch", "taco_strerror", "taco_version", "taco_build_id")
DEBUG_EXPORTS = ("taco_debug_cvt_e4m3", "taco_debug_copy", "taco_debug_traffic")


class taco_params(ctypes.Structure):
    _fields_ = [("block", ctypes.c_int32), ("tau", ctypes.c_float), ("eps", ctypes.c_float),
                ("format", ctypes.c_int32), ("impl", ctypes.c_int32), ("layout", ctypes.c_int32),
                ("mode", ctypes.c_int32)]


class taco_compress_item(ctypes.Structure):
    _fields_ = [("x_bf16", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("payload", ctypes.c_void_p), ("scales", ctypes.c_void_p)]


class taco_decode_item(ctypes.Structure):
    _fields_ = [("payloads", ctypes.POINTER(ctypes.c_void_p)), ("scales", ctypes.POINTER(ctypes.c_void_p)),
                ("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("out_bf16", ctypes.c_void_p)]


class taco_recompress_item(ctypes.Structure):
    _fields_ = [("payloads", ctypes.POINTER(ctypes.c_void_p)), ("scales", ctypes.POINTER(ctypes.c_void_p)),
                ("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("payload_out", ctypes.c_void_p),
                ("scales_out", ctypes.c_void_p)]


class TacoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {taco_strerror(status)} (status {status})")


_LIB = None


def lib() -> ctypes.CDLL:
    """Load libtaco_hip.so (built in-tree by paper_2604_24088_amd.build)."""
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -m paper_2604_24088_amd.build` "
                              "(hipcc, gfx950); there is no fallback path")
        L = ctypes.CDLL(path)
        c = ctypes
        L.taco_default_params.restype = None
        L.taco_default_params.argtypes = [c.POINTER(taco_params)]
        L.taco_payload_bytes.restype = c.c_size_t
        L.taco_payload_bytes.argtypes = [c.c_int64, c.c_int32]
        L.taco_scales_bytes.restype = c.c_size_t
        L.taco_scales_bytes.argtypes = [c.c_int64, c.c_int32]
        L.taco_compress.restype = c.c_int
        L.taco_compress.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.POINTER(taco_params),
                                    c.c_void_p, c.c_void_p, c.c_void_p]
        L.taco_decompress.restype = c.c_int
        L.taco_decompress.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int64,
                                      c.POINTER(taco_params), c.c_void_p, c.c_void_p]
        L.taco_decompress_sum.restype = c.c_int
        L.taco_decompress_sum.argtypes = [c.POINTER(c.c_void_p), c.POINTER(c.c_void_p), c.c_int32,
                                          c.c_int64, c.c_int64, c.POINTER(taco_params),
                                          c.c_void_p, c.c_void_p]
        L.taco_decompress_sum_compress.restype = c.c_int
        L.taco_decompress_sum_compress.argtypes = [c.POINTER(c.c_void_p), c.POINTER(c.c_void_p), c.c_int32,
                                                   c.c_int64, c.c_int64, c.POINTER(taco_params),
                                                   c.c_void_p, c.c_void_p, c.c_void_p]
        L.taco_compress_batch.restype = c.c_int
        L.taco_compress_batch.argtypes = [c.POINTER(taco_compress_item), c.c_int32, c.POINTER(taco_params), c.c_void_p]
        L.taco_decompress_sum_batch.restype = c.c_int
        L.taco_decompress_sum_batch.argtypes = [c.POINTER(taco_decode_item), c.c_int32, c.c_int32, c.POINTER(taco_params),
                                                c.c_void_p]
        L.taco_decompress_sum_compress_batch.restype = c.c_int
        L.taco_decompress_sum_compress_batch.argtypes = [c.POINTER(taco_recompress_item), c.c_int32, c.c_int32,
                                                         c.POINTER(taco_params), c.c_void_p]
        L.taco_build_id.restype = c.c_char_p
        L.taco_build_id.argtypes = []
        L.taco_debug_cvt_e4m3.restype = c.c_int
        L.taco_debug_cvt_e4m3.argtypes = [c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p]
        L.taco_debug_copy.restype = c.c_int
        L.taco_debug_copy.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_void_p]
        L.taco_debug_traffic.restype = c.c_int
        L.taco_debug_traffic.argtypes = [c.POINTER(c.c_void_p), c.c_int32, c.c_int32, c.c_void_p, c.c_int32,
                                         c.c_int64, c.c_void_p]
        L.taco_strerror.restype = c.c_char_p
        L.taco_strerror.argtypes = [c.c_int]
        L.taco_version.restype = c.c_char_p
        L.taco_version.argtypes = []
        _LIB = L
    return _LIB


def taco_strerror(status: int) -> str:
    return lib().taco_strerror(int(status)).decode()


def taco_version() -> str:
    return lib().taco_version().decode()


def taco_build_id() -> str:
    """Digest of the sources the loaded library was built from."""
    return lib().taco_build_id().decode()


def taco_default_params(block: int = 128, tau: float = 1.0, eps: float = 1e-12,
                        impl: int = TACO_IMPL_AUTO, layout: int = TACO_LAYOUT_SPLIT,
                        mode: int = TACO_MODE_FULL, fmt: int = TACO_FORMAT_E4M3) -> taco_params:
    p = taco_params()
    lib().taco_default_params(ctypes.byref(p))
    p.block, p.tau, p.eps, p.impl, p.layout, p.mode, p.format = block, tau, eps, impl, layout, mode, fmt
    return p


def taco_payload_bytes(n: int, block: int) -> int:
    return int(lib().taco_payload_bytes(n, block))


def taco_scales_bytes(n: int, block: int) -> int:
    return int(lib().taco_scales_bytes(n, block))


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    try:
        return stream.cuda_stream
    except AttributeError:
        return int(stream)


def _check(status: int, where: str):
    if status != 0:
        raise TacoError(status, where)


def _ptr_or_null(t):
    return None if t is None else t.data_ptr()


def _require(cond: bool, what: str):
    if not cond:
        raise ValueError(what)


_ESIZE = {torch.uint8: 1, torch.bfloat16: 2, torch.float32: 4}


def _check_buffer(t, dtype, min_bytes: int, name: str, device=None):
    """A tensor handed to a kernel: on the GPU, contiguous, of the expected dtype and large enough.  The C entry
    points see only a pointer, so this is where an undersized buffer is caught before a kernel writes past its end.
    One combined test on the hot path; the individual messages are produced only when it fails."""
    try:
        if (t.is_cuda and t.dtype is dtype and t.is_contiguous() and t.numel() * _ESIZE[dtype] >= min_bytes
                and (device is None or t.device == device)):
            return
    except AttributeError:
        pass
    _require(isinstance(t, torch.Tensor) and t.is_cuda, f"{name}: expected a CUDA tensor")
    _require(t.dtype == dtype, f"{name}: expected dtype {dtype}, got {t.dtype}")
    _require(t.is_contiguous(), f"{name}: must be contiguous")
    _require(t.numel() * t.element_size() >= min_bytes, f"{name}: {t.numel() * t.element_size()} bytes, {min_bytes} needed")
    _require(device is None or t.device == device, f"{name}: on {t.device}, expected {device}")


def _sizes(n: int, block: int):
    """(payload bytes, scales bytes) as taco_payload_bytes / taco_scales_bytes give them, without the two library calls."""
    if n <= 0 or n > (1 << 36) or block not in (32, 64, 128, 256, 512):
        return 0, 0
    blocks = -(-n // block)
    return blocks * block, blocks * 8


def _check_payload_args(n: int, p: "taco_params", payloads, scales, device):
    il = p.layout == TACO_LAYOUT_INTERLEAVED
    codes, sc_bytes = _sizes(n, p.block)
    _require(codes > 0, f"bad shape or block size (n = {n}, block = {p.block})")
    need = codes + (sc_bytes if il else 0)
    for i, t in enumerate(payloads):
        _check_buffer(t, torch.uint8, need, f"payload[{i}]", device)
    if not il:
        for i, t in enumerate(scales):
            _check_buffer(t, torch.float32, sc_bytes, f"scales[{i}]", device)


def _alloc_outputs(n: int, p: taco_params, device, payload, scales):
    """Split layout: (codes, scales[n_blocks, 2]).  Interleaved: (one buffer of B + 8 byte records, None)."""
    if payload is not None and (scales is not None or p.layout == TACO_LAYOUT_INTERLEAVED):
        return payload, (None if p.layout == TACO_LAYOUT_INTERLEAVED else scales)
    codes, sc_bytes = _sizes(n, p.block)
    _require(codes > 0, f"bad shape or block size (n = {n}, block = {p.block})")
    if p.layout == TACO_LAYOUT_INTERLEAVED:
        return torch.empty(codes + sc_bytes, dtype=torch.uint8, device=device), None
    if payload is None:
        payload = torch.empty(codes, dtype=torch.uint8, device=device)
    if scales is None:
        scales = torch.empty((sc_bytes // 8, 2), dtype=torch.float32, device=device)
    return payload, scales


_PTR_ARRAYS = {k: ctypes.c_void_p * k for k in range(1, TACO_MAX_K + 1)}


def _pointer_array(tensors, k):
    return _PTR_ARRAYS[max(k, 1)](*[None if t is None else t.data_ptr() for t in tensors])


def _rows_cols(shape) -> tuple:
    if len(shape) == 1:
        return 1, int(shape[0])
    rows = 1
    for d in shape[:-1]:
        rows *= int(d)
    return rows, int(shape[-1])


def taco_compress(x: torch.Tensor, params: Optional[taco_params] = None,
                  payload: Optional[torch.Tensor] = None, scales: Optional[torch.Tensor] = None,
                  stream=None):
    """Sender side of Algorithm 1.  x: contiguous CUDA bf16 tensor.  Returns (payload, scales)."""
    p = params or taco_default_params()
    _check_buffer(x, torch.bfloat16, 2, "x")
    rows, cols = _rows_cols(x.shape)
    n = rows * cols
    payload, scales = _alloc_outputs(n, p, x.device, payload, scales)
    _check_payload_args(n, p, [payload], [scales], x.device)
    st = lib().taco_compress(x.data_ptr(), rows, cols, ctypes.byref(p), payload.data_ptr(),
                             _ptr_or_null(scales), _stream_handle(stream))
    _check(st, "taco_compress")
    return payload, scales


def taco_decompress(payload: torch.Tensor, scales: torch.Tensor, shape,
                    params: Optional[taco_params] = None, out: Optional[torch.Tensor] = None,
                    stream=None) -> torch.Tensor:
    """Receiver side of Algorithm 1.  Returns a bf16 tensor of `shape`."""
    p = params or taco_default_params()
    rows, cols = _rows_cols(tuple(shape))
    _require(isinstance(payload, torch.Tensor) and payload.is_cuda, "payload: expected a CUDA tensor")
    if out is None:
        out = torch.empty(tuple(shape), dtype=torch.bfloat16, device=payload.device)
    _check_payload_args(rows * cols, p, [payload], [scales], payload.device)
    _check_buffer(out, torch.bfloat16, 2 * rows * cols, "out", payload.device)
    st = lib().taco_decompress(payload.data_ptr(), _ptr_or_null(scales), rows, cols, ctypes.byref(p),
                               out.data_ptr(), _stream_handle(stream))
    _check(st, "taco_decompress")
    return out


def taco_decompress_sum(payloads: Sequence[torch.Tensor], scales: Sequence[torch.Tensor], shape,
                        params: Optional[taco_params] = None, out: Optional[torch.Tensor] = None,
                        stream=None) -> torch.Tensor:
    """Decode k payloads and add them (fp32 accumulation, one bf16 rounding)."""
    p = params or taco_default_params()
    k = len(payloads)
    _require(1 <= k <= TACO_MAX_K, f"k = {k}: between 1 and {TACO_MAX_K} payloads")
    scales = list(scales) if scales is not None else [None] * k
    _require(k == len(scales), "as many scales as payloads")
    rows, cols = _rows_cols(tuple(shape))
    _require(isinstance(payloads[0], torch.Tensor) and payloads[0].is_cuda, "payload[0]: expected a CUDA tensor")
    if out is None:
        out = torch.empty(tuple(shape), dtype=torch.bfloat16, device=payloads[0].device)
    _check_payload_args(rows * cols, p, payloads, scales, payloads[0].device)
    _check_buffer(out, torch.bfloat16, 2 * rows * cols, "out", payloads[0].device)
    parr = _pointer_array(payloads, k)
    sarr = _pointer_array(scales, k)
    st = lib().taco_decompress_sum(parr, sarr, k, rows, cols, ctypes.byref(p), out.data_ptr(),
                                   _stream_handle(stream))
    _check(st, "taco_decompress_sum")
    return out


def taco_decompress_sum_compress(payloads: Sequence[torch.Tensor], scales: Sequence[torch.Tensor], shape,
                                 params: Optional[taco_params] = None,
                                 payload_out: Optional[torch.Tensor] = None,
                                 scales_out: Optional[torch.Tensor] = None, stream=None):
    """Decode and add k payloads, round the sum to bf16 and compress it again, in one pass."""
    p = params or taco_default_params()
    k = len(payloads)
    _require(1 <= k <= TACO_MAX_K, f"k = {k}: between 1 and {TACO_MAX_K} payloads")
    scales = list(scales) if scales is not None else [None] * k
    _require(k == len(scales), "as many scales as payloads")
    rows, cols = _rows_cols(tuple(shape))
    n = rows * cols
    _require(isinstance(payloads[0], torch.Tensor) and payloads[0].is_cuda, "payload[0]: expected a CUDA tensor")
    payload_out, scales_out = _alloc_outputs(n, p, payloads[0].device, payload_out, scales_out)
    _check_payload_args(n, p, list(payloads) + [payload_out], scales + [scales_out], payloads[0].device)
    parr = _pointer_array(payloads, k)
    sarr = _pointer_array(scales, k)
    st = lib().taco_decompress_sum_compress(parr, sarr, k, rows, cols, ctypes.byref(p), payload_out.data_ptr(),
                                            _ptr_or_null(scales_out), _stream_handle(stream))
    _check(st, "taco_decompress_sum_compress")
    return payload_out, scales_out


def taco_compress_batch(xs: Sequence[torch.Tensor], params: Optional[taco_params] = None,
                        payloads: Optional[Sequence[torch.Tensor]] = None,
                        scales: Optional[Sequence[torch.Tensor]] = None, stream=None):
    """taco_compress of up to TACO_MAX_BATCH tensors in ONE kernel.  Returns (payloads, scales) lists."""
    p = params or taco_default_params()
    count = len(xs)
    _require(1 <= count <= TACO_MAX_BATCH, f"{count} tensors: between 1 and {TACO_MAX_BATCH}")
    payloads = list(payloads) if payloads is not None else [None] * count
    scales = list(scales) if scales is not None else [None] * count
    _require(len(payloads) == count and len(scales) == count, "as many payloads and scales as tensors")
    items = (taco_compress_item * count)()
    for i, x in enumerate(xs):
        _check_buffer(x, torch.bfloat16, 2, f"x[{i}]")
        rows, cols = _rows_cols(x.shape)
        payloads[i], scales[i] = _alloc_outputs(rows * cols, p, x.device, payloads[i], scales[i])
        _check_payload_args(rows * cols, p, [payloads[i]], [scales[i]], xs[0].device)
        items[i] = taco_compress_item(x.data_ptr(), rows, cols, payloads[i].data_ptr(), _ptr_or_null(scales[i]))
    st = lib().taco_compress_batch(items, count, ctypes.byref(p), _stream_handle(stream))
    _check(st, "taco_compress_batch")
    return payloads, scales


def taco_decompress_sum_batch(payloads: Sequence[Sequence[torch.Tensor]], scales, shapes, params: Optional[taco_params] = None,
                              outs: Optional[Sequence[torch.Tensor]] = None, stream=None):
    """taco_decompress_sum of up to TACO_MAX_BATCH tensors in ONE kernel: payloads[t] (and scales[t]) are the k
    payloads of tensor t, the same k for every tensor.  Returns the list of bf16 outputs."""
    p = params or taco_default_params()
    count = len(payloads)
    _require(1 <= count <= TACO_MAX_BATCH, f"{count} tensors: between 1 and {TACO_MAX_BATCH}")
    k = len(payloads[0])
    _require(1 <= k <= TACO_MAX_K and count * k <= TACO_MAX_BATCH_PAYLOADS,
             f"k = {k}: between 1 and {TACO_MAX_K}, and at most {TACO_MAX_BATCH_PAYLOADS} payloads in all")
    scales = [list(s) if s is not None else [None] * k for s in (scales if scales is not None else [None] * count)]
    outs = list(outs) if outs is not None else [None] * count
    _require(len(scales) == count and len(shapes) == count and len(outs) == count, "one scales list, shape and output per tensor")
    items = (taco_decode_item * count)()
    keep = []
    dev = payloads[0][0].device
    for t in range(count):
        _require(len(payloads[t]) == k and len(scales[t]) == k, "every tensor needs the same number of payloads")
        rows, cols = _rows_cols(tuple(shapes[t]))
        if outs[t] is None:
            outs[t] = torch.empty(tuple(shapes[t]), dtype=torch.bfloat16, device=dev)
        _check_payload_args(rows * cols, p, payloads[t], scales[t], dev)
        _check_buffer(outs[t], torch.bfloat16, 2 * rows * cols, f"out[{t}]", dev)
        parr, sarr = _pointer_array(payloads[t], k), _pointer_array(scales[t], k)
        keep.append((parr, sarr))
        items[t] = taco_decode_item(ctypes.cast(parr, ctypes.POINTER(ctypes.c_void_p)),
                                    ctypes.cast(sarr, ctypes.POINTER(ctypes.c_void_p)), rows, cols, outs[t].data_ptr())
    st = lib().taco_decompress_sum_batch(items, count, k, ctypes.byref(p), _stream_handle(stream))
    _check(st, "taco_decompress_sum_batch")
    return outs


def taco_decompress_sum_compress_batch(payloads: Sequence[Sequence[torch.Tensor]], scales, shapes,
                                       params: Optional[taco_params] = None, payloads_out=None, scales_out=None, stream=None):
    """taco_decompress_sum_compress of up to TACO_MAX_BATCH tensors in ONE kernel (same k for every tensor).
    Returns (payloads_out, scales_out) lists."""
    p = params or taco_default_params()
    count = len(payloads)
    _require(1 <= count <= TACO_MAX_BATCH, f"{count} tensors: between 1 and {TACO_MAX_BATCH}")
    k = len(payloads[0])
    _require(1 <= k <= TACO_MAX_K and count * k <= TACO_MAX_BATCH_PAYLOADS,
             f"k = {k}: between 1 and {TACO_MAX_K}, and at most {TACO_MAX_BATCH_PAYLOADS} payloads in all")
    scales = [list(s) if s is not None else [None] * k for s in (scales if scales is not None else [None] * count)]
    payloads_out = list(payloads_out) if payloads_out is not None else [None] * count
    scales_out = list(scales_out) if scales_out is not None else [None] * count
    _require(len(scales) == count and len(shapes) == count and len(payloads_out) == count and len(scales_out) == count,
             "one scales list, shape and output pair per tensor")
    items = (taco_recompress_item * count)()
    keep = []
    dev = payloads[0][0].device
    for t in range(count):
        _require(len(payloads[t]) == k and len(scales[t]) == k, "every tensor needs the same number of payloads")
        rows, cols = _rows_cols(tuple(shapes[t]))
        _check_payload_args(rows * cols, p, payloads[t], scales[t], dev)
        payloads_out[t], scales_out[t] = _alloc_outputs(rows * cols, p, dev, payloads_out[t], scales_out[t])
        _check_payload_args(rows * cols, p, [payloads_out[t]], [scales_out[t]], dev)
        parr, sarr = _pointer_array(payloads[t], k), _pointer_array(scales[t], k)
        keep.append((parr, sarr))
        items[t] = taco_recompress_item(ctypes.cast(parr, ctypes.POINTER(ctypes.c_void_p)),
                                        ctypes.cast(sarr, ctypes.POINTER(ctypes.c_void_p)), rows, cols,
                                        payloads_out[t].data_ptr(), _ptr_or_null(scales_out[t]))
    st = lib().taco_decompress_sum_compress_batch(items, count, k, ctypes.byref(p), _stream_handle(stream))
    _check(st, "taco_decompress_sum_compress_batch")
    return payloads_out, scales_out


def taco_debug_cvt_e4m3(values: torch.Tensor, stream=None) -> torch.Tensor:
    """Hardware float32 -> E4M3 conversion of a CUDA float tensor (diagnostic)."""
    _check_buffer(values, torch.float32, 4, "values")
    out = torch.empty(values.numel(), dtype=torch.uint8, device=values.device)
    st = lib().taco_debug_cvt_e4m3(values.data_ptr(), values.numel(), out.data_ptr(),
                                   _stream_handle(stream))
    _check(st, "taco_debug_cvt_e4m3")
    return out


def taco_debug_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> torch.Tensor:
    """Plain device copy of src into dst (same byte size, a multiple of 16): bandwidth yardstick."""
    _require(isinstance(src, torch.Tensor) and isinstance(dst, torch.Tensor) and src.is_cuda and dst.is_cuda
             and src.is_contiguous() and dst.is_contiguous(), "src, dst: contiguous CUDA tensors")
    nbytes = src.numel() * src.element_size()
    _require(nbytes == dst.numel() * dst.element_size(), "src and dst differ in size")
    st = lib().taco_debug_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_handle(stream))
    _check(st, "taco_debug_copy")
    return dst


def taco_debug_traffic(srcs: Sequence[torch.Tensor], src_chunks: int, dst: torch.Tensor, dst_chunks: int,
                       n_tiles: int, stream=None) -> torch.Tensor:
    """Memory-only stand-in for the operator: per tile reads src_chunks 16-byte words from every source and
    writes dst_chunks words to dst (bandwidth yardstick for that mix of reads and writes)."""
    k = len(srcs)
    _require(n_tiles >= 1 and 1 <= src_chunks <= 256 and 1 <= dst_chunks <= 256, "chunk counts 1..256, n_tiles >= 1")
    for i, t in enumerate(srcs):
        _require(isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()
                 and t.numel() * t.element_size() >= n_tiles * src_chunks * 16, f"srcs[{i}]: contiguous CUDA tensor of "
                 f"at least {n_tiles * src_chunks * 16} bytes")
    _require(isinstance(dst, torch.Tensor) and dst.is_cuda and dst.is_contiguous()
             and dst.numel() * dst.element_size() >= n_tiles * dst_chunks * 16, f"dst: contiguous CUDA tensor of at least "
             f"{n_tiles * dst_chunks * 16} bytes")
    st = lib().taco_debug_traffic(_pointer_array(srcs, k), k, src_chunks, dst.data_ptr(), dst_chunks, n_tiles,
                                  _stream_handle(stream))
    _check(st, "taco_debug_traffic")
    return dst


class PreparedCall:
    """An entry point with its arguments checked and marshalled once, for loops that launch the same call on
    the same buffers many times (static activations buffers, serving loops): `plan(stream)` then costs little more
    than the bare library call.  The plan keeps references to its tensors, so their storage stays alive; their
    CONTENTS may change between launches, their addresses may not."""

    def __init__(self, fn, args, keep, where):
        self._fn, self._args, self._keep, self._where = fn, args, keep, where

    def __call__(self, stream=None):
        st = self._fn(*self._args, _stream_handle(stream))
        if st != 0:
            raise TacoError(st, self._where)


def prepare_compress(x, params: Optional[taco_params], payload, scales=None) -> PreparedCall:
    """taco_compress(x, params, payload, scales) as a PreparedCall; the outputs must be given."""
    p = params or taco_default_params()
    _check_buffer(x, torch.bfloat16, 2, "x")
    rows, cols = _rows_cols(x.shape)
    _check_payload_args(rows * cols, p, [payload], [scales], x.device)
    args = (x.data_ptr(), rows, cols, ctypes.byref(p), payload.data_ptr(), _ptr_or_null(scales))
    return PreparedCall(lib().taco_compress, args, (x, p, payload, scales), "taco_compress")


def prepare_decompress_sum(payloads, scales, shape, params: Optional[taco_params], out) -> PreparedCall:
    """taco_decompress_sum(payloads, scales, shape, params, out) as a PreparedCall (k = 1: taco_decompress)."""
    p = params or taco_default_params()
    k = len(payloads)
    _require(1 <= k <= TACO_MAX_K, f"k = {k}: between 1 and {TACO_MAX_K} payloads")
    scales = list(scales) if scales is not None else [None] * k
    _require(k == len(scales), "as many scales as payloads")
    rows, cols = _rows_cols(tuple(shape))
    _require(isinstance(payloads[0], torch.Tensor) and payloads[0].is_cuda, "payload[0]: expected a CUDA tensor")
    _check_payload_args(rows * cols, p, payloads, scales, payloads[0].device)
    _check_buffer(out, torch.bfloat16, 2 * rows * cols, "out", payloads[0].device)
    parr, sarr = _pointer_array(payloads, k), _pointer_array(scales, k)
    args = (parr, sarr, k, rows, cols, ctypes.byref(p), out.data_ptr())
    return PreparedCall(lib().taco_decompress_sum, args, (list(payloads), scales, p, out, parr, sarr), "taco_decompress_sum")


def prepare_decompress_sum_compress(payloads, scales, shape, params: Optional[taco_params], payload_out,
                                    scales_out=None) -> PreparedCall:
    """taco_decompress_sum_compress(...) as a PreparedCall; the outputs must be given."""
    p = params or taco_default_params()
    k = len(payloads)
    _require(1 <= k <= TACO_MAX_K, f"k = {k}: between 1 and {TACO_MAX_K} payloads")
    scales = list(scales) if scales is not None else [None] * k
    _require(k == len(scales), "as many scales as payloads")
    rows, cols = _rows_cols(tuple(shape))
    _require(isinstance(payloads[0], torch.Tensor) and payloads[0].is_cuda, "payload[0]: expected a CUDA tensor")
    _check_payload_args(rows * cols, p, list(payloads) + [payload_out], scales + [scales_out], payloads[0].device)
    parr, sarr = _pointer_array(payloads, k), _pointer_array(scales, k)
    args = (parr, sarr, k, rows, cols, ctypes.byref(p), payload_out.data_ptr(), _ptr_or_null(scales_out))
    return PreparedCall(lib().taco_decompress_sum_compress, args,
                        (list(payloads), scales, p, payload_out, scales_out, parr, sarr), "taco_decompress_sum_compress")
