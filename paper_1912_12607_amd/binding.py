"""Thin ctypes binding of csrc/libint8t.so: same names as the C ABI (include/int8t.h), argument
marshalling only.  Tensors are torch CUDA(ROCm) tensors used purely as device memory; every step
of the path runs inside the library's HIP kernels.  There is no CPU fallback: if the library is
missing or fails to load, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libint8t.so")

OK = 0
ROUND_NEAREST_EVEN, ROUND_STOCHASTIC = 0, 1
ACT, WGT, ACT_PLANAR, WGT_PLANAR = 0, 1, 2, 3
OP_QUANTIZE, OP_DSGC, OP_CONV_FWD, OP_CONV_BWD_DATA, OP_CONV_BWD_WEIGHT = range(5)
(VARIANT_AUTO, VARIANT_BAND, VARIANT_TILE, VARIANT_TILE_SPLIT, VARIANT_WIDE128, VARIANT_WIDE256,
 VARIANT_WGRAD_FEWER, VARIANT_WGRAD_MORE, VARIANT_WGRAD_IMAGES, VARIANT_WGRAD_LINES, VARIANT_WIDE_SQ128,
 VARIANT_WIDE_SQ128_DEEP, VARIANT_WIDE_128X64, VARIANT_WIDE_CELLS) = range(14)
VARIANT_NAMES = ["auto", "band", "tile", "tile_split", "wide128", "wide256", "wgrad_fewer", "wgrad_more", "wgrad_images",
                 "wgrad_lines", "wide_sq128", "wide_sq128_deep", "wide_128x64", "wide_cells"]
MAX_CANDIDATES = 64
MAX_BATCH = 8

EXPORTS = ["int8t_status_string", "int8t_code_bytes", "int8t_unpack_codes", "int8t_workspace_bytes",
           "int8t_quantize_workspace_bytes", "int8t_quantize", "int8t_quantize_batch_workspace_bytes",
           "int8t_quantize_batch", "int8t_quantize_batch_prepare", "int8t_dsgc_clip", "int8t_dsgc_clip_static", "int8t_dsgc_prepare", "int8t_dsgc_search", "int8t_conv_fwd", "int8t_conv_fwd_fused",
           "int8t_conv_bwd_data", "int8t_conv_bwd_weight", "int8t_dclr_scale",
           "int8t_conv_variant_ok", "int8t_conv_select_variant", "int8t_conv_selected_variant",
           "int8t_profile_start", "int8t_profile_start_sampled", "int8t_profile_stop", "int8t_profile_mfma_ceiling"]


class KernelTime(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int), ("total_ms", C.c_double)]


class QuantizeItem(C.Structure):
    _fields_ = [("x_dev", C.c_void_p), ("dims", C.c_int * 4), ("kind", C.c_int), ("clip_dev", C.c_void_p),
                ("q_dev", C.c_void_p), ("scale_dev", C.c_void_p), ("mode", C.c_int), ("seed", C.c_uint64)]


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "groups")]


def make_desc(N, Cin, H, W, K, R, S, stride=(1, 1), pad=(0, 0), groups=1) -> ConvDesc:
    return ConvDesc(N, Cin, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1], groups)


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_1912_12607_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    L = C.CDLL(LIB_PATH)
    vp, sz, u64, i32 = C.c_void_p, C.c_size_t, C.c_uint64, C.c_int
    dims = C.POINTER(C.c_int)
    dp = C.POINTER(ConvDesc)
    L.int8t_status_string.restype = C.c_char_p
    L.int8t_status_string.argtypes = [i32]
    L.int8t_code_bytes.restype = sz
    L.int8t_code_bytes.argtypes = [dims, i32]
    L.int8t_unpack_codes.restype = i32
    L.int8t_unpack_codes.argtypes = [vp, dims, i32, i32, vp, C.POINTER(sz)]
    L.int8t_workspace_bytes.restype = sz
    L.int8t_workspace_bytes.argtypes = [i32, dp, sz, i32]
    L.int8t_quantize_workspace_bytes.restype = sz
    L.int8t_quantize_workspace_bytes.argtypes = [dims, i32]
    L.int8t_quantize.restype = i32
    L.int8t_quantize.argtypes = [vp, dims, i32, vp, i32, u64, vp, vp, vp, vp, sz, vp]
    L.int8t_quantize_batch_workspace_bytes.restype = sz
    L.int8t_quantize_batch_workspace_bytes.argtypes = [i32, C.POINTER(QuantizeItem)]
    L.int8t_quantize_batch.restype = i32
    L.int8t_quantize_batch.argtypes = [i32, C.POINTER(QuantizeItem), vp, sz, vp]
    L.int8t_quantize_batch_prepare.restype = i32
    L.int8t_quantize_batch_prepare.argtypes = [i32, C.POINTER(QuantizeItem), vp, sz, vp, sz, vp, sz, vp]
    L.int8t_dsgc_clip.restype = i32
    L.int8t_dsgc_clip.argtypes = [vp, sz, vp, i32, i32, u64, vp, vp, vp, vp, sz, vp]
    L.int8t_dsgc_clip_static.restype = i32
    L.int8t_dsgc_clip_static.argtypes = [vp, sz, vp, i32, i32, u64, vp, vp, vp, vp]
    L.int8t_dsgc_search.restype = i32
    L.int8t_dsgc_search.argtypes = [vp, sz, vp, i32, i32, u64, vp, vp, vp, vp, sz, vp]
    L.int8t_dsgc_prepare.restype = i32
    L.int8t_dsgc_prepare.argtypes = [vp, sz, vp, sz, vp]
    for name in ("int8t_conv_fwd", "int8t_conv_bwd_data", "int8t_conv_bwd_weight"):
        f = getattr(L, name)
        f.restype = i32
        f.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.int8t_conv_fwd_fused.restype = i32
    L.int8t_conv_fwd_fused.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.int8t_conv_variant_ok.restype = i32
    L.int8t_conv_variant_ok.argtypes = [i32, dp, i32]
    L.int8t_conv_select_variant.restype = i32
    L.int8t_conv_select_variant.argtypes = [i32, dp, i32]
    L.int8t_conv_selected_variant.restype = i32
    L.int8t_conv_selected_variant.argtypes = [i32, dp]
    L.int8t_dclr_scale.restype = C.c_double
    L.int8t_dclr_scale.argtypes = [C.c_double, C.c_double, C.c_double]
    L.int8t_profile_start.restype = i32
    L.int8t_profile_start.argtypes = [C.c_char_p]
    L.int8t_profile_start_sampled.restype = i32
    L.int8t_profile_start_sampled.argtypes = [C.c_char_p, C.c_int]
    L.int8t_profile_mfma_ceiling.restype = i32
    L.int8t_profile_mfma_ceiling.argtypes = [i32, i32, i32, C.POINTER(C.c_double), C.POINTER(C.c_double), vp, vp]
    L.int8t_profile_stop.restype = i32
    L.int8t_profile_stop.argtypes = [C.POINTER(KernelTime), i32, C.POINTER(i32)]
    return L


lib = _load()


class Int8tError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"int8t status {status}: {lib.int8t_status_string(status).decode()}")


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def _dims(d):
    return (C.c_int * 4)(*[int(v) for v in d])


def _check(status: int):
    if status != OK:
        raise Int8tError(status)


def bind(func, *cargs):
    """A call with its arguments marshalled once: bind(lib.int8t_conv_fwd, byref(desc), _ptr(xq), ...)
    returns f(stream_pointer) that appends the stream and checks the status.  For callers that issue the
    same call on the same buffers many times (a training step): converting a dozen tensors to pointers
    costs more host time per call than the launch itself."""
    def call(stream_ptr):
        status = func(*cargs, stream_ptr)
        if status != OK:
            raise Int8tError(status)
    return call


def stream_pointer(stream=None):
    return _stream(stream)


def int8t_status_string(status: int) -> str:
    return lib.int8t_status_string(status).decode()


def int8t_code_bytes(dims, kind: int) -> int:
    return int(lib.int8t_code_bytes(_dims(dims), kind))


def int8t_unpack_codes(codes_host, dims, kind: int, copy: int = 0):
    """Host numpy int8 array in the library's layout -> (codes in logical order, shape dims; number of
    non-zero padding bytes).  The loops run inside the library (host code)."""
    import numpy as np
    src = np.ascontiguousarray(codes_host, dtype=np.int8).reshape(-1)
    assert src.size >= int8t_code_bytes(dims, kind), "code tensor shorter than int8t_code_bytes()"
    out = np.empty(tuple(int(v) for v in dims), dtype=np.int8)
    bad = C.c_size_t(0)
    _check(lib.int8t_unpack_codes(src.ctypes.data_as(C.c_void_p), _dims(dims), kind, copy,
                                  out.ctypes.data_as(C.c_void_p), C.byref(bad)))
    return out, int(bad.value)


def int8t_workspace_bytes(op: int, desc: ConvDesc | None = None, n: int = 0, n_cand: int = 0) -> int:
    return int(lib.int8t_workspace_bytes(op, C.byref(desc) if desc is not None else None, n, n_cand))


def int8t_quantize_workspace_bytes(dims, kind: int) -> int:
    return int(lib.int8t_quantize_workspace_bytes(_dims(dims), kind))


def int8t_quantize(x, dims, kind, clip, mode, seed, q, scale, deviation=None, ws=None, stream=None):
    _check(lib.int8t_quantize(_ptr(x), _dims(dims), kind, _ptr(clip), mode, seed, _ptr(q), _ptr(scale),
                              _ptr(deviation), _ptr(ws), _nbytes(ws), _stream(stream)))


def _items(items):
    """[(x, dims, kind, clip or None, q, scale[, mode, seed]), ...] -> ctypes array (round to nearest
    unless mode and seed are given); the tensors must stay alive until the call returns."""
    arr = (QuantizeItem * len(items))()
    for a, it in zip(arr, items):
        x, dims, kind, clip, q, scale = it[:6]
        a.mode, a.seed = (int(it[6]), int(it[7])) if len(it) > 6 else (ROUND_NEAREST_EVEN, 0)
        a.x_dev, a.kind, a.clip_dev, a.q_dev, a.scale_dev = _ptr(x), kind, _ptr(clip), _ptr(q), _ptr(scale)
        for j in range(4):
            a.dims[j] = int(dims[j])
    return arr


def int8t_quantize_batch_workspace_bytes(items) -> int:
    return int(lib.int8t_quantize_batch_workspace_bytes(len(items), _items(items)))


def int8t_quantize_batch(items, ws=None, stream=None):
    _check(lib.int8t_quantize_batch(len(items), _items(items), _ptr(ws), _nbytes(ws), _stream(stream)))


def int8t_quantize_batch_prepare(items, ws, g, n, dsgc_ws, stream=None):
    _check(lib.int8t_quantize_batch_prepare(len(items), _items(items), _ptr(ws), _nbytes(ws), _ptr(g), n, _ptr(dsgc_ws),
                                            _nbytes(dsgc_ws), _stream(stream)))


def int8t_dsgc_clip(g, n, ratios, n_cand, mode, seed, clip, deviation, deviation_all=None, ws=None,
                    stream=None):
    _check(lib.int8t_dsgc_clip(_ptr(g), n, _ptr(ratios), n_cand, mode, seed, _ptr(clip), _ptr(deviation),
                               _ptr(deviation_all), _ptr(ws), _nbytes(ws), _stream(stream)))


def int8t_dsgc_clip_static(g, n, ratios, n_cand, mode, seed, clip, deviation, deviation_all=None, stream=None):
    _check(lib.int8t_dsgc_clip_static(_ptr(g), n, _ptr(ratios), n_cand, mode, seed, _ptr(clip), _ptr(deviation),
                                      _ptr(deviation_all), _stream(stream)))


def int8t_dsgc_prepare(g, n, ws, stream=None):
    _check(lib.int8t_dsgc_prepare(_ptr(g), n, _ptr(ws), _nbytes(ws), _stream(stream)))


def int8t_dsgc_search(g, n, ratios, n_cand, mode, seed, clip, deviation, deviation_all=None, ws=None,
                      stream=None):
    _check(lib.int8t_dsgc_search(_ptr(g), n, _ptr(ratios), n_cand, mode, seed, _ptr(clip), _ptr(deviation),
                                 _ptr(deviation_all), _ptr(ws), _nbytes(ws), _stream(stream)))


def int8t_conv_fwd(desc, xq, sx, wq, sw, y, acc=None, ws=None, stream=None):
    _check(lib.int8t_conv_fwd(C.byref(desc), _ptr(xq), _ptr(sx), _ptr(wq), _ptr(sw), _ptr(y), _ptr(acc),
                              _ptr(ws), _nbytes(ws), _stream(stream)))


def int8t_conv_fwd_fused(desc, x, clip, wq, sw, y, acc=None, xq=None, sx=None, ws=None, stream=None):
    _check(lib.int8t_conv_fwd_fused(C.byref(desc), _ptr(x), _ptr(clip), _ptr(wq), _ptr(sw), _ptr(y), _ptr(acc),
                                    _ptr(xq), _ptr(sx), _ptr(ws), _nbytes(ws), _stream(stream)))


def int8t_conv_bwd_data(desc, dyq, sdy, wq, sw, dx, acc=None, ws=None, stream=None):
    _check(lib.int8t_conv_bwd_data(C.byref(desc), _ptr(dyq), _ptr(sdy), _ptr(wq), _ptr(sw), _ptr(dx),
                                   _ptr(acc), _ptr(ws), _nbytes(ws), _stream(stream)))


def int8t_conv_bwd_weight(desc, xq, sx, dyq, sdy, dw, acc=None, ws=None, stream=None):
    _check(lib.int8t_conv_bwd_weight(C.byref(desc), _ptr(xq), _ptr(sx), _ptr(dyq), _ptr(sdy), _ptr(dw),
                                     _ptr(acc), _ptr(ws), _nbytes(ws), _stream(stream)))


def int8t_conv_variant_ok(op: int, desc: ConvDesc, variant: int) -> bool:
    return bool(lib.int8t_conv_variant_ok(op, C.byref(desc), variant))


def int8t_conv_select_variant(op: int, desc: ConvDesc, variant: int):
    _check(lib.int8t_conv_select_variant(op, C.byref(desc), variant))


def int8t_conv_selected_variant(op: int, desc: ConvDesc) -> int:
    return int(lib.int8t_conv_selected_variant(op, C.byref(desc)))


def int8t_dclr_scale(d_c: float, alpha: float = 20.0, beta: float = 0.1) -> float:
    return float(lib.int8t_dclr_scale(d_c, alpha, beta))


def int8t_profile_start(kernel: str | None = None):
    _check(lib.int8t_profile_start(None if kernel is None else kernel.encode()))


def int8t_profile_start_sampled(kernel: str | None, every: int):
    _check(lib.int8t_profile_start_sampled(None if kernel is None else kernel.encode(), int(every)))


def int8t_profile_stop() -> dict:
    """{kernel name: (launches, total milliseconds)} of the launches since int8t_profile_start."""
    buf = (KernelTime * 32)()
    n = C.c_int(0)
    _check(lib.int8t_profile_stop(buf, 32, C.byref(n)))
    return {buf[i].name.decode(): (int(buf[i].launches), float(buf[i].total_ms)) for i in range(min(n.value, 32))}


def int8t_profile_mfma_ceiling(random_operands: bool, lds_reads: bool, iters: int = 20000, stream=None):
    """(int8 TOP/s, shader clock in GHz) of the MFMA loop described in include/int8t.h."""
    ws = torch.zeros(8, dtype=torch.int64, device="cuda")
    tops, ghz = C.c_double(0), C.c_double(0)
    _check(lib.int8t_profile_mfma_ceiling(int(bool(random_operands)), int(bool(lds_reads)), int(iters), C.byref(tops), C.byref(ghz),
                                          _ptr(ws), _stream(stream)))
    return tops.value, ghz.value
