"""int8t oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

ctypes front end of ``int8t_oracle.c``: the plain CPU statement of the paper's
INT8 training convolution path (Eq.1-3 quantizer, Eq.6 direction deviation and
the clip search built on it, Eq.7 LR scaling, the three integer convolutions of
Sec.3.4).  Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import this package.  It imports nothing from the GPU
package and the GPU package imports nothing from here.

All tensors are numpy arrays in *logical* order: activations / gradients
N,C,H,W; weights K,C/g,R,S.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "int8t_oracle.c")
_LIB = os.path.join(_HERE, "libint8t_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fused multiply-add, OpenMP on outer loops)."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "groups")]


def make_desc(N, Cin, H, W, K, R, S, stride=(1, 1), pad=(0, 0), groups=1) -> ConvDesc:
    return ConvDesc(N, Cin, H, W, K, R, S, stride[0], stride[1], pad[0], pad[1], groups)


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, u64, sz = C.c_void_p, C.c_uint64, C.c_size_t
        L.orc_absmax.restype = C.c_float
        L.orc_absmax.argtypes = [vp, sz]
        L.orc_rng24.restype = C.c_uint32
        L.orc_rng24.argtypes = [u64, u64]
        L.orc_scale.restype = C.c_float
        L.orc_scale.argtypes = [C.c_float]
        L.orc_quantize.restype = None
        L.orc_quantize.argtypes = [vp, sz, C.c_float, C.c_int, u64, vp, vp]
        L.orc_deviation.restype = C.c_double
        L.orc_deviation.argtypes = [vp, vp, C.c_float, sz]
        L.orc_dsgc.restype = C.c_float
        L.orc_dsgc.argtypes = [vp, sz, vp, C.c_int, C.c_int, u64, vp, vp, vp]
        L.orc_dclr.restype = C.c_double
        L.orc_dclr.argtypes = [C.c_double, C.c_double, C.c_double]
        dp = C.POINTER(ConvDesc)
        L.orc_out_h.restype = C.c_int
        L.orc_out_h.argtypes = [dp]
        L.orc_out_w.restype = C.c_int
        L.orc_out_w.argtypes = [dp]
        for name in ("orc_conv_fwd", "orc_conv_bwd_data", "orc_conv_bwd_weight"):
            f = getattr(L, name)
            f.restype = None
            f.argtypes = [dp, vp, vp, vp]
            g = getattr(L, name + "_at")
            g.restype = C.c_int64
            g.argtypes = [dp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_wrap32.restype = None
        L.orc_wrap32.argtypes = [vp, sz, vp, vp]
        L.orc_dequant.restype = None
        L.orc_dequant.argtypes = [vp, sz, C.c_float, C.c_float, vp]
        _lib = L
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i8(a):
    return np.ascontiguousarray(a, dtype=np.int8)


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


ROUND_NEAREST_EVEN = 0
ROUND_STOCHASTIC = 1


def absmax(x) -> np.float32:
    x = _f32(x)
    return np.float32(lib().orc_absmax(_p(x), x.size))


def rng24(seed: int, index: int) -> int:
    return int(lib().orc_rng24(seed, index))


def scale(c) -> np.float32:
    return np.float32(lib().orc_scale(C.c_float(float(c))))


def quantize(x, c=None, mode=ROUND_NEAREST_EVEN, seed=0):
    """Eq.1 (+Eq.3 when mode is stochastic). Returns (codes int8 same shape, scale fp32)."""
    x = _f32(x)
    if c is None:
        c = absmax(x)
    q = np.empty(x.shape, dtype=np.int8)
    s = C.c_float(0)
    lib().orc_quantize(_p(x), x.size, C.c_float(float(c)), int(mode), int(seed), _p(q), C.byref(s))
    return q, np.float32(s.value)


def deviation(g, q, s) -> float:
    """Eq.6 between g and q*s."""
    g = _f32(g)
    q = _i8(q)
    assert g.size == q.size
    return float(lib().orc_deviation(_p(g), _p(q), C.c_float(float(s)), g.size))


def dsgc(g, ratios, mode=ROUND_STOCHASTIC, seed=0):
    """Brute-force clip search. Returns dict(absmax, clips[J], dev[J], jstar, clip, deviation)."""
    g = _f32(g)
    ratios = _f32(ratios)
    J = ratios.size
    clips = np.empty(J, dtype=np.float32)
    dev = np.empty(J, dtype=np.float64)
    js = C.c_int(0)
    m = lib().orc_dsgc(_p(g), g.size, _p(ratios), J, int(mode), int(seed), _p(clips), _p(dev), C.byref(js))
    j = js.value
    return dict(absmax=np.float32(m), clips=clips, dev=dev, jstar=j, clip=clips[j], deviation=float(dev[j]))


def dclr(d, alpha=20.0, beta=0.1) -> float:
    return float(lib().orc_dclr(float(d), float(alpha), float(beta)))


def out_hw(desc: ConvDesc):
    return lib().orc_out_h(C.byref(desc)), lib().orc_out_w(C.byref(desc))


def conv_fwd(desc: ConvDesc, xq, wq) -> np.ndarray:
    xq, wq = _i8(xq), _i8(wq)
    P, Q = out_hw(desc)
    assert xq.shape == (desc.N, desc.C, desc.H, desc.W)
    assert wq.shape == (desc.K, desc.C // desc.groups, desc.R, desc.S)
    acc = np.empty((desc.N, desc.K, P, Q), dtype=np.int64)
    lib().orc_conv_fwd(C.byref(desc), _p(xq), _p(wq), _p(acc))
    return acc


def conv_bwd_data(desc: ConvDesc, dyq, wq) -> np.ndarray:
    dyq, wq = _i8(dyq), _i8(wq)
    P, Q = out_hw(desc)
    assert dyq.shape == (desc.N, desc.K, P, Q)
    assert wq.shape == (desc.K, desc.C // desc.groups, desc.R, desc.S)
    acc = np.empty((desc.N, desc.C, desc.H, desc.W), dtype=np.int64)
    lib().orc_conv_bwd_data(C.byref(desc), _p(dyq), _p(wq), _p(acc))
    return acc


def conv_bwd_weight(desc: ConvDesc, xq, dyq) -> np.ndarray:
    xq, dyq = _i8(xq), _i8(dyq)
    P, Q = out_hw(desc)
    assert xq.shape == (desc.N, desc.C, desc.H, desc.W)
    assert dyq.shape == (desc.N, desc.K, P, Q)
    acc = np.empty((desc.K, desc.C // desc.groups, desc.R, desc.S), dtype=np.int64)
    lib().orc_conv_bwd_weight(C.byref(desc), _p(xq), _p(dyq), _p(acc))
    return acc


def conv_fwd_at(desc, xq, wq, n, k, p, q) -> int:
    return int(lib().orc_conv_fwd_at(C.byref(desc), _p(xq), _p(wq), n, k, p, q))


def conv_bwd_data_at(desc, dyq, wq, n, c, h, w) -> int:
    return int(lib().orc_conv_bwd_data_at(C.byref(desc), _p(dyq), _p(wq), n, c, h, w))


def conv_bwd_weight_at(desc, xq, dyq, k, c, r, s) -> int:
    return int(lib().orc_conv_bwd_weight_at(C.byref(desc), _p(xq), _p(dyq), k, c, r, s))


def wrap32(acc64):
    """Low 32 bits (two's complement) of exact sums, and how many left the int32 range."""
    a = np.ascontiguousarray(acc64, dtype=np.int64)
    out = np.empty(a.shape, dtype=np.int32)
    ov = C.c_int64(0)
    lib().orc_wrap32(_p(a), a.size, _p(out), C.byref(ov))
    return out, int(ov.value)


def dequant(acc32, sa, sb) -> np.ndarray:
    """Eq.2 epilogue: acc * s_a * s_b in double, rounded once to fp32."""
    a = np.ascontiguousarray(acc32, dtype=np.int32)
    out = np.empty(a.shape, dtype=np.float32)
    lib().orc_dequant(_p(a), a.size, C.c_float(float(sa)), C.c_float(float(sb)), _p(out))
    return out
