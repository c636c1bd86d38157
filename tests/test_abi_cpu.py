"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every function the
header declares, sizes layouts and scratch as documented, and rejects bad arguments before any
launch."""
import ctypes as C
import math
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1912_12607_amd", "csrc", "libint8t.so")
HDR = os.path.join(ROOT, "include", "int8t.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_1912_12607_amd import build
        build.build(force=False)
    L = C.CDLL(LIB)
    L.int8t_code_bytes.restype = C.c_size_t
    L.int8t_workspace_bytes.restype = C.c_size_t
    L.int8t_quantize_workspace_bytes.restype = C.c_size_t
    L.int8t_status_string.restype = C.c_char_p
    L.int8t_dclr_scale.restype = C.c_double
    L.int8t_dclr_scale.argtypes = [C.c_double] * 3
    return L


class Desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("N", "C", "H", "W", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "groups")]


def dims(*v):
    return (C.c_int * 4)(*v)


def test_every_declared_symbol_is_exported(lib):
    text = open(HDR).read()
    names = set(re.findall(r"\b(int8t_[a-z_0-9]+)\s*\(", text))
    assert {"int8t_quantize", "int8t_dsgc_clip", "int8t_conv_fwd", "int8t_conv_bwd_data",
            "int8t_conv_bwd_weight"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_binding_names_match_header():
    text = open(os.path.join(ROOT, "paper_1912_12607_amd", "binding.py")).read()
    hdr = set(re.findall(r"\b(int8t_[a-z_0-9]+)\s*\(", open(HDR).read()))
    for n in hdr:
        assert f"def {n}(" in text, n


def test_code_bytes(lib):
    assert lib.int8t_code_bytes(dims(2, 16, 16, 16), 0) == 2 * 16 * 16 * 16
    assert lib.int8t_code_bytes(dims(64, 24, 56, 56), 0) == 64 * 56 * 56 * 32      # C padded to 32
    assert lib.int8t_code_bytes(dims(64, 24, 56, 56), 2) == 64 * 24 * 56 * 56      # planar
    k, c, r, s = 70, 33, 3, 3
    n1 = k * r * s * 48
    assert lib.int8t_code_bytes(dims(k, c, r, s), 1) == ((n1 + 255) // 256) * 256 + c * r * s * 80
    assert lib.int8t_code_bytes(dims(k, c, r, s), 3) == k * c * r * s
    assert lib.int8t_code_bytes(dims(0, 1, 1, 1), 0) == 0
    assert lib.int8t_code_bytes(dims(2, 2, 2, 2), 7) == 0


def test_workspace_sizes(lib):
    assert lib.int8t_quantize_workspace_bytes(dims(2, 16, 16, 16), 0) >= 4096 + 8 * 24
    assert lib.int8t_quantize_workspace_bytes(dims(2, 16, 16, -1), 0) == 0
    # clip search: absmax partials + 32 accumulator sets x 64 candidates x 3 words + sum-of-squares partials
    assert lib.int8t_workspace_bytes(1, None, C.c_size_t(1 << 20), 32) >= 1024 * 4 + 32 * 64 * 3 * 8 + 8 + 1024 * 8
    d = Desc(64, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1)
    assert lib.int8t_workspace_bytes(4, C.byref(d), C.c_size_t(0), 0) >= 64 * 9 * 64 * 4
    assert lib.int8t_workspace_bytes(2, C.byref(d), C.c_size_t(0), 0) == 0
    # forward / backward-data of a layer with few output tiles: optional scratch for a split reduction,
    # a whole number of int32 result copies
    few = Desc(64, 768, 17, 17, 192, 3, 3, 2, 2, 0, 0, 1)
    nf = lib.int8t_workspace_bytes(2, C.byref(few), C.c_size_t(0), 0)
    assert nf >= 2 * 64 * 192 * 8 * 8 * 4 and nf % (64 * 192 * 8 * 8 * 4) == 0
    bad = Desc(64, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 2)     # grouped but not depthwise
    assert lib.int8t_workspace_bytes(4, C.byref(bad), C.c_size_t(0), 0) == 0


def test_dclr_scale_golden_table(lib):
    # the library's host function against the fixture written from Eq.7 (tests/golden/dclr_eq7.txt)
    n = 0
    for line in open(os.path.join(ROOT, "tests", "golden", "dclr_eq7.txt")):
        if line.startswith("#"):
            continue
        alpha, beta, d, phi = (float(v) for v in line.split())
        assert lib.int8t_dclr_scale(d, alpha, beta) == pytest.approx(phi, rel=1e-15)
        n += 1
    assert n == 36


def test_dclr_scale_eq7(lib):
    assert lib.int8t_dclr_scale(0.0, 20.0, 0.1) == 1.0
    assert lib.int8t_dclr_scale(0.05, 20.0, 0.1) == pytest.approx(math.exp(-1.0), rel=1e-15)
    assert lib.int8t_dclr_scale(0.5, 20.0, 0.1) == 0.1


def test_argument_errors_before_any_launch(lib):
    vp = C.c_void_p
    fake = vp(0x1000)            # aligned, never dereferenced on these paths
    odd = vp(0x1004)
    q = lib.int8t_quantize
    q.restype = C.c_int
    q.argtypes = [vp, C.POINTER(C.c_int), C.c_int, vp, C.c_int, C.c_uint64, vp, vp, vp, vp, C.c_size_t, vp]
    assert q(None, dims(1, 1, 1, 1), 0, None, 0, 0, fake, fake, None, fake, 1 << 20, None) == 1
    assert q(fake, dims(1, 0, 1, 1), 0, None, 0, 0, fake, fake, None, fake, 1 << 20, None) == 2
    assert q(fake, dims(1, 1, 1, 1), 5, None, 0, 0, fake, fake, None, fake, 1 << 20, None) == 3
    assert q(fake, dims(1, 1, 1, 1), 0, None, 2, 0, fake, fake, None, fake, 1 << 20, None) == 3
    assert q(odd, dims(1, 1, 1, 1), 0, None, 0, 0, fake, fake, None, fake, 1 << 20, None) == 3
    assert q(fake, dims(1, 1, 1, 1), 0, None, 0, 0, fake, fake, None, fake, 16, None) == 4
    assert q(fake, dims(1, 1, 1, 1), 0, None, 0, 0, fake, fake, None, None, 0, None) == 1
    g = lib.int8t_dsgc_clip
    g.restype = C.c_int
    g.argtypes = [vp, C.c_size_t, vp, C.c_int, C.c_int, C.c_uint64, vp, vp, vp, vp, C.c_size_t, vp]
    assert g(fake, 100, fake, 0, 1, 0, fake, fake, None, fake, 1 << 24, None) == 3
    assert g(fake, 100, fake, 65, 1, 0, fake, fake, None, fake, 1 << 24, None) == 3
    assert g(fake, 0, fake, 4, 1, 0, fake, fake, None, fake, 1 << 24, None) == 2
    assert g(fake, 100, None, 4, 1, 0, fake, fake, None, fake, 1 << 24, None) == 1
    assert g(fake, 100, fake, 4, 1, 0, fake, fake, None, fake, 64, None) == 4
    for name in ("int8t_conv_fwd", "int8t_conv_bwd_data", "int8t_conv_bwd_weight"):
        f = getattr(lib, name)
        f.restype = C.c_int
        f.argtypes = [C.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        good = Desc(1, 4, 5, 5, 4, 3, 3, 1, 1, 1, 1, 1)
        assert f(None, fake, fake, fake, fake, fake, None, fake, 1 << 20, None) == 1
        assert f(C.byref(Desc(1, 4, 5, 5, 4, 3, 3, 0, 1, 1, 1, 1)), fake, fake, fake, fake, fake, None, fake, 1 << 20, None) == 2
        assert f(C.byref(Desc(1, 4, 5, 5, 6, 3, 3, 1, 1, 1, 1, 2)), fake, fake, fake, fake, fake, None, fake, 1 << 20, None) == 2
        assert f(C.byref(Desc(1, 4, 2, 2, 4, 7, 7, 1, 1, 0, 0, 1)), fake, fake, fake, fake, fake, None, fake, 1 << 20, None) == 2
        assert f(C.byref(good), None, fake, fake, fake, fake, None, fake, 1 << 20, None) == 1
        assert f(C.byref(good), odd, fake, fake, fake, fake, None, fake, 1 << 20, None) == 3
    f = lib.int8t_conv_bwd_weight
    assert f(C.byref(Desc(1, 4, 5, 5, 4, 3, 3, 1, 1, 1, 1, 1)), fake, fake, fake, fake, fake, None, fake, 8, None) == 4
    assert lib.int8t_status_string(4) == b"workspace too small"


def test_profile_entry_points_without_launches(lib):
    class KT(C.Structure):
        _fields_ = [("name", C.c_char_p), ("launches", C.c_int), ("total_ms", C.c_double)]
    assert lib.int8t_profile_start(b"no_such_kernel") == 3          # INT8T_ERR_ARG, timing stays off
    assert lib.int8t_profile_start(b"dsgc_sweep_kernel") == 0
    n = C.c_int(-1)
    buf = (KT * 4)()
    assert lib.int8t_profile_stop(buf, 4, C.byref(n)) == 0 and n.value == 0
    assert lib.int8t_profile_start(None) == 0
    assert lib.int8t_profile_stop(None, 0, C.byref(n)) == 0 and n.value == 0
    assert lib.int8t_profile_stop(None, 4, C.byref(n)) == 3          # capacity without a buffer
    assert lib.int8t_profile_start_sampled(b"band_kernel", 0) == 3   # every >= 1
    assert lib.int8t_profile_start_sampled(b"igemm_reduce_kernel", 5) == 0
    assert lib.int8t_profile_stop(buf, 4, C.byref(n)) == 0 and n.value == 0


def test_quantize_batch_argument_errors(lib):
    class Item(C.Structure):
        _fields_ = [("x_dev", C.c_void_p), ("dims", C.c_int * 4), ("kind", C.c_int), ("clip_dev", C.c_void_p),
                    ("q_dev", C.c_void_p), ("scale_dev", C.c_void_p), ("mode", C.c_int), ("seed", C.c_uint64)]
    lib.int8t_quantize_batch_workspace_bytes.restype = C.c_size_t
    lib.int8t_quantize_batch_workspace_bytes.argtypes = [C.c_int, C.POINTER(Item)]
    f = lib.int8t_quantize_batch
    f.restype = C.c_int
    f.argtypes = [C.c_int, C.POINTER(Item), C.c_void_p, C.c_size_t, C.c_void_p]
    items = (Item * 2)()
    for it in items:
        it.x_dev, it.q_dev, it.scale_dev, it.kind = 0x1000, 0x2000, 0x3000, 0
        it.dims[:] = [1, 16, 4, 4]
    assert lib.int8t_quantize_batch_workspace_bytes(2, items) == 2 * 4096
    assert lib.int8t_quantize_batch_workspace_bytes(0, items) == 0
    assert lib.int8t_quantize_batch_workspace_bytes(9, items) == 0
    assert f(2, None, 0x4000, 1 << 20, None) == 1                  # INT8T_ERR_NULL
    assert f(0, items, 0x4000, 1 << 20, None) == 3                 # INT8T_ERR_ARG: count
    assert f(9, items, 0x4000, 1 << 20, None) == 3
    assert f(2, items, None, 0, None) == 1                         # absmax needs the scratch
    assert f(2, items, 0x4000, 4096, None) == 4                    # INT8T_ERR_WORKSPACE
    items[1].kind = 9
    assert f(2, items, 0x4000, 1 << 20, None) == 3
    items[1].kind = 0
    items[1].mode = 2                                              # neither nearest-even nor stochastic
    assert f(2, items, 0x4000, 1 << 20, None) == 3
    items[1].mode = 1
    items[1].dims[2] = 0
    assert f(2, items, 0x4000, 1 << 20, None) == 2                 # INT8T_ERR_SHAPE
    items[1].dims[2] = 4
    items[0].q_dev = 0x2004
    assert f(2, items, 0x4000, 1 << 20, None) == 3                 # alignment
    items[0].q_dev = 0x2000
    # ... with the first phase of a clip search in the same launch
    lib.int8t_workspace_bytes.restype = C.c_size_t
    lib.int8t_workspace_bytes.argtypes = [C.c_int, C.c_void_p, C.c_size_t, C.c_int]
    need = lib.int8t_workspace_bytes(1, None, 1000, 32)            # INT8T_OP_DSGC
    g = lib.int8t_quantize_batch_prepare
    g.restype = C.c_int
    g.argtypes = [C.c_int, C.POINTER(Item), C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]
    assert g(2, items, 0x4000, 1 << 20, None, 1000, 0x100000, need, None) == 1       # g is required
    assert g(2, items, 0x4000, 1 << 20, 0x8000, 1000, None, 0, None) == 1            # ... and the search's scratch
    assert g(2, items, 0x4000, 1 << 20, 0x8000, 0, 0x100000, need, None) == 2        # n == 0
    assert g(2, items, 0x4000, 1 << 20, 0x8004, 1000, 0x100000, need, None) == 3     # alignment of g
    assert g(2, items, 0x4000, 1 << 20, 0x8000, 1000, 0x100000, need - 1, None) == 4
    assert g(0, items, 0x4000, 1 << 20, 0x8000, 1000, 0x100000, need, None) == 3     # the batch's own checks still apply


def test_dsgc_two_phase_argument_errors(lib):
    vp = C.c_void_p
    prep, search = lib.int8t_dsgc_prepare, lib.int8t_dsgc_search
    prep.restype = search.restype = C.c_int
    prep.argtypes = [vp, C.c_size_t, vp, C.c_size_t, vp]
    search.argtypes = [vp, C.c_size_t, vp, C.c_int, C.c_int, C.c_uint64, vp, vp, vp, vp, C.c_size_t, vp]
    need = lib.int8t_workspace_bytes(1, None, C.c_size_t(1000), 32)
    assert prep(None, 1000, 0x4000, need, None) == 1
    assert prep(0x1000, 0, 0x4000, need, None) == 2
    assert prep(0x1004, 1000, 0x4000, need, None) == 3
    assert prep(0x1000, 1000, 0x4000, need - 1, None) == 4
    assert search(0x1000, 1000, None, 32, 1, 0, 0x2000, 0x3000, None, 0x4000, need, None) == 1
    assert search(0x1000, 1000, 0x5000, 65, 1, 0, 0x2000, 0x3000, None, 0x4000, need, None) == 3
    assert search(0x1000, 1000, 0x5000, 32, 1, 0, 0x2000, 0x3000, None, 0x4000, need - 1, None) == 4



def test_unpack_codes_matches_the_documented_layouts():
    """int8t_unpack_codes against the layout formulas of include/int8t.h written out with numpy."""
    import numpy as np

    from paper_1912_12607_amd import binding as B
    r = np.random.RandomState(3)
    N, Cc, H, W = 3, 24, 5, 7
    q = r.randint(-127, 128, size=(N, Cc, H, W)).astype(np.int8)
    packed = np.zeros((N, H, W, 32), np.int8)
    packed[..., :Cc] = q.transpose(0, 2, 3, 1)
    out, bad = B.int8t_unpack_codes(packed.reshape(-1), (N, Cc, H, W), B.ACT)
    assert bad == 0 and np.array_equal(out, q)
    packed[1, 2, 3, 30] = 1
    assert B.int8t_unpack_codes(packed.reshape(-1), (N, Cc, H, W), B.ACT)[1] == 1
    K, Cg, R, S = 20, 40, 3, 2
    w = r.randint(-127, 128, size=(K, Cg, R, S)).astype(np.int8)
    n1 = K * R * S * 48
    buf = np.zeros(((n1 + 255) // 256) * 256 + Cg * R * S * 32, np.int8)
    a = np.zeros((K, R, S, 48), np.int8)
    a[..., :Cg] = w.transpose(0, 2, 3, 1)
    b = np.zeros((Cg, R, S, 32), np.int8)
    b[..., :K] = w.transpose(1, 2, 3, 0)
    buf[:n1] = a.reshape(-1)
    buf[((n1 + 255) // 256) * 256:] = b.reshape(-1)
    assert buf.size == B.int8t_code_bytes((K, Cg, R, S), B.WGT)
    for copy in (0, 1):
        out, bad = B.int8t_unpack_codes(buf, (K, Cg, R, S), B.WGT, copy)
        assert bad == 0 and np.array_equal(out, w)
    out, _ = B.int8t_unpack_codes(w.reshape(-1), (K, Cg, R, S), B.WGT_PLANAR)
    assert np.array_equal(out, w)
    with pytest.raises(B.Int8tError):
        B.int8t_unpack_codes(buf, (K, Cg, R, S), B.ACT_PLANAR, 1)
