"""Pins for the oracle's three integer convolutions (Sec.3.4: forward, g_a and g_W = g_z^T a)."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

rs = np.random.RandomState

# (N, C, H, W, K, R, S, stride, pad, groups)
SHAPES = [
    (2, 3, 5, 5, 4, 3, 3, (1, 1), (1, 1), 1),
    (1, 4, 6, 7, 2, 3, 3, (2, 2), (0, 0), 1),
    (2, 2, 7, 5, 3, 3, 3, (2, 1), (1, 0), 1),
    (1, 3, 5, 9, 2, 1, 7, (1, 1), (0, 3), 1),
    (1, 3, 9, 5, 2, 7, 1, (1, 1), (3, 0), 1),
    (2, 4, 5, 5, 4, 3, 3, (1, 1), (1, 1), 4),     # depthwise
    (1, 4, 6, 6, 6, 3, 3, (2, 2), (1, 1), 2),     # grouped, stride 2
    (3, 5, 4, 4, 7, 1, 1, (1, 1), (0, 0), 1),
    (1, 2, 8, 8, 2, 5, 5, (3, 2), (2, 2), 1),
    (2, 6, 5, 4, 6, 3, 2, (1, 2), (2, 1), 3),
]


def mk(shape, seed=0):
    N, C, H, W, K, R, S, st, pd, g = shape
    d = oracle.make_desc(N, C, H, W, K, R, S, st, pd, g)
    P, Q = oracle.out_hw(d)
    r = rs(seed)
    x = r.randint(-127, 128, size=(N, C, H, W)).astype(np.int8)
    w = r.randint(-127, 128, size=(K, C // g, R, S)).astype(np.int8)
    dy = r.randint(-127, 128, size=(N, K, P, Q)).astype(np.int8)
    return d, x, w, dy


@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identity_exact(shape):
    # <dy, conv(x,w)> = <bwd_data(dy,w), x> = <bwd_weight(x,dy), w>, all in exact integers
    d, x, w, dy = mk(shape, 1)
    y = oracle.conv_fwd(d, x, w)
    dx = oracle.conv_bwd_data(d, dy, w)
    dw = oracle.conv_bwd_weight(d, x, dy)
    a = int((dy.astype(np.int64) * y).sum())
    b = int((dx * x.astype(np.int64)).sum())
    c = int((dw * w.astype(np.int64)).sum())
    assert a == b == c and a != 0


@pytest.mark.parametrize("shape", SHAPES)
def test_against_torch_float64(shape):
    # integer-valued float64 tensors: torch's conv2d and its autograd are exact below 2^53
    d, x, w, dy = mk(shape, 2)
    N, C, H, W, K, R, S, st, pd, g = shape
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    yt = F.conv2d(xt, wt, None, st, pd, 1, g)
    gx, gw = torch.autograd.grad(yt, (xt, wt), torch.tensor(dy, dtype=torch.float64))
    assert np.array_equal(oracle.conv_fwd(d, x, w), yt.detach().numpy().astype(np.int64))
    assert np.array_equal(oracle.conv_bwd_data(d, dy, w), gx.numpy().astype(np.int64))
    assert np.array_equal(oracle.conv_bwd_weight(d, x, dy), gw.numpy().astype(np.int64))


def test_point_functions_equal_full_tensors():
    d, x, w, dy = mk(SHAPES[6], 3)
    y = oracle.conv_fwd(d, x, w)
    dx = oracle.conv_bwd_data(d, dy, w)
    dw = oracle.conv_bwd_weight(d, x, dy)
    for idx in itertools.islice(np.ndindex(*y.shape), 0, None, 7):
        assert oracle.conv_fwd_at(d, x, w, *idx) == y[idx]
    for idx in itertools.islice(np.ndindex(*dx.shape), 0, None, 5):
        assert oracle.conv_bwd_data_at(d, dy, w, *idx) == dx[idx]
    for idx in itertools.islice(np.ndindex(*dw.shape), 0, None, 3):
        assert oracle.conv_bwd_weight_at(d, x, dy, *idx) == dw[idx]


def test_1x1_is_matmul():
    N, C, H, W, K = 3, 5, 4, 6, 7
    d, x, w, dy = mk((N, C, H, W, K, 1, 1, (1, 1), (0, 0), 1), 4)
    X = x.astype(np.int64).transpose(0, 2, 3, 1).reshape(-1, C)          # pixels x C
    Wm = w.astype(np.int64).reshape(K, C)
    DY = dy.astype(np.int64).transpose(0, 2, 3, 1).reshape(-1, K)        # pixels x K
    assert np.array_equal(oracle.conv_fwd(d, x, w).transpose(0, 2, 3, 1).reshape(-1, K), X @ Wm.T)
    assert np.array_equal(oracle.conv_bwd_data(d, dy, w).transpose(0, 2, 3, 1).reshape(-1, C), DY @ Wm)
    assert np.array_equal(oracle.conv_bwd_weight(d, x, dy).reshape(K, C), DY.T @ X)


def test_centre_tap_delta_is_identity():
    N, C, H, W = 2, 3, 6, 5
    d = oracle.make_desc(N, C, H, W, C, 3, 3, (1, 1), (1, 1), 1)
    x = rs(5).randint(-127, 128, size=(N, C, H, W)).astype(np.int8)
    w = np.zeros((C, C, 3, 3), np.int8)
    for c in range(C):
        w[c, c, 1, 1] = 1
    assert np.array_equal(oracle.conv_fwd(d, x, w), x.astype(np.int64))
    assert np.array_equal(oracle.conv_bwd_data(d, x, w), x.astype(np.int64))
    # off-centre tap shifts: w[c,c,0,1]=1 reads the row above
    w2 = np.zeros_like(w)
    for c in range(C):
        w2[c, c, 0, 1] = 1
    y = oracle.conv_fwd(d, x, w2)
    assert np.array_equal(y[:, :, 1:, :], x[:, :, :-1, :].astype(np.int64)) and not y[:, :, 0, :].any()


@pytest.mark.parametrize("stride,pad", [((1, 1), (1, 1)), ((2, 2), (1, 1)), ((2, 2), (0, 0)), ((1, 1), (0, 3))])
def test_all_ones_counts_inbounds_taps(stride, pad):
    N, C, H, W, K = 1, 3, 7, 8, 2
    R, S = (1, 7) if pad == (0, 3) else (3, 3)
    d = oracle.make_desc(N, C, H, W, K, R, S, stride, pad, 1)
    P, Q = oracle.out_hw(d)
    assert P == (H + 2 * pad[0] - R) // stride[0] + 1 and Q == (W + 2 * pad[1] - S) // stride[1] + 1
    y = oracle.conv_fwd(d, np.ones((N, C, H, W), np.int8), np.ones((K, C, R, S), np.int8))
    for p in range(P):
        for q in range(Q):
            rows = sum(0 <= p * stride[0] + r - pad[0] < H for r in range(R))
            cols = sum(0 <= q * stride[1] + s - pad[1] < W for s in range(S))
            assert y[0, 0, p, q] == rows * cols * C == y[0, 1, p, q]


def test_linearity():
    d, x, w, dy = mk(SHAPES[0], 6)
    _, x2, w2, dy2 = mk(SHAPES[0], 7)
    h = lambda a: (a // 2).astype(np.int8)        # keep sums inside int8
    lhs = oracle.conv_fwd(d, h(x) + h(x2), w)
    assert np.array_equal(lhs, oracle.conv_fwd(d, h(x), w) + oracle.conv_fwd(d, h(x2), w))
    lhs = oracle.conv_bwd_weight(d, x, h(dy) + h(dy2))
    assert np.array_equal(lhs, oracle.conv_bwd_weight(d, x, h(dy)) + oracle.conv_bwd_weight(d, x, h(dy2)))
    lhs = oracle.conv_bwd_data(d, dy, h(w) + h(w2))
    assert np.array_equal(lhs, oracle.conv_bwd_data(d, dy, h(w)) + oracle.conv_bwd_data(d, dy, h(w2)))


def test_int32_wrap_known_value():
    # reduction of 133145 products 127*127 = 2147495705 > 2^31 - 1: low 32 bits are -2147471591
    N, P, Q = 5, 31, 859
    assert N * P * Q == 133145
    d = oracle.make_desc(N, 1, P, Q, 1, 1, 1)
    x = np.full((N, 1, P, Q), 127, np.int8)
    dy = np.full((N, 1, P, Q), 127, np.int8)
    acc = oracle.conv_bwd_weight(d, x, dy)
    assert acc[0, 0, 0, 0] == 133145 * 16129 == 2147495705
    a32, ov = oracle.wrap32(acc)
    assert ov == 1 and a32[0, 0, 0, 0] == 2147495705 - 2 ** 32 == -2147471591
    a32, ov = oracle.wrap32(np.array([5, -7, 2 ** 31 - 1, -2 ** 31], np.int64))
    assert ov == 0 and a32.tolist() == [5, -7, 2 ** 31 - 1, -2 ** 31]


def test_dequant_epilogue():
    acc = np.array([0, 1, -3, 123456789, -2 ** 31], np.int32)
    # power-of-two scales: exact
    out = oracle.dequant(acc, 2.0 ** -9, 2.0 ** -4)
    assert np.array_equal(out, (acc.astype(np.float64) * 2.0 ** -13).astype(np.float32))
    assert out[0] == 0.0
    # general scales: one rounding of the exact product
    sa, sb = np.float32(0.0123), np.float32(3.3e-5)
    out = oracle.dequant(acc, sa, sb)
    want = (acc.astype(np.float64) * float(sa) * float(sb))
    assert np.all(np.abs(out - want) <= np.abs(want) * 2.0 ** -24)


def test_end_to_end_plausibility():
    # not a parity pin: dequantized INT8 conv tracks the fp32 conv to O(1/127)
    r = rs(8)
    x = r.standard_normal((2, 8, 10, 10)).astype(np.float32)
    w = (r.standard_normal((6, 8, 3, 3)) * 0.1).astype(np.float32)
    d = oracle.make_desc(2, 8, 10, 10, 6, 3, 3, (1, 1), (1, 1), 1)
    xq, sx = oracle.quantize(x)
    wq, sw = oracle.quantize(w)
    a32, ov = oracle.wrap32(oracle.conv_fwd(d, xq, wq))
    y = oracle.dequant(a32, sx, sw)
    ref = F.conv2d(torch.tensor(x), torch.tensor(w), padding=1).numpy()
    cos = (y * ref).sum() / np.sqrt((y * y).sum() * (ref * ref).sum())
    assert ov == 0 and cos > 0.999
