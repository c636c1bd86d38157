"""The synthetic-input recipe: shapes of the benchmark layers, determinism, distributions."""
import numpy as np

from paper_1912_12607_amd import inputs


def test_layer_shapes():
    L = inputs.CONFIGS[1][0]
    assert (L.P, L.Q) == (56, 56) and L.macs == 64 * 64 * 56 * 56 * 64 * 9
    a, b, c = inputs.CONFIGS[4]
    assert (a.P, a.Q) == (17, 17) and (b.P, b.Q) == (17, 17) and (c.P, c.Q) == (8, 8)
    dw = inputs.CONFIGS[3][1]
    assert dw.w_shape == (144, 1, 3, 3) and dw.groups == 144


def test_config0_deterministic_and_distributed_as_stated():
    L, x, w, dy = inputs.make_layer_inputs(0, 0)
    L2, x2, w2, dy2 = inputs.make_layer_inputs(0, 0)
    assert np.array_equal(x, x2) and np.array_equal(w, w2) and np.array_equal(dy, dy2)
    assert x.shape == (2, 16, 16, 16) and w.shape == (32, 16, 3, 3) and dy.shape == (2, 32, 16, 16)
    assert x.dtype == w.dtype == dy.dtype == np.float32
    assert abs(x.std() - 1.0) < 0.05 and abs(w.std() - np.sqrt(2 / 144)) < 0.01
    assert round(1e-4 * dy.size) == 2


def test_default_ratios():
    r = inputs.default_ratios()
    assert r.dtype == np.float32 and r.size == 32 and r[0] == 1.0 and r[4] == 0.5 and r[8] == 0.25
    assert np.all(np.diff(r) < 0)


def test_relu_variants():
    L = inputs.CONFIGS[3][1]
    small = inputs.Layer("t", 1, 4, 8, 8, 4, 3, 3, pad=(1, 1), groups=4, x_dist="relu6")
    x = inputs.make_x(small, 9, 0)
    assert x.min() >= 0 and x.max() <= 6
    assert L.x_dist == "relu6" and inputs.CONFIGS[1][0].x_dist == "relu"
