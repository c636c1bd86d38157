"""Pins for the oracle's direction deviation (Eq.6) and the clip search built on it (Sec.3.4)."""
import numpy as np
import pytest

import oracle

RTN, STO = oracle.ROUND_NEAREST_EVEN, oracle.ROUND_STOCHASTIC
rs = np.random.RandomState


def heavy_tail(n, seed):
    g = rs(seed).standard_t(3, size=n).astype(np.float32) * np.float32(1e-3)
    g[:: max(1, n // 7)] *= 100
    return g


def test_deviation_hand_computed_cases():
    # g = (3,4), ghat = (127 s, 0): cos = 3/5
    assert oracle.deviation([3, 4], [127, 0], 0.01) == pytest.approx(0.4, abs=1e-15)
    # orthogonal and opposite directions
    assert oracle.deviation([1, 1], [1, -1], 1.0) == pytest.approx(1.0, abs=1e-15)
    assert oracle.deviation([1, 2, -3], [-10, -20, 30], 0.5) == pytest.approx(2.0, abs=1e-15)
    # ghat parallel to g
    assert oracle.deviation([0.5, -1.0, 1.5], [1, -2, 3], 7.0) == pytest.approx(0.0, abs=1e-15)
    # two-level input: g = (a,a,b), codes (1,1,127):  cos = (2a + 127b) / (sqrt(2a^2+b^2) sqrt(2+127^2))
    a, b = 0.01, 1.0
    want = 1 - (2 * a + 127 * b) / (np.sqrt(2 * a * a + b * b) * np.sqrt(2 + 127.0 ** 2))
    assert oracle.deviation(np.float32([a, a, b]), [1, 1, 127], 1 / 127) == pytest.approx(
        1 - (2 * float(np.float32(a)) + 127 * b) /
        (np.sqrt(2 * float(np.float32(a)) ** 2 + b * b) * np.sqrt(2 + 127.0 ** 2)), abs=1e-15)
    assert abs(want - oracle.deviation(np.float32([a, a, b]), [1, 1, 127], 1 / 127)) < 1e-8


def test_deviation_degenerate():
    assert oracle.deviation(np.zeros(4), np.zeros(4, np.int8), 0.0) == 0.0
    assert oracle.deviation([1, 2, 3, 4], np.zeros(4, np.int8), 0.1) == 1.0


def test_deviation_bounds_cauchy_schwarz():
    for seed in range(5):
        g = heavy_tail(5000, seed)
        for c_ratio in (1.0, 0.1, 0.001):
            for mode in (RTN, STO):
                q, s = oracle.quantize(g, c=oracle.absmax(g) * c_ratio, mode=mode, seed=seed)
                d = oracle.deviation(g, q, s)
                assert -1e-15 <= d <= 2.0


def test_zero_deviation_on_representable_inputs():
    # ratio 1 and g on the code grid: ghat == g, so d = 0 up to rounding of the double sums
    k = rs(1).randint(-127, 128, size=4096)
    k[0] = 127
    g = (k * 2.0 ** -12).astype(np.float32)
    for mode in (RTN, STO):
        r = oracle.dsgc(g, [1.0], mode=mode, seed=5)
        assert abs(r["deviation"]) < 1e-15
        assert r["clip"] == oracle.absmax(g) == np.float32(127 * 2.0 ** -12)


def test_scale_invariance_exact():
    g = heavy_tail(20000, 2)
    ratios = np.exp2(-np.arange(8) / 2.0).astype(np.float32)
    for mode in (RTN, STO):
        a = oracle.dsgc(g, ratios, mode=mode, seed=3)
        b = oracle.dsgc(g * np.float32(2.0 ** 9), ratios, mode=mode, seed=3)
        c = oracle.dsgc(g * np.float32(2.0 ** -7), ratios, mode=mode, seed=3)
        assert np.array_equal(a["dev"], b["dev"]) and np.array_equal(a["dev"], c["dev"])
        assert a["jstar"] == b["jstar"] == c["jstar"]
        assert b["clip"] == a["clip"] * np.float32(2.0 ** 9)


def test_closed_form_when_everything_clips():
    # clip below min|g|: every code is +-127 (RTN), so cos = ||g||_1 / (sqrt(n) ||g||_2)
    g = rs(3).uniform(1.0, 5.0, size=3000).astype(np.float32) * rs(4).choice([-1, 1], size=3000)
    g = g.astype(np.float32)
    m = oracle.absmax(g)
    ratio = np.float32(0.5 / m)          # c ~ 0.5 < min|g| = 1
    r = oracle.dsgc(g, [ratio], mode=RTN)
    g64 = g.astype(np.float64)
    want = 1 - np.abs(g64).sum() / (np.sqrt(g.size) * np.sqrt((g64 ** 2).sum()))
    assert r["deviation"] == pytest.approx(want, abs=1e-13)


def test_bruteforce_equals_scale_free_form_and_exhaustive_argmin():
    g = rs(5).standard_t(3, size=200000).astype(np.float32) * np.float32(1e-3)
    g[rs(6).choice(g.size, 20, replace=False)] *= 100     # "sharp and wide" (Sec.3.2, C1)
    ratios = np.exp2(-np.arange(16) / 2.0).astype(np.float32)
    for mode in (RTN, STO):
        r = oracle.dsgc(g, ratios, mode=mode, seed=8)
        m = oracle.absmax(g)
        G = (g.astype(np.float64) ** 2).sum()
        dev = []
        for j, ratio in enumerate(ratios):
            c = np.float32(m * ratio)
            assert r["clips"][j] == c
            q, s = oracle.quantize(g, c=c, mode=mode, seed=8)
            A = (g.astype(np.float64) * q.astype(np.float64)).sum()
            B = float((q.astype(np.int64) ** 2).sum())
            dev.append(1 - A / np.sqrt(G * B))        # scale s cancels
        dev = np.array(dev)
        assert np.allclose(r["dev"], dev, rtol=0, atol=1e-12)
        assert r["jstar"] == int(np.argmin(r["dev"]))
        assert r["deviation"] == r["dev"][r["jstar"]] and r["clip"] == r["clips"][r["jstar"]]
        if mode == STO:
            # heavy tails + rounding noise: the best clip is strictly inside the range
            # (an interior optimum, as the paper's "effect of clipping" figure shows)
            assert 0 < r["jstar"] < len(ratios) - 1
            assert r["deviation"] < r["dev"][0]


def test_single_ratio_one_is_absmax_quantizer():
    g = heavy_tail(5000, 6)
    r = oracle.dsgc(g, [1.0], mode=STO, seed=2)
    q, s = oracle.quantize(g, mode=STO, seed=2)           # c = absmax
    assert r["clip"] == oracle.absmax(g)
    assert r["deviation"] == oracle.deviation(g, q, s)


def test_ties_go_to_largest_clip_and_zero_tensor():
    # representable inputs: ratios 1 and 1 (duplicate) tie exactly -> first wins
    k = np.arange(-127, 128)
    g = (k * 0.5).astype(np.float32)
    r = oracle.dsgc(g, [1.0, 1.0, 0.5], mode=RTN)
    assert r["jstar"] == 0
    z = oracle.dsgc(np.zeros(100, np.float32), [1.0, 0.5], mode=STO, seed=1)
    assert z["jstar"] == 0 and z["clip"] == 0.0 and z["deviation"] == 0.0 and z["absmax"] == 0.0


def test_search_uses_same_draws_as_final_quantization():
    # the deviation reported for the winner is the deviation of the codes a later
    # quantize call with (clip, seed) produces
    g = heavy_tail(20000, 9)
    ratios = np.exp2(-np.arange(12) / 2.0).astype(np.float32)
    r = oracle.dsgc(g, ratios, mode=STO, seed=77)
    q, s = oracle.quantize(g, c=r["clip"], mode=STO, seed=77)
    assert oracle.deviation(g, q, s) == r["deviation"]
    q2, s2 = oracle.quantize(g, c=r["clip"], mode=STO, seed=78)
    assert oracle.deviation(g, q2, s2) != r["deviation"]
