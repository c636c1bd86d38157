"""Pins for the oracle's quantizer (Eq.1, Eq.2, Eq.3 of the paper) and its uniform draw.

None of these re-types the oracle's own formula: they are invariants the
definitions force, closed forms, special cases that reduce to numpy routines,
and statistics of Eq.3.
"""
import numpy as np
import pytest

import oracle

RTN, STO = oracle.ROUND_NEAREST_EVEN, oracle.ROUND_STOCHASTIC
rs = np.random.RandomState


def test_absmax_is_numpy_abs_max():
    x = rs(1).standard_normal(10007).astype(np.float32)
    assert oracle.absmax(x) == np.abs(x).max()
    x[17] = -99.5
    assert oracle.absmax(x) == np.float32(99.5)
    assert oracle.absmax(np.zeros(5, np.float32)) == 0.0


def test_scale_is_c_over_127():
    # text after Eq.1: s = c / (2^(8-1) - 1)
    for c in (1.0, 127.0, 0.3, 6.1e-5):
        assert oracle.scale(c) == np.float32(np.float32(c) / np.float32(127))


def test_rtn_error_bound_and_range():
    x = rs(2).standard_normal(50000).astype(np.float32) * 3
    q, s = oracle.quantize(x)
    assert q.min() >= -127 and q.max() <= 127
    err = np.abs(q.astype(np.float64) * float(s) - x.astype(np.float64))
    assert err.max() <= float(s) / 2 * (1 + 2 ** -20)


def test_rtn_endpoints_zero_symmetry_monotone():
    x = np.array([-4.0, 0.0, 4.0, 1.0, -1.0, 3.99, 2.5], np.float32)
    q, s = oracle.quantize(x)
    assert q[0] == -127 and q[1] == 0 and q[2] == 127
    y = rs(3).standard_normal(4000).astype(np.float32)
    qp, _ = oracle.quantize(y, c=2.0)
    qm, _ = oracle.quantize(-y, c=2.0)
    assert np.array_equal(qp, -qm)                    # odd symmetry
    ys = np.sort(y)
    qs, _ = oracle.quantize(ys, c=2.0)
    assert np.all(np.diff(qs.astype(np.int32)) >= 0)   # monotone
    assert qs[0] == -127 and qs[-1] == 127              # clipped tails saturate


def test_rtn_exactly_representable_roundtrip():
    # x = k * 2^e with c = 127 * 2^e  =>  q = k exactly and q*s = x exactly
    for e in (-10, 0, 5):
        k = np.arange(-127, 128, dtype=np.int32)
        x = (k * 2.0 ** e).astype(np.float32)
        q, s = oracle.quantize(x, c=127 * 2.0 ** e)
        assert np.array_equal(q.astype(np.int32), k)
        assert np.array_equal(q.astype(np.float32) * s, x)
        q2, _ = oracle.quantize(q.astype(np.float32) * s, c=127 * 2.0 ** e)
        assert np.array_equal(q2, q)                   # idempotent


def test_rtn_ties_go_to_even():
    x = np.array([0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 126.5], np.float32)
    q, _ = oracle.quantize(x, c=127.0)
    assert q.tolist() == [0, 2, 2, 4, 0, -2, -2, 126]


def test_rtn_reduces_to_numpy_rint():
    x = rs(4).standard_normal(100000).astype(np.float32)
    c = np.float32(2.25)
    inv = np.float32(127.0) / c
    ref_scaled_clip = np.rint(np.clip(x * inv, np.float32(-127), np.float32(127))).astype(np.int32)
    q, _ = oracle.quantize(x, c=c)
    assert np.array_equal(q.astype(np.int32), ref_scaled_clip)
    # the literal order of Eq.1 (clip first, then divide by s) gives the same codes
    # except possibly within one rounding of the clip boundary
    lit = np.clip(np.rint(np.clip(x, -c, c) * inv), -127, 127).astype(np.int32)
    assert np.array_equal(q.astype(np.int32), lit)


def test_zero_tensor():
    q, s = oracle.quantize(np.zeros(64, np.float32))
    assert not q.any() and s == 0.0
    q, s = oracle.quantize(np.zeros(64, np.float32), mode=STO, seed=3)
    assert not q.any() and s == 0.0


def test_rng24_range_determinism_uniformity():
    L = oracle.lib()
    n = 1 << 18
    u = np.array([L.orc_rng24(7, i) for i in range(n)], dtype=np.int64)
    assert u.min() >= 0 and u.max() < (1 << 24)
    assert np.array_equal(u[:100], [L.orc_rng24(7, i) for i in range(100)])
    # chi-square on the top 8 bits: 255 dof, mean 255, sd ~22.6
    cnt = np.bincount(u >> 16, minlength=256)
    chi = ((cnt - n / 256.0) ** 2 / (n / 256.0)).sum()
    assert chi < 255 + 6 * 22.6
    # and on the low 8 bits of the 24
    cnt = np.bincount(u & 255, minlength=256)
    chi = ((cnt - n / 256.0) ** 2 / (n / 256.0)).sum()
    assert chi < 255 + 6 * 22.6
    # neighbouring indices and neighbouring seeds are uncorrelated
    f = u / float(1 << 24) - 0.5
    assert abs(np.mean(f[:-1] * f[1:]) * 12) < 6 / np.sqrt(n)
    v = np.array([L.orc_rng24(8, i) for i in range(n)], dtype=np.int64) / float(1 << 24) - 0.5
    assert abs(np.mean(f * v) * 12) < 6 / np.sqrt(n)
    w = np.array([L.orc_rng24(7 + (1 << 32), i) for i in range(n)], dtype=np.int64) / float(1 << 24) - 0.5
    assert abs(np.mean(f * w) * 12) < 6 / np.sqrt(n)


def test_rng24_related_seeds_do_not_share_their_tables():
    """The seed is hashed into the draw's keys first (reading of the replaced generator of Suppl.
    "Stochastic Rounding", Eq.8).  With the raw seed words as keys -- low word xor-ed into the index, high
    word times an odd constant added -- seeds s and s ^ d gave the SAME table at indices i ^ d, and
    seeds that differ in the high word the same table at shifted indices: a training loop that seeds its
    layers and iterations 1, 2, 3, ... would re-use one noise table.  Both relations must be gone."""
    L = oracle.lib()
    n = 1 << 12
    for s, d in ((0, 1), (1, 2), (7, 15), (100, 3), (2 ** 40 + 5, 64)):
        a = np.array([L.orc_rng24(s, i) for i in range(n)], dtype=np.int64)
        b = np.array([L.orc_rng24(s ^ d, i ^ d) for i in range(n)], dtype=np.int64)
        assert np.mean(a == b) < 0.01, (s, d)
    golden = 0x9E3779B9
    for s, h in ((5, 1), (5, 2), (123456, 7)):
        lo = s & 0xFFFFFFFF
        a = np.array([L.orc_rng24(s, i) for i in range(n)], dtype=np.int64)
        # the index at which the old generator repeated draw(s, i) under seed s + (h << 32)
        j = [((((i ^ lo) - h * golden) & 0xFFFFFFFF) ^ lo) for i in range(n)]
        b = np.array([L.orc_rng24(s + (h << 32), jj) for jj in j], dtype=np.int64)
        assert np.mean(a == b) < 0.01, (s, h)
    # and the tables of consecutive seeds are uncorrelated position by position and at small offsets
    f = [np.array([L.orc_rng24(s, i) for i in range(1 << 14)], dtype=np.float64) / (1 << 24) - 0.5 for s in (1, 2, 3)]
    for a, b in ((0, 1), (1, 2), (0, 2)):
        for off in (0, 1, 2, 3, 5, 8):
            x, y = f[a][off:], f[b][:len(f[b]) - off]
            assert abs(np.mean(x * y) * 12) < 6 / np.sqrt(len(x)), (a, b, off)


def test_rng24_is_equidistributed_bijection_on_a_block():
    # for a fixed seed the 32-bit state is a bijection of the index: no collisions of the
    # full 24-bit draw beyond what 2^16 samples of a bijection's top bits allow
    L = oracle.lib()
    u = np.array([L.orc_rng24(123, i) for i in range(1 << 16)], dtype=np.int64)
    # birthday bound: expected collisions ~ n^2 / 2^25 = 128
    assert (len(u) - len(np.unique(u))) < 128 + 6 * 12


def test_stochastic_brackets_and_error():
    x = rs(5).standard_normal(100000).astype(np.float32)
    c = np.float32(3.0)
    inv = np.float32(127.0) / c
    t = np.clip(x * inv, np.float32(-127), np.float32(127)).astype(np.float64)
    for seed in (0, 1, 2 ** 40 + 5):
        q, s = oracle.quantize(x, c=c, mode=STO, seed=seed)
        qi = q.astype(np.float64)
        f = np.floor(t)
        assert np.all((qi == f) | (qi == f + 1))
        assert q.min() >= -127 and q.max() <= 127
        inside = np.abs(x) <= c
        err = np.abs(qi * float(s) - x.astype(np.float64))[inside]
        assert err.max() < float(s) * (1 + 1e-5)


def test_stochastic_integers_are_fixed_points():
    k = np.arange(-127, 128, dtype=np.int32)
    x = k.astype(np.float32) * np.float32(0.25)
    for seed in range(20):
        q, _ = oracle.quantize(x, c=127 * 0.25, mode=STO, seed=seed)
        assert np.array_equal(q.astype(np.int32), k)


def test_stochastic_unbiased():
    # Eq.3: E[round_s(t)] = t.  Average over many seeds at fixed positions.
    t = np.array([0.1, 0.5, 0.9, -0.3, -7.25, 100.625, 3.0, -126.99], np.float64)
    c = np.float32(127.0)
    x = t.astype(np.float32)
    S = 20000
    acc = np.zeros(len(t))
    for seed in range(S):
        q, _ = oracle.quantize(x, c=c, mode=STO, seed=seed)
        acc += q
    mean = acc / S
    frac = x.astype(np.float64) - np.floor(x.astype(np.float64))
    sd = np.sqrt(np.maximum(frac * (1 - frac), 1e-12) / S)
    assert np.all(np.abs(mean - x.astype(np.float64)) <= 5 * sd + 1e-6)
    # same, averaging over positions with one seed
    xx = np.full(200000, 0.3, np.float32)
    q, _ = oracle.quantize(xx, c=c, mode=STO, seed=11)
    assert abs(q.mean() - 0.3) < 5 * np.sqrt(0.21 / len(xx))


def test_stochastic_probability_is_frac_to_24_bits():
    # up-probability = floor(frac * 2^24) / 2^24: frac = 0 never goes up; frac = 1 - 2^-24 goes
    # up for every draw but u = 0; frac = 2^-24 goes up only for u = 2^24 - 1
    x = np.array([5.0, 0.99999994, 2.0 ** -24], np.float32)   # second = 1 - 2^-24
    for seed in range(3000):
        q, _ = oracle.quantize(x, c=127.0, mode=STO, seed=seed)
        u1, u2 = oracle.rng24(seed, 1), oracle.rng24(seed, 2)
        assert q[0] == 5
        assert q[1] == (1 if u1 >= 1 else 0)
        assert q[2] == (1 if u2 == (1 << 24) - 1 else 0)


def test_stochastic_same_seed_same_codes_and_index_keyed():
    x = rs(6).standard_normal(5000).astype(np.float32)
    a, _ = oracle.quantize(x, c=2.0, mode=STO, seed=42)
    b, _ = oracle.quantize(x, c=2.0, mode=STO, seed=42)
    c, _ = oracle.quantize(x, c=2.0, mode=STO, seed=43)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    # the draw is a function of (seed, logical index) only: quantizing a constant tensor
    # reproduces rng24 directly: q_i = 1 iff u_i >= 2^24 - thr
    xc = np.full(4096, 0.25, np.float32)
    q, _ = oracle.quantize(xc, c=127.0, mode=STO, seed=9)
    u = np.array([oracle.rng24(9, i) for i in range(4096)])
    assert np.array_equal(q.astype(bool), u >= (1 << 24) - (1 << 22))


def test_dclr_eq7():
    import math
    assert oracle.dclr(0.0) == 1.0
    assert oracle.dclr(1.0) == 0.1
    assert oracle.dclr(0.2) == 0.1                       # exp(-4) < beta
    assert oracle.dclr(0.05) == pytest.approx(math.exp(-1.0), rel=1e-15)
    knee = math.log(1 / 0.1) / 20
    assert oracle.dclr(knee * 0.999) > 0.1 and oracle.dclr(knee * 1.001) == 0.1
    d = np.linspace(0, 0.3, 50)
    phi = [oracle.dclr(v) for v in d]
    assert all(a >= b for a, b in zip(phi, phi[1:]))
    assert oracle.dclr(0.01, alpha=5.0, beta=0.5) == pytest.approx(math.exp(-0.05))
