"""Fixtures under tests/golden/: values fixed by the paper's own formulas and settings."""
import os

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def test_dclr_scaling_table():
    """Eq.7 at the hyperparameter settings of the paper's sensitivity table."""
    n = 0
    for line in open(os.path.join(HERE, "golden", "dclr_eq7.txt")):
        if line.startswith("#"):
            continue
        alpha, beta, d, phi = (float(v) for v in line.split())
        got = oracle.dclr(d, alpha, beta)
        assert abs(got - phi) <= 1e-15 * max(1.0, phi), (alpha, beta, d)
        assert beta <= got <= 1.0
        n += 1
    assert n == 36


def test_dclr_closed_forms():
    """Eq.7 pinned by what the formula fixes, not by re-evaluating it: phi(0) = 1; phi equals beta from
    d_c = ln(1/beta)/alpha on (0.11513 at the paper's alpha = 20, beta = 0.1); exp(-1) = 0.36787944117144233
    and 1/2 at the deviations that make the exponent -1 and -ln 2; never increasing; beta <= phi <= 1."""
    import math
    assert oracle.dclr(0.0, 20.0, 0.1) == 1.0
    assert abs(oracle.dclr(0.05, 20.0, 0.1) - 0.36787944117144233) < 1e-16
    assert abs(oracle.dclr(0.1, 10.0, 0.2) - 0.36787944117144233) < 1e-16
    assert abs(oracle.dclr(0.6931471805599453 / 20.0, 20.0, 0.1) - 0.5) < 1e-15
    knee = math.log(10.0) / 20.0
    assert abs(knee - 0.11513) < 5e-6
    assert oracle.dclr(knee * (1 - 1e-9), 20.0, 0.1) > 0.1
    for d in (knee * (1 + 1e-9), 0.2, 1.0, 2.0):
        assert oracle.dclr(d, 20.0, 0.1) == 0.1
    prev = 2.0
    for i in range(2001):
        v = oracle.dclr(i * 1e-3, 20.0, 0.1)
        assert 0.1 <= v <= 1.0 and v <= prev
        prev = v
