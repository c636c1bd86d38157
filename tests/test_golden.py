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
