#!/usr/bin/env python3
"""Writes tests/golden/dclr_eq7.txt: Eq.7, phi(d_c) = max(exp(-alpha d_c), beta), tabulated with the
oracle (oracle.dclr, the only arithmetic called here) at the four (alpha, beta) settings of the
sensitivity table of Sec.4.1 and direction deviations across [0, 2].  Run from the repository root:
    python tests/golden/make_dclr_eq7.py
The table guards the oracle against later edits; what pins Eq.7 itself are the closed-form checks in
tests/test_golden.py (phi(0) = 1, phi = beta from d_c = ln(1/beta)/alpha on, exp(-1), monotone)."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402

HEADER = """# Deviation Counteractive Learning Rate Scaling, Eq.7: phi(d_c) = max(exp(-alpha * d_c), beta),
# at the four (alpha, beta) settings of the sensitivity table of Sec.4.1 (alpha in {10, 20}, beta in {0.1, 0.2};
# the experiments use alpha = 20, beta = 0.1) and direction deviations d_c across its range [0, 2].
# Written by tests/golden/make_dclr_eq7.py from oracle.dclr, 17 significant digits.
# alpha beta d_c phi
"""


def main():
    lines = [HEADER]
    for alpha in (10, 20):
        for beta in (0.1, 0.2):
            for d in (0.0, 0.001, 0.01, 0.05, 0.1, 0.2, 0.5, 1.0, 2.0):
                lines.append("%d %s %s %s\n" % (alpha, repr(beta), repr(d), "%.17g" % oracle.dclr(d, alpha, beta)))
    with open(os.path.join(HERE, "dclr_eq7.txt"), "w") as f:
        f.writelines(lines)


if __name__ == "__main__":
    main()
