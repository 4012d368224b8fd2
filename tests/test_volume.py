"""The communication-efficiency analysis (Eq. 2 and the appendix's data-volume expressions).

The library derives gamma from the four volume expressions of the appendix, the oracle writes Eq. 2
out; the paper states that the two are the same thing, so each checks the other.  Further pins are
the limits the paper itself draws.  The gamma values the paper tabulates for its two large datasets
cannot serve as fixtures: it does not print the B, M and R that went into them."""
import math

import numpy as np
import pytest

from oracle import volume as ov
from paper_2302_13053_amd import binding as B


CASES = [  # B, R, H0, sum_H, sum_C, M
    (1.2e6, 500.0, 400.0, 2048.0, 48128.0, 1.1e6),
    (175e3, 3000.0, 2408.0, 3072.0, 31488.0, 2.9e6),
    (0.0, 10.0, 100.0, 256.0, 1000.0, 5e4),
    (3.0, 1.0, 7.0, 5.0, 0.0, 11.0),
]


@pytest.mark.parametrize("case", CASES)
def test_gamma_from_volumes_equals_equation_two(case):
    Bn, R, H0, sH, sC, M = case
    got = B.retexo_gamma(Bn, R, H0, sH, sC, M)
    assert math.isclose(got, ov.gamma(Bn, R, H0, sH, sC, M), rel_tol=1e-13)
    for n in (1.0, 8.0):
        st, v = B.retexo_data_volumes(n, Bn, R, H0, sH, sC, M)
        assert st == 0 and math.isclose((v[0] + v[2]) / (v[1] + v[3]), got, rel_tol=1e-13)
        # the appendix's phase ratios
        if Bn > 0:
            assert math.isclose(v[0] / v[1], (2 * R * sH + H0) / (sH + H0), rel_tol=1e-13)
        assert math.isclose(v[2] / v[3], 1.0 / (1.0 + sC / M), rel_tol=1e-13)


def test_limits_the_paper_states():
    R, H0, sH, sC, M = 500.0, 100.0, 512.0, 12032.0, 3e5
    # no boundary nodes: only gradient aggregation remains, ratio 1 / (1 + sum_C / M), close to 1
    assert math.isclose(B.retexo_gamma(0.0, R, H0, sH, sC, M), 1.0 / (1.0 + sC / M), rel_tol=1e-14)
    # many boundary nodes: gamma rises with B and settles at the local-training ratio, Theta(R)
    g = [B.retexo_gamma(b, R, H0, sH, sC, M) for b in (1e2, 1e4, 1e6, 1e9, 1e13)]
    assert all(x < y for x, y in zip(g, g[1:]))
    limit = (2 * R * sH + H0) / (sH + H0)
    assert math.isclose(g[-1], limit, rel_tol=1e-6) and R < limit < 2 * R
    # with M twenty times the added classifiers the aggregation phase alone gives 1 / 1.05
    st, v = B.retexo_data_volumes(4.0, 10.0, R, H0, sH, M / 20.0, M)
    assert math.isclose(v[2] / v[3], 1.0 / 1.05, rel_tol=1e-14)


def test_invalid_arguments():
    assert B.retexo_gamma(1.0, 0.0, 1.0, 1.0, 1.0, 1.0) == -1.0
    assert B.retexo_gamma(1.0, 1.0, 1.0, 1.0, 1.0, 0.0) == -1.0
    assert B.retexo_gamma(-1.0, 1.0, 1.0, 1.0, 1.0, 1.0) == -1.0
    assert B.retexo_gamma(float("nan"), 1.0, 1.0, 1.0, 1.0, 1.0) == -1.0
    assert B.retexo_data_volumes(1.0, 1.0, 1.0, 1.0, 1.0, 1.0, -2.0)[0] == -2
