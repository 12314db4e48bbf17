"""Pins for alpha* (Sec. 3.1): closed form at b = 1, quadrature, Monte Carlo, brute force."""
import math

import numpy as np
import pytest
from scipy import integrate

from oracle import alpha_star as a


def _mse_by_quadrature(alpha, bits):
    levels = 1 << bits

    def err2(x):
        v = min(max(x, -alpha), alpha)
        grid = [alpha * (2 * k + 1) / (levels - 1) for k in range(-levels // 2, levels // 2)]
        q = min(grid, key=lambda g: abs(g - v))
        return (x - q) ** 2 * math.exp(-0.5 * x * x) / math.sqrt(2 * math.pi)

    step = 2 * alpha / (levels - 1)
    knots = [k * step for k in range(-levels // 2 + 1, levels // 2)]
    edges = [-12.0] + knots + [12.0]
    return sum(integrate.quad(err2, lo, hi, epsabs=1e-13)[0] for lo, hi in zip(edges, edges[1:]))


def test_one_bit_closed_form():
    # b = 1: the grid is {-alpha, +alpha}; E(|xi| - alpha)^2 is minimised at alpha = E|xi|.
    assert a.alpha_star(1) == pytest.approx(math.sqrt(2 / math.pi), abs=1e-7)
    assert a.gaussian_mse(a.alpha_star(1), 1) == pytest.approx(1 - 2 / math.pi, abs=1e-10)
    for alpha in (0.3, 0.8, 1.7):
        assert a.gaussian_mse(alpha, 1) == pytest.approx(1 - 2 * alpha * math.sqrt(2 / math.pi) + alpha ** 2,
                                                         abs=1e-12)


@pytest.mark.parametrize("bits,alpha", [(1, 0.6), (2, 1.5), (2, 0.7), (3, 2.0), (4, 2.5), (4, 4.0)])
def test_closed_form_equals_quadrature_of_definition(bits, alpha):
    assert a.gaussian_mse(alpha, bits) == pytest.approx(_mse_by_quadrature(alpha, bits), abs=1e-9)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_closed_form_matches_monte_carlo(bits, alpha_table):
    rng = np.random.default_rng(bits)
    xi = rng.standard_normal(2_000_000)
    alpha = alpha_table[bits]
    levels = 1 << bits
    k = np.clip(np.floor(xi / (2 * alpha / (levels - 1))), -levels // 2, levels // 2 - 1)
    mse = np.mean((xi - alpha * (2 * k + 1) / (levels - 1)) ** 2)
    assert mse == pytest.approx(a.gaussian_mse(alpha, bits), rel=5e-3)


@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_minimiser_beats_a_brute_force_sweep(bits, alpha_table):
    best = alpha_table[bits]
    sweep = np.linspace(0.2, 6.0, 2901)
    values = np.array([a.gaussian_mse(float(s), bits) for s in sweep])
    assert a.gaussian_mse(best, bits) <= values.min() + 1e-12
    assert abs(sweep[values.argmin()] - best) <= 2e-3 + 1e-2 * (bits == 8)
    # stationarity: the error is flat to first order at the minimiser
    h = 1e-4
    slope = (a.gaussian_mse(best + h, bits) - a.gaussian_mse(best - h, bits)) / (2 * h)
    assert abs(slope) < 1e-6


def test_alpha_grows_with_bits_and_error_falls(alpha_table):
    bits = [1, 2, 3, 4, 8]
    alphas = [alpha_table[b] for b in bits]
    errors = [a.gaussian_mse(alpha_table[b], b) for b in bits]
    assert alphas == sorted(alphas) and errors == sorted(errors, reverse=True)


def test_stored_table_is_what_the_oracle_derives(alpha_table):
    # tests/golden/alpha_star.txt is written by tests/golden/make_alpha_star.py from the oracle only.
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "alpha_star.txt")
    rows = [line.split() for line in open(path) if line.strip() and not line.startswith("#")]
    fp4 = [r for r in rows if r[0] == "fp4"]
    rows = [r for r in rows if r[0] != "fp4"]
    assert len(fp4) == 1 and float(fp4[0][1]) == pytest.approx(a.alpha_star_fp4(), abs=2e-6)
    assert float(fp4[0][2]) == pytest.approx(a.gaussian_mse_fp4(a.alpha_star_fp4()), rel=1e-6)
    assert [int(r[0]) for r in rows] == [1, 2, 3, 4, 8]
    for r in rows:
        assert float(r[1]) == pytest.approx(alpha_table[int(r[0])], abs=2e-6)
        assert float(r[2]) == pytest.approx(a.gaussian_mse(alpha_table[int(r[0])], int(r[0])), rel=1e-6)


def test_untrusted_fraction_at_one_bit():
    # b = 1, outer_trust = 1: the trust region reaches a whole alpha beyond the grid (Sec. 3.3,
    # "The 1-bit Case"), i.e. M = 0 iff |xi| > 2 alpha.
    from scipy.special import ndtr
    alpha = a.alpha_star(1)
    assert a.untrusted_fraction(alpha, 1) == pytest.approx(2 * ndtr(-2 * alpha), rel=1e-12)
