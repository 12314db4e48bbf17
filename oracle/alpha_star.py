"""Oracle side of the clip constant alpha* (Sec. 3.1, "Gaussian Fitting").

TEST INFRASTRUCTURE ONLY.  alpha*(b) is the alpha that minimises the mean squared error of
projecting a standard normal variable onto the 2^b-level zero-free symmetric grid of Eq. 1
after clipping at alpha.  The paper prints no value, so the oracle derives it here, by
numeric minimisation of the closed-form error, independently of the constant table that is
compiled into the HIP library.

Pins (tests/test_oracle_alpha.py): b = 1 closed form alpha* = E|xi| = sqrt(2/pi) with error
1 - 2/pi; the closed-form error against adaptive quadrature of the definition and against
a Monte-Carlo estimate; the minimiser against a brute-force sweep over alpha.
"""
from __future__ import annotations

import math

from scipy.optimize import minimize_scalar
from scipy.special import ndtr  # standard normal CDF


def _pdf(x: float) -> float:
    if math.isinf(x):
        return 0.0
    return math.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def _cell_error(lo: float, hi: float, q: float) -> float:
    """Integral over [lo, hi] of (xi - q)^2 phi(xi) d xi.

    An antiderivative of (xi - q)^2 phi(xi) is (1 + q^2) Phi(xi) + (2 q - xi) phi(xi),
    since the integral of xi^2 phi is Phi - xi phi and that of xi phi is -phi.
    """
    def anti(x: float) -> float:
        tail = 0.0 if math.isinf(x) else (2.0 * q - x) * _pdf(x)
        return (1.0 + q * q) * float(ndtr(x)) + tail

    return anti(hi) - anti(lo)


def gaussian_mse(alpha: float, bits: int) -> float:
    """E (xi - alpha * round(clip(xi, alpha) / alpha))^2 for xi ~ N(0, 1) on the Eq. 1 grid.

    Grid points q_k = alpha (2k + 1) / (L - 1), k = -L/2 .. L/2 - 1; cell k is
    [k D, (k + 1) D) with D = 2 alpha / (L - 1); the two outer cells run to infinity
    (clipping sends everything beyond alpha to the outermost point).
    """
    levels = 1 << bits
    step = 2.0 * alpha / (levels - 1)
    total = 0.0
    for k in range(-levels // 2, levels // 2):
        q = alpha * (2 * k + 1) / (levels - 1)
        lo = -math.inf if k == -levels // 2 else k * step
        hi = math.inf if k == levels // 2 - 1 else (k + 1) * step
        total += _cell_error(lo, hi, q)
    return total


def alpha_star(bits: int) -> float:
    """argmin over alpha of gaussian_mse(alpha, bits), by bounded scalar minimisation."""
    result = minimize_scalar(gaussian_mse, bounds=(0.05, 8.0), args=(bits,), method="bounded",
                             options={"xatol": 1e-10})
    return float(result.x)


def untrusted_fraction(alpha: float, bits: int, outer_trust: float = 1.0) -> float:
    """P(M = 0) for a standard normal input: |xi| > alpha (1 + outer_trust / (L - 1))."""
    levels = 1 << bits
    edge = alpha * (1.0 + outer_trust / (levels - 1))
    return 2.0 * float(ndtr(-edge))


# ------------------------------------------------------------------ FP4 grid (Sec. 4.4, "The FP4 Format")

# Magnitudes of the 4-bit floating-point format with 2 exponent and 1 mantissa bit (E2M1),
# in code order; divided by the largest one they span [-1, 1] like the integer grid (Sec. 4.4).
FP4_MAGNITUDES = (0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0)


def fp4_grid() -> list[float]:
    """The 15 distinct points of the scaled grid, ascending."""
    pos = [m / 6.0 for m in FP4_MAGNITUDES]
    return [-p for p in reversed(pos[1:])] + pos


def gaussian_mse_fp4(alpha: float) -> float:
    """E (xi - alpha * round_FP4(clip(xi, alpha) / alpha))^2 for xi ~ N(0, 1): each grid point
    owns the interval between the midpoints to its neighbours, the outer ones run to infinity."""
    grid = [alpha * g for g in fp4_grid()]
    total = 0.0
    for i, q in enumerate(grid):
        lo = -math.inf if i == 0 else 0.5 * (grid[i - 1] + q)
        hi = math.inf if i == len(grid) - 1 else 0.5 * (q + grid[i + 1])
        total += _cell_error(lo, hi, q)
    return total


def alpha_star_fp4() -> float:
    """argmin over alpha of gaussian_mse_fp4: the paper's alpha*_FP4, i.e. the definition of alpha*
    with the rounding step swapped for rounding to this grid (Sec. 4.4)."""
    result = minimize_scalar(gaussian_mse_fp4, bounds=(0.05, 8.0), method="bounded", options={"xatol": 1e-10})
    return float(result.x)


FP4_TRUST = 1.0 / 6.0   # largest half-interval of the scaled grid: (1 - 2/3) / 2, in units of alpha
