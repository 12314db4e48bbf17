"""Pins for the FP4 variant (Sec. 4.4, "The FP4 Format"): rounding to the E2M1 grid scaled to
[-1, 1], alpha*_FP4 from the same Gaussian-fit definition, T = largest half-interval of the grid."""
import math

import numpy as np
import pytest

from oracle import alpha_star as a
from oracle import quest_oracle as qo

MAG = np.array(a.FP4_MAGNITUDES)


def test_grid_is_the_e2m1_value_set_scaled_to_one():
    # E2M1: exponent field e (bias 1), mantissa bit m: e = 0 -> m / 2, else 2^(e-1) (1 + m / 2)
    values = sorted({(mm / 2.0) if e == 0 else 2.0 ** (e - 1) * (1 + mm / 2.0) for e in range(4) for mm in range(2)})
    assert values == list(a.FP4_MAGNITUDES)
    g = a.fp4_grid()
    assert len(g) == 15 and g[0] == -1.0 and g[-1] == 1.0 and g[7] == 0.0
    gaps = np.diff(g)
    assert gaps.max() / 2 == pytest.approx(a.FP4_TRUST) and a.FP4_TRUST == pytest.approx(1 / 6)


def test_projection_is_the_nearest_grid_point():
    rng = np.random.default_rng(0)
    xh = rng.standard_normal((32, 256)) * np.exp(rng.uniform(-3, 3, size=(32, 1)))
    alpha = 2.5
    p = qo.project_fp4(xh, alpha)
    grid = np.array(a.fp4_grid())
    for r in range(xh.shape[0]):
        rms = math.sqrt(np.mean(xh[r] ** 2))
        assert p.rms[r] == pytest.approx(rms, rel=1e-14)
        clipped = np.clip(xh[r] / rms / alpha, -1.0, 1.0)
        nearest = grid[np.argmin(np.abs(clipped[:, None] - grid[None, :]), axis=1)]   # no exact ties in random data
        assert np.allclose(p.xhat[r], alpha * rms * nearest, rtol=1e-13, atol=1e-300)
        assert p.scale[r] == pytest.approx(alpha * rms / 6, rel=1e-14)
    assert np.allclose(p.xhat, p.scale[:, None] * p.value, rtol=1e-13)
    assert np.array_equal(p.value, np.where(p.code & 8, -1.0, 1.0) * MAG[p.code & 7])


def test_hand_checked_row_with_ties_and_signed_zero():
    # 64 entries whose squares sum to 256: rms = 2 exactly; alpha = 3 makes t = 6 x_n / alpha = x with no
    # rounding (x / 2 and 3 x are exact).  Grid magnitudes 0 .5 1 1.5 2 3 4 6 are codes 0..7.
    head = [0.0, 0.25, -0.25, 0.5, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -5.0, 5.5, 12.0, -0.125, 2.0, 1.875, 0.375, 0.125]
    x = np.zeros((1, 64))
    x[0, :len(head)] = head
    assert np.sum(x ** 2) == 256.0
    p = qo.project_fp4(x, alpha=3.0)
    assert p.rms[0] == 2.0 and p.scale[0] == 1.0
    # ties go to the even code: .25 -> 0, .75 -> 1.0, 1.25 -> 1.0, 1.75 -> 2, 2.5 -> 2, 3.5 -> 4, 5 -> 4
    assert p.code[0, :18].tolist() == [0, 0, 8, 1, 2, 2, 4, 4, 6, 6, 14, 7, 7, 8, 4, 4, 1, 0]
    assert p.value[0, :18].tolist() == [0, 0, -0.0, 0.5, 1, 1, 2, 2, 4, 4, -4, 6, 6, -0.0, 2, 2, 0.5, 0]
    assert np.array_equal(p.xhat[0, :18], p.value[0, :18])
    # everything inside the clip range is trusted; 12 lies beyond alpha (1 + 1/6) rms = 7
    assert p.trust[0, :12].tolist() == [1] * 12 and p.trust[0, 12] == 0 and np.all(p.trust[0, 13:] == 1)
    assert p.codes[0, 0] == 0x00 and p.codes[0, 1] == (8 | (1 << 4))      # low nibble first


def test_error_bounds_and_trust_edge():
    rng = np.random.default_rng(1)
    xh = rng.standard_t(3, size=(64, 512))
    alpha = a.alpha_star_fp4()
    p = qo.project_fp4(xh)
    assert p.alpha == alpha
    xn = xh / p.rms[:, None]
    inside = np.abs(xn) <= alpha
    assert np.all(np.abs(p.xhat - xh)[inside] <= (alpha / 6) * np.broadcast_to(p.rms[:, None], xh.shape)[inside] * (1 + 1e-12))
    assert np.all(p.trust[inside] == 1)
    edge = alpha * (1 + 1 / 6)
    assert np.array_equal(p.trust == 1, np.abs(xn) <= edge) or np.all(np.abs(np.abs(xn[(p.trust == 1) != (np.abs(xn) <= edge)]) - edge) < 1e-12)
    assert np.all(np.abs(p.value[np.abs(xn) > alpha]) == 6.0)


def test_alpha_star_fp4_minimises_the_closed_form_and_the_empirical_error():
    alpha = a.alpha_star_fp4()
    sweep = np.linspace(1.5, 4.5, 3001)
    errs = np.array([a.gaussian_mse_fp4(v) for v in sweep])
    assert abs(sweep[np.argmin(errs)] - alpha) <= 2e-3
    rng = np.random.default_rng(2)
    xi = rng.standard_normal(2_000_000)
    grid = np.array(a.fp4_grid())

    def empirical(al):
        c = np.clip(xi / al, -1, 1)
        idx = np.searchsorted((grid[:-1] + grid[1:]) / 2, c)
        return np.mean((xi - al * grid[idx]) ** 2)

    assert empirical(alpha) == pytest.approx(a.gaussian_mse_fp4(alpha), rel=5e-3)
    assert empirical(alpha) < empirical(0.9 * alpha) and empirical(alpha) < empirical(1.1 * alpha)


def test_fp4_fits_a_gaussian_worse_than_int4_when_clipping_is_allowed():
    """The paper's explanation of FP4's lower parameter efficiency (Sec. 4.4, last sentence)."""
    mse_fp4 = a.gaussian_mse_fp4(a.alpha_star_fp4())
    mse_int4 = a.gaussian_mse(a.alpha_star(4), 4)
    assert mse_fp4 > mse_int4
    assert mse_fp4 == pytest.approx(0.012685, rel=1e-3) and mse_int4 == pytest.approx(0.011543, rel=1e-3)


def test_zero_row_scale_invariance_and_gemm_exactness():
    x = np.zeros((2, 64))
    x[1] = np.random.default_rng(3).standard_normal(64)
    p = qo.project_fp4(x)
    assert np.all(p.code[0] == 0) and np.all(p.trust[0] == 1) and p.scale[0] == 0
    p2 = qo.project_fp4(x * 4.0)
    assert np.array_equal(p.code, p2.code) and np.array_equal(p2.xhat, 4.0 * p.xhat)
    va = qo.unpack_fp4(p.codes, 64)
    acc = qo.gemm_fp4(va, va)
    assert acc[1, 1] == np.sum(va[1] ** 2) and np.all(acc * 4 == np.rint(acc * 4))


def test_gemm_fp4_is_the_plain_sum_of_products():
    """The FP4 accumulator oracle against Python loops on a tiny case, and against the integer
    product on doubled values: 2 v is an integer, so acc = sum (2 v_a)(2 v_b) / 4 exactly."""
    rng = np.random.default_rng(4)
    code_a = rng.integers(0, 16, size=(5, 24), dtype=np.uint8)
    code_b = rng.integers(0, 16, size=(7, 24), dtype=np.uint8)
    va = np.where(code_a & 8, -1.0, 1.0) * MAG[code_a & 7]
    vb = np.where(code_b & 8, -1.0, 1.0) * MAG[code_b & 7]
    acc = qo.gemm_fp4(va, vb)
    assert acc.shape == (5, 7)
    for m in range(5):
        for n in range(7):
            total = 0.0
            for k in range(24):
                total += float(va[m, k]) * float(vb[n, k])
            assert acc[m, n] == total
    # a transposed operand, a dropped term or a wrong sign would break one of these
    assert not np.array_equal(acc, qo.gemm_fp4(va, -vb)) and np.array_equal(acc, -qo.gemm_fp4(va, -vb))
    va_big = np.where(rng.integers(0, 2, size=(33, 512)), -1.0, 1.0) * MAG[rng.integers(0, 8, size=(33, 512))]
    vb_big = np.where(rng.integers(0, 2, size=(17, 512)), -1.0, 1.0) * MAG[rng.integers(0, 8, size=(17, 512))]
    doubled = qo.gemm_odd((2 * va_big).astype(np.int32), (2 * vb_big).astype(np.int32))
    assert np.array_equal(qo.gemm_fp4(va_big, vb_big) * 4.0, doubled.astype(np.float64))
    one_hot = np.zeros((1, 512)); one_hot[0, 37] = 1.0
    assert np.array_equal(qo.gemm_fp4(one_hot, vb_big)[0], vb_big[:, 37])
