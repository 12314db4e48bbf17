"""Pins for the AbsMax comparison quantizer (Sec. 4.1: the rotation-based baseline "with AbsMax
scaling instead of proper distribution matching").  The paper prints no formula for it, so the pins
are what the definition fixes: it is the RMS projection with the clip moved to the row's largest
magnitude, nothing is clipped, and on Gaussian rows it loses to the Gaussian-fitted clip."""
import math

import numpy as np
import pytest

from oracle import quest_oracle as qo

BITS = (1, 2, 3, 4, 8)


@pytest.mark.parametrize("bits", BITS)
def test_reduces_to_the_rms_projection_with_alpha_at_the_row_maximum(bits):
    rng = np.random.default_rng(bits)
    xh = rng.standard_normal((64, 256)) * np.exp(rng.uniform(-3, 3, size=(64, 1)))
    p = qo.project_absmax(xh, bits)
    for r in range(xh.shape[0]):
        rms = qo.row_rms(xh[r:r + 1])[0]
        amax = np.abs(xh[r]).max()
        ref = qo.project(xh[r:r + 1], bits, alpha=amax / rms)
        # the element that defines the maximum sits on the clip itself; a rounding of alpha * rms may
        # put it one ulp outside, which changes nothing but that element's trust bit
        assert np.array_equal(p.k[r], ref.k[0])
        assert np.allclose(p.xhat[r], ref.xhat[0], rtol=1e-13, atol=0)
        assert p.scale[r] == pytest.approx(ref.scale[0], rel=1e-14)
        assert p.rms[r] == amax


def test_hand_checked_two_bit_row():
    # a = 3, L = 4: grid -3, -1, 1, 3 with cells [-3,-2) [-2,0) [0,2) [2,3]; scale 1
    x = np.array([[3.0, -3.0, 0.0, -0.5, 1.999, 2.0, -2.0, -2.001]])
    p = qo.project_absmax(x, 2)
    assert p.k[0].tolist() == [1, -2, 0, -1, 0, 1, -1, -2]
    assert p.xhat[0].tolist() == [3.0, -3.0, 1.0, -1.0, 1.0, 3.0, -1.0, -3.0]
    assert p.scale[0] == 1.0
    assert np.all(p.trust == 1)


@pytest.mark.parametrize("bits", BITS)
def test_nothing_is_clipped_every_element_is_trusted_extremes_are_exact(bits):
    rng = np.random.default_rng(10 + bits)
    xh = rng.standard_t(3, size=(128, 512))
    p = qo.project_absmax(xh, bits)
    levels = 1 << bits
    amax = np.abs(xh).max(axis=1)
    assert np.all(np.abs(p.xhat - xh) <= amax[:, None] / (levels - 1) * (1 + 1e-12))
    assert np.all(p.trust == 1) and np.all(p.mask == 0xFF)
    top = np.argmax(np.abs(xh), axis=1)
    rows = np.arange(xh.shape[0])
    assert np.allclose(p.xhat[rows, top], xh[rows, top], rtol=1e-15)       # the maximum is a grid point
    assert np.all(np.abs(p.k[rows, top] * 2 + 1) == levels - 1)


def test_zero_row_and_scale_invariance():
    x = np.zeros((2, 64))
    x[1] = np.random.default_rng(0).standard_normal(64)
    p = qo.project_absmax(x, 4)
    assert np.all(p.k[0] == 0) and np.all(p.xhat[0] == 0) and np.all(p.trust[0] == 1) and p.scale[0] == 0
    p2 = qo.project_absmax(x * 8.0, 4)           # powers of two commute with every rounding
    assert np.array_equal(p.k, p2.k) and np.array_equal(p2.xhat, p.xhat * 8.0)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_gaussian_fitted_clip_beats_absmax_on_gaussian_rows(bits):
    """The mechanism behind the comparison of Sec. 4.1 / Table 1: with 2048 Gaussian values in a
    row the maximum is near 3.5 sigma, far beyond the MSE-optimal clip, and the grid is too coarse."""
    rng = np.random.default_rng(30 + bits)
    xh = rng.standard_normal((64, 2048))
    mse_absmax = np.mean((qo.project_absmax(xh, bits).xhat - xh) ** 2)
    mse_quest = np.mean((qo.project(xh, bits).xhat - xh) ** 2)
    assert mse_quest < 0.8 * mse_absmax


def test_no_transform_is_block_one():
    x = np.random.default_rng(3).standard_normal((8, 64)).astype(np.float32)
    p = qo.hadamard_quantize_absmax(x, 1, 4)
    assert np.array_equal(p.xh, x.astype(np.float64))
    q = qo.hadamard_quantize_absmax(x, 64, 4)
    assert np.allclose(np.sum(q.xh ** 2, axis=1), np.sum(x.astype(np.float64) ** 2, axis=1), rtol=1e-12)
