"""Pins for the projection and the trust mask (Eq. 1, Sec. 3.1, Sec. 3.2)."""
import math

import numpy as np
import pytest

from oracle import alpha_star as a
from oracle import quest_oracle as qo

BITS = (1, 2, 3, 4, 8)


def _brute_force_row(row, bits, alpha):
    """Eq. 1 written literally, one element at a time: clip, then nearest grid point."""
    levels = 1 << bits
    rms = math.sqrt(sum(v * v for v in row) / len(row))
    grid = [alpha * (2 * k + 1) / (levels - 1) for k in range(-levels // 2, levels // 2)]
    ks, xhat, trust = [], [], []
    for v in row:
        xn = v / rms
        clipped = min(max(xn, -alpha), alpha)
        best = min(range(levels), key=lambda i: (abs(grid[i] - clipped), -i))   # tie -> upper point
        ks.append(best - levels // 2)
        xhat.append(alpha * rms * (grid[best] / alpha))
        trust.append(1 if abs(xhat[-1] - v) <= (alpha / (levels - 1)) * rms else 0)
    return rms, ks, xhat, trust


@pytest.mark.parametrize("bits", BITS)
def test_projection_is_the_nearest_grid_point(bits, alpha_table):
    rng = np.random.default_rng(bits)
    x = rng.standard_normal((3, 64)) * np.array([[0.1], [1.0], [30.0]])
    x[1, :4] = [5.0, -5.0, 9.0, -9.0]                       # certainly clipped
    p = qo.project(x, bits, alpha_table[bits])
    for r in range(3):
        rms, ks, xhat, trust = _brute_force_row(list(x[r]), bits, alpha_table[bits])
        assert p.rms[r] == pytest.approx(rms, rel=1e-14)
        assert p.k[r].tolist() == ks
        assert np.allclose(p.xhat[r], xhat, rtol=1e-13)
        assert p.trust[r].tolist() == trust


def test_hand_checked_two_bit_vector():
    # b = 2, alpha = 1.5: grid in RMS units {-1.5, -0.5, 0.5, 1.5}, cells split at -1, 0, 1, T = 0.5.
    x = np.array([[2.0, -2.0, 0.25, -0.25, 0.99, 1.01, -1.0, 0.0,
                   1.9, 2.1, -1.99, -2.01, 1.0, -0.99, 3.0, -0.5]])
    x *= 1.0 / math.sqrt(np.mean(x * x))                    # unit RMS so x_n = x
    assert qo.row_rms(x)[0] == pytest.approx(1.0, rel=1e-15)
    xn = x[0]
    p = qo.project(x, 2, alpha=1.5)
    expect_k = [int(min(max(math.floor(v), -2), 1)) for v in xn]
    assert p.k[0].tolist() == expect_k
    assert np.allclose(p.xhat[0], [(2 * k + 1) * 0.5 for k in expect_k], rtol=1e-14)
    assert p.trust[0].tolist() == [1 if abs(v) <= 2.0 else 0 for v in xn]
    assert p.scale[0] == pytest.approx(0.5, rel=1e-15)


def test_boundary_values_go_to_the_upper_cell_and_zero_is_positive():
    # unit-RMS row whose entries sit exactly on cell boundaries (D = 1 at b = 2, alpha = 1.5)
    x = np.array([[1.0, -1.0, 1.0, -1.0, 0.0, 0.0, math.sqrt(2.0), -math.sqrt(2.0)]])
    assert qo.row_rms(x)[0] == pytest.approx(1.0, rel=1e-15)
    p = qo.project(x, 2, alpha=1.5)
    assert p.k[0, :6].tolist() == [1, -1, 1, -1, 0, 0]


@pytest.mark.parametrize("bits", BITS)
def test_error_bound_clipping_and_mask_invariants(bits, alpha_table):
    alpha = alpha_table[bits]
    levels = 1 << bits
    rng = np.random.default_rng(10 + bits)
    x = rng.standard_normal((64, 512))
    p = qo.project(x, bits, alpha)
    xn = x / p.rms[:, None]
    err_n = np.abs(p.xhat - x) / p.rms[:, None]
    T = alpha / (levels - 1)
    inside = np.abs(xn) <= alpha
    assert np.all(err_n[inside] <= T * (1 + 1e-12))                     # Sec. 3.2: error <= T below alpha
    assert np.all(p.trust[inside] == 1)
    assert np.all(p.k[xn > alpha] == levels // 2 - 1) and np.all(p.k[xn < -alpha] == -levels // 2)
    closed_form = (np.abs(xn) <= alpha * levels / (levels - 1)).astype(np.uint8)
    near_edge = np.abs(np.abs(xn) - alpha * levels / (levels - 1)) < 1e-12
    assert np.array_equal(p.trust[~near_edge], closed_form[~near_edge])
    assert np.allclose(p.xhat, p.scale[:, None] * (2 * p.k + 1), rtol=1e-14)
    assert np.allclose(p.scale, alpha * p.rms / (levels - 1), rtol=1e-15)
    if bits == 1:
        assert np.array_equal(p.trust, (np.abs(xn) <= 2 * alpha).astype(np.uint8))


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_mask_density_and_code_symmetry_on_gaussian_rows(bits, alpha_table):
    rng = np.random.default_rng(20 + bits)
    x = rng.standard_normal((256, 4096))
    p = qo.project(x, bits, alpha_table[bits])
    frac = 1.0 - p.trust.mean()
    expect = a.untrusted_fraction(alpha_table[bits], bits)
    sigma = math.sqrt(expect * (1 - expect) / x.size)
    assert abs(frac - expect) < 5 * sigma + 0.02 * expect     # rows are normalised by their own RMS
    levels = 1 << bits
    hist = np.bincount((p.k + levels // 2).ravel(), minlength=levels).astype(np.float64)
    assert np.all(np.abs(hist - hist[::-1]) <= 6 * np.sqrt(hist + hist[::-1]) + 1)


@pytest.mark.parametrize("bits", [1, 2, 4])
def test_alpha_star_minimises_the_empirical_error(bits, alpha_table):
    rng = np.random.default_rng(30 + bits)
    x = rng.standard_normal((1, 1 << 16))
    sweep = np.linspace(0.5 * alpha_table[bits], 1.6 * alpha_table[bits], 111)
    mse = [np.mean((qo.project(x, bits, float(s)).xhat - x) ** 2) for s in sweep]
    assert abs(sweep[int(np.argmin(mse))] - alpha_table[bits]) < 0.08 * alpha_table[bits]
    at_star = np.mean((qo.project(x, bits, alpha_table[bits]).xhat - x) ** 2)
    assert at_star == pytest.approx(a.gaussian_mse(alpha_table[bits], bits), rel=0.05)


def test_outer_trust_only_moves_the_outer_edge(alpha_table):
    alpha = alpha_table[1]
    rng = np.random.default_rng(5)
    x = rng.standard_normal((8, 1024))
    base = qo.project(x, 1, alpha, outer_trust=1.0)
    for ot in (0.0, 0.30, 0.769, 1.0, 2.0):
        p = qo.project(x, 1, alpha, outer_trust=ot)
        xn = x / p.rms[:, None]
        assert np.array_equal(p.k, base.k)
        assert np.all(p.trust[np.abs(xn) <= alpha] == 1)
        assert np.array_equal(p.trust, (np.abs(xn) <= alpha * (1 + ot)).astype(np.uint8))


def test_zero_row_and_scale_invariance(alpha_table):
    x = np.zeros((2, 64))
    x[1] = np.random.default_rng(1).standard_normal(64)
    p = qo.project(x, 4, alpha_table[4])
    assert p.rms[0] == 0 and p.scale[0] == 0 and np.all(p.k[0] == 0)
    assert np.all(p.xhat[0] == 0) and np.all(p.trust[0] == 1)
    q = qo.project(x * 1024.0, 4, alpha_table[4])           # power-of-two rescale: same codes and mask
    assert np.array_equal(p.k[1], q.k[1]) and np.array_equal(p.trust[1], q.trust[1])
    assert q.scale[1] == pytest.approx(1024.0 * p.scale[1], rel=1e-15)


def test_packing_layouts_byte_by_byte():
    k = np.array([[-8, -7, 0, 7, -1, 1, 3, -4]], dtype=np.int32)          # b = 4: c = k + 8
    from oracle.quest_oracle import _load, _ptr
    out = np.zeros((1, 4), dtype=np.uint8)
    _load().qo_pack_codes(_ptr(k), 1, 8, 4, _ptr(out))
    assert out[0].tolist() == [0x10, 0xF8, 0x97, 0x4B]                  # even element = low nibble
    assert qo.unpack_odd(out, 8, 4)[0].tolist() == (2 * k[0] + 1).tolist()
    k1 = np.array([[0, -1, -1, 0, 0, 0, -1, 0]], dtype=np.int32)         # b = 1: c = k + 1
    out1 = np.zeros((1, 1), dtype=np.uint8)
    _load().qo_pack_codes(_ptr(k1), 1, 8, 1, _ptr(out1))
    assert out1[0, 0] == 0b10111001
    k2 = np.array([[-2, -1, 0, 1, 1, 0, -1, -2]], dtype=np.int32)        # b = 2: c = k + 2
    out2 = np.zeros((1, 2), dtype=np.uint8)
    _load().qo_pack_codes(_ptr(k2), 1, 8, 2, _ptr(out2))
    assert out2[0].tolist() == [0b11100100, 0b00011011]
    k3 = np.array([[-4, 3, 0, -1, 2, -3, 1, -2]], dtype=np.int32)        # b = 3 in a nibble: c = k + 4
    out3 = np.zeros((1, 4), dtype=np.uint8)
    _load().qo_pack_codes(_ptr(k3), 1, 8, 3, _ptr(out3))
    assert out3[0].tolist() == [0x70, 0x34, 0x16, 0x25]
    assert qo.unpack_odd(out3, 8, 3)[0].tolist() == (2 * k3[0] + 1).tolist()
    k8 = np.array([[-128, 127, 0, -1, 5, 6, 7, 8]], dtype=np.int32)
    out8 = np.zeros((1, 8), dtype=np.uint8)
    _load().qo_pack_codes(_ptr(k8), 1, 8, 8, _ptr(out8))
    assert out8[0].tolist() == [0, 255, 128, 127, 133, 134, 135, 136]
    trust = np.array([[1, 0, 0, 1, 1, 1, 0, 1, 0, 0, 0, 0, 0, 0, 0, 1]], dtype=np.uint8)
    bm = np.zeros((1, 2), dtype=np.uint8)
    _load().qo_pack_mask(_ptr(trust), 1, 16, _ptr(bm))
    assert bm[0].tolist() == [0b10111001, 0b10000000]
    assert np.array_equal(qo.unpack_mask(bm, 16), trust)


@pytest.mark.parametrize("bits", BITS)
def test_exact_zero_is_trusted_at_any_scale(bits):
    """Sec. 3.2: M = 1[|xhat - x_h| <= T].  x_h = 0 (exact cancellation in the transform) sits on
    the boundary of cell 0; its error is exactly T, so it is trusted whatever the row's RMS is,
    also where T rms and xhat would round differently if written as different products."""
    rng = np.random.default_rng(bits)
    xh = rng.standard_normal((4000, 16)) * np.exp(rng.uniform(-8, 8, size=(4000, 1)))
    xh[:, 5] = 0.0
    p = qo.project(xh, bits)
    assert np.all(p.k[:, 5] == 0)
    assert np.all(p.trust[:, 5] == 1)
    # and through the transform: (1, 1) -> (sqrt 2, 0), (3, -3) -> (0, 3 sqrt 2), at random scales
    x = np.tile(np.array([1.0, 1.0, 3.0, -3.0]), (500, 4)) * np.exp(rng.uniform(-8, 8, size=(500, 1)))
    q = qo.hadamard_quantize(x.astype(np.float32), 2, bits)
    assert np.all(q.xh[:, 1::4] == 0.0) and np.all(q.xh[:, 2::4] == 0.0)
    assert np.all(q.trust[:, 1::4] == 1) and np.all(q.trust[:, 2::4] == 1)
