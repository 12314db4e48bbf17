"""Pins for the oracle's Hadamard transform (Sec. 3.1, Eq. 3): things the mathematics fixes."""
import numpy as np
import pytest
import scipy.linalg

from oracle import quest_oracle as qo


def test_small_matrices_match_the_textbook():
    assert qo.hadamard_matrix(1).tolist() == [[1]]
    assert qo.hadamard_matrix(2).tolist() == [[1, 1], [1, -1]]
    assert qo.hadamard_matrix(4).tolist() == [[1, 1, 1, 1], [1, -1, 1, -1],
                                              [1, 1, -1, -1], [1, -1, -1, 1]]


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048])
def test_h_ht_is_n_identity_exactly(n):
    h = qo.hadamard_matrix(n)
    assert set(np.unique(h)) == {-1, 1}
    assert np.array_equal(h @ h.T, n * np.eye(n, dtype=np.int64))
    assert np.array_equal(h, h.T)
    assert np.all(h[0] == 1) and np.all(h[:, 0] == 1)


@pytest.mark.parametrize("n", [2, 8, 64, 512])
def test_matrix_is_the_sylvester_construction(n):
    # scipy builds the Sylvester matrix by repeated Kronecker doubling: an independent routine.
    assert np.array_equal(qo.hadamard_matrix(n), scipy.linalg.hadamard(n).astype(np.int64))
    if n >= 4:
        half = qo.hadamard_matrix(n // 2)
        assert np.array_equal(qo.hadamard_matrix(n), np.kron(qo.hadamard_matrix(2), half))


@pytest.mark.parametrize("n", [1, 2, 16, 128, 512])
def test_dense_transform_is_the_matrix_product(n):
    rng = np.random.default_rng(n)
    x = rng.standard_normal((5, n))
    expect = x @ scipy.linalg.hadamard(n).astype(np.float64) / np.sqrt(n) if n > 1 else x
    assert np.allclose(qo.hadamard(x, n, dense=True), expect, rtol=0, atol=1e-12)


@pytest.mark.parametrize("n,cols", [(1, 24), (2, 8), (64, 192), (128, 1024), (512, 5632 // 11 * 2),
                                    (1024, 1024), (2048, 2048)])
def test_recursion_equals_dense_definition(n, cols):
    rng = np.random.default_rng(7 * n + cols)
    x = rng.standard_normal((3, cols))
    dense = qo.hadamard(x, n, dense=True)
    fast = qo.hadamard(x, n)
    assert np.allclose(fast, dense, rtol=0, atol=1e-11)


@pytest.mark.parametrize("n", [8, 256, 2048])
def test_unit_vectors_extract_columns(n):
    eye = np.eye(n)
    cols = qo.hadamard(eye, n) * np.sqrt(n)
    assert np.array_equal(np.rint(cols).astype(np.int64), qo.hadamard_matrix(n))
    assert np.allclose(cols, np.rint(cols), atol=1e-12)


@pytest.mark.parametrize("n,cols", [(128, 1024), (512, 5632), (2048, 2048)])
def test_orthonormal_involution_and_norm(n, cols):
    rng = np.random.default_rng(cols)
    x = rng.standard_normal((4, cols)) * 3.0
    xh = qo.hadamard(x, n)
    assert np.allclose(qo.hadamard(xh, n), x, rtol=0, atol=1e-11)          # IHT == HT
    assert np.allclose(np.linalg.norm(xh, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)
    assert np.allclose(qo.row_rms(xh), np.sqrt(np.mean(x * x, axis=1)), rtol=1e-12)


def test_blocks_are_independent():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 512))
    y = x.copy()
    y[:, 128:256] += 1.0                      # touch block 1 of 4 only
    dx = qo.hadamard(y, 128) - qo.hadamard(x, 128)
    assert np.all(dx[:, :128] == 0) and np.all(dx[:, 256:] == 0)
    assert np.any(dx[:, 128:256] != 0)


def test_constant_block_goes_to_first_coefficient():
    x = np.full((1, 64), 2.0)
    xh = qo.hadamard(x, 64)
    assert xh[0, 0] == pytest.approx(2.0 * 8.0) and np.all(xh[0, 1:] == 0)


def test_bf16_widening_is_exact():
    from paper_2502_05003_amd import synth
    rng = np.random.default_rng(0)
    f = rng.standard_normal(1000).astype(np.float32)
    bits = synth.to_bf16_bits(f)
    back = qo.widen(bits)
    assert np.array_equal(back.astype(np.float32).view(np.uint32) >> 16, bits.astype(np.uint32))
    assert np.max(np.abs(back - f) / np.abs(f)) <= 2.0 ** -8
    assert np.array_equal(qo.widen(f), f.astype(np.float64))
