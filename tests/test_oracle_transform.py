"""Pins for the oracle's spectral transform (paper section 3.2, orthonormality used in section 5)."""
import numpy as np
import pytest
from scipy.fft import dctn, idctn

from oracle import freqformer as O


@pytest.mark.parametrize("n", [1, 2, 3, 4, 8, 16, 31, 64, 128])
def test_dct_matrix_is_orthonormal(n):
    F = O.dct_matrix(n)
    assert np.abs(F @ F.T - np.eye(n)).max() < 1e-12
    assert np.abs(F.T @ F - np.eye(n)).max() < 1e-12


def test_dct_matrix_matches_library_routine():
    # rows are frequencies: F @ x must be scipy's orthonormal DCT-II of x (a transposed matrix would fail)
    rng = np.random.default_rng(0)
    for n in (5, 8, 32):
        x = rng.standard_normal(n)
        assert np.abs(O.dct_matrix(n) @ x - dctn(x, type=2, norm="ortho")).max() < 1e-12


def test_dct_matrix_closed_forms():
    # n = 2: [[1, 1], [1, -1]] / sqrt(2); DC row is 1/sqrt(n); first AC row of n = 4 by hand
    assert np.allclose(O.dct_matrix(2), np.array([[1, 1], [1, -1]]) / np.sqrt(2), atol=1e-15)
    assert np.allclose(O.dct_matrix(7)[0], 1 / np.sqrt(7), atol=1e-15)
    row1 = np.sqrt(2 / 4) * np.cos(np.pi * np.array([1, 3, 5, 7]) / 8)
    assert np.allclose(O.dct_matrix(4)[1], row1, atol=1e-15)


@pytest.mark.parametrize("shape", [(4, 8, 8, 3), (3, 5, 7, 2), (16, 32, 32, 4)])
def test_forward_matches_scipy_and_round_trips(shape):
    rng = np.random.default_rng(1)
    x = rng.standard_normal(shape)
    c = O.spectral_forward(x)
    assert np.abs(c - dctn(x, type=2, norm="ortho", axes=(0, 1, 2))).max() < 1e-10
    assert np.abs(O.spectral_inverse(c) - x).max() < 1e-10
    assert np.abs(O.spectral_inverse(x) - idctn(x, type=2, norm="ortho", axes=(0, 1, 2))).max() < 1e-10
    # Parseval (section 5)
    assert abs(np.sum(c * c) - np.sum(x * x)) < 1e-10 * np.sum(x * x)


def test_axes_are_not_mixed_up():
    # a field varying only along H must have coefficients only on the k_h axis (k_t = k_w = 0)
    T, H, W = 4, 8, 16
    x = np.zeros((T, H, W, 1))
    x[:, :, :, 0] = np.cos(np.pi * (2 * np.arange(H) + 1) * 3 / (2 * H))[None, :, None]
    c = O.spectral_forward(x)[..., 0]
    expect = np.zeros((T, H, W))
    expect[0, 3, 0] = np.sqrt(T * W) * np.sqrt(H / 2)
    assert np.abs(c - expect).max() < 1e-10


def test_constant_field_is_pure_dc_and_basis_vector_is_one_hot():
    T, H, W = 4, 8, 8
    x = np.full((T, H, W, 2), 0.75)
    c = O.spectral_forward(x)
    e = np.zeros_like(c)
    e[0, 0, 0, :] = 0.75 * np.sqrt(T * H * W)
    assert np.abs(c - e).max() < 1e-12
    onehot = np.zeros((T, H, W, 1))
    onehot[2, 5, 1, 0] = 1.0
    basis = O.spectral_inverse(onehot)
    assert np.abs(O.spectral_forward(basis) - onehot).max() < 1e-12
    # channels are untouched: transforming channel by channel gives the same result
    y = np.random.default_rng(2).standard_normal((T, H, W, 3))
    cy = O.spectral_forward(y)
    for ch in range(3):
        assert np.abs(cy[..., ch:ch + 1] - O.spectral_forward(y[..., ch:ch + 1])).max() < 1e-12
