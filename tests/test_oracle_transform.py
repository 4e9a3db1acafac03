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


# --------------------------------------------------------------------------- Haar variant (section 3.2: "wavelets are also possible")
def _haar_pyramid(x):
    """Textbook Haar analysis of a length-2^p vector: repeated pairwise (a+b)/sqrt2 averages and (a-b)/sqrt2 details,
    details of the finest level last; written as plain loops, independently of the matrix."""
    x = [float(t) for t in x]
    n = len(x)
    out = [0.0] * n
    while n > 1:
        half = n // 2
        avg = [(x[2 * i] + x[2 * i + 1]) / np.sqrt(2.0) for i in range(half)]
        det = [(x[2 * i] - x[2 * i + 1]) / np.sqrt(2.0) for i in range(half)]
        out[half:n] = det
        x = avg
        n = half
    out[0] = x[0]
    return np.array(out)


@pytest.mark.parametrize("n", [1, 2, 4, 16, 64, 128])
def test_haar_matrix_is_orthonormal(n):
    Wm = O.haar_matrix(n)
    assert np.abs(Wm @ Wm.T - np.eye(n)).max() < 1e-13
    assert np.abs(Wm.T @ Wm - np.eye(n)).max() < 1e-13


@pytest.mark.parametrize("n", [2, 8, 32, 128])
def test_haar_matrix_matches_pyramid_algorithm(n):
    rng = np.random.default_rng(n)
    for _ in range(3):
        x = rng.standard_normal(n)
        assert np.abs(O.haar_matrix(n) @ x - _haar_pyramid(x)).max() < 1e-12


def test_haar_closed_forms():
    n = 16
    Wm = O.haar_matrix(n)
    c = Wm @ np.full(n, 3.0)                    # constant -> scaling coefficient only
    assert abs(c[0] - 3.0 * np.sqrt(n)) < 1e-13 and np.abs(c[1:]).max() < 1e-13
    step = np.r_[np.ones(n // 2), -np.ones(n // 2)]   # a step at n/2 is the coarsest wavelet itself
    c = Wm @ step
    assert abs(c[1] - np.sqrt(n)) < 1e-13 and np.abs(np.delete(c, 1)).max() < 1e-13
    assert np.allclose(O.haar_matrix(2), np.array([[1, 1], [1, -1]]) / np.sqrt(2), atol=1e-15)
    with pytest.raises(ValueError):
        O.haar_matrix(12)


def test_haar_spectral_round_trip_and_parseval():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, 8, 16, 5))
    c = O.spectral_forward(x, transform=1)
    assert abs(np.sum(c ** 2) - np.sum(x ** 2)) < 1e-10 * np.sum(x ** 2)
    assert np.abs(O.spectral_inverse(c, transform=1) - x).max() < 1e-12
    # separable: one coefficient equals the triple product of matrix rows with the field
    Wt, Wh, Ww = O.haar_matrix(4), O.haar_matrix(8), O.haar_matrix(16)
    want = np.einsum("t,h,w,thwc->c", Wt[3], Wh[5], Ww[9], x)
    assert np.abs(c[3, 5, 9] - want).max() < 1e-12
    # and differs from the DCT
    assert np.abs(c - O.spectral_forward(x, transform=0)).max() > 1e-3


def test_haar_pipeline_identities():
    """With the Haar transform the pipeline keeps its invariants: no active band returns V, a one-hot mask changes
    only that band's coefficients."""
    rng = np.random.default_rng(8)
    grid, d = (4, 8, 8), 8
    cfg = O.BandConfig(mid_block=16, mid_diag=1, mid_stride=4, high_window=16, n_summary=4, transform=1)
    q, k, v = (rng.standard_normal(grid + (d,)) for _ in range(3))
    assert np.abs(O.head_forward(q, k, v, cfg, 0) - v).max() < 1e-12
    out = O.head_forward(q, k, v, cfg, 2)
    diff = O.spectral_forward(out - v, transform=1).reshape(-1, d)
    low, mid, high = O.band_partition(*grid, cfg)
    assert np.abs(diff[low]).max() < 1e-10 and np.abs(diff[high]).max() < 1e-10 and np.abs(diff[mid]).max() > 1e-4
