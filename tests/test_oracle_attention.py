"""Pins for the three band operators and the exchange (paper sections 3.3, 3.4, 3.6)."""
import math

import numpy as np
import pytest

from oracle import freqformer as O


def brute_attention(Q, K, V, scale, allowed):
    """Per-row loops over an explicit key set: the definition, with nothing vectorised."""
    n, d = Q.shape
    Y = np.zeros((n, V.shape[1]))
    for i in range(n):
        keys = [j for j in range(K.shape[0]) if allowed(i, j)]
        s = [scale * sum(Q[i, c] * K[j, c] for c in range(d)) for j in keys]
        mx = max(s)
        w = [math.exp(x - mx) for x in s]
        z = sum(w)
        for wj, j in zip(w, keys):
            Y[i] += (wj / z) * V[j]
    return Y


def rand_qkv(n, d, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d))


def test_dense_attention_matches_definition():
    Q, K, V = rand_qkv(19, 6, 0)
    assert np.abs(O.dense_attention(Q, K, V, 0.4) - brute_attention(Q, K, V, 0.4, lambda i, j: True)).max() < 1e-12
    # K = 0 gives uniform weights: every row is the mean of V
    assert np.abs(O.dense_attention(Q, 0 * K, V, 1.0) - V.mean(axis=0)).max() < 1e-12


# ------------------------------------------------------------------ low band
def test_low_no_compression_is_dense():
    Q, K, V = rand_qkv(24, 8, 1)
    assert np.abs(O.low_band_attention(Q, K, V, 1, 0.3) - O.dense_attention(Q, K, V, 0.3)).max() < 1e-12


def test_low_single_group_returns_mean_of_v():
    Q, K, V = rand_qkv(4, 8, 2)
    Y = O.low_band_attention(Q, K, V, 4, 0.3)
    assert np.abs(Y - V.mean(axis=0)).max() < 1e-14


def test_low_compression_by_hand_with_ragged_tail():
    # 10 tokens, c = 4 -> groups {0..3}, {4..7}, {8, 9}; output row i is the group's output
    Q, K, V = rand_qkv(10, 5, 3)
    groups = [range(0, 4), range(4, 8), range(8, 10)]
    pool = lambda X: np.stack([np.mean([X[i] for i in g], axis=0) for g in groups])
    assert np.abs(O.compress_tokens(K, 4) - pool(K)).max() < 1e-14
    Ybar = brute_attention(pool(Q), pool(K), pool(V), 0.5, lambda i, j: True)
    Y = O.low_band_attention(Q, K, V, 4, 0.5)
    for gi, g in enumerate(groups):
        for i in g:
            assert np.abs(Y[i] - Ybar[gi]).max() < 1e-12


# ------------------------------------------------------------------ mid band
def test_mid_all_ones_mask_is_dense():
    Q, K, V = rand_qkv(28, 8, 4)
    cfg = O.BandConfig(mid_block=16, mid_diag=0, mid_stride=1, mid_block0=0)
    assert np.abs(O.mid_band_attention(Q, K, V, cfg, 0.35) - O.dense_attention(Q, K, V, 0.35)).max() < 1e-12


@pytest.mark.parametrize("n,B,diag,stride,block0", [(28, 16, 1, 4, 1), (50, 4, 1, 4, 1), (37, 5, 0, 3, 0), (64, 8, 2, 5, 1)])
def test_mid_matches_per_row_brute_force(n, B, diag, stride, block0):
    Q, K, V = rand_qkv(n, 4, 5)
    cfg = O.BandConfig(mid_block=B, mid_diag=diag, mid_stride=stride, mid_block0=block0)

    def allowed(i, j):
        I, J = i // B, j // B
        return abs(I - J) <= diag or (I - J) % stride == 0 or (block0 and J == 0)

    assert np.abs(O.mid_band_attention(Q, K, V, cfg, 0.5) - brute_attention(Q, K, V, 0.5, allowed)).max() < 1e-12


# ------------------------------------------------------------------ high band
def test_high_wide_window_is_dense_and_zero_window_is_identity():
    Q, K, V = rand_qkv(40, 8, 6)
    assert np.abs(O.high_band_attention(Q, K, V, 40, 0.3) - O.dense_attention(Q, K, V, 0.3)).max() < 1e-12
    assert np.abs(O.high_band_attention(Q, K, V, 10 ** 6, 0.3, chunk=7) - O.dense_attention(Q, K, V, 0.3)).max() < 1e-12
    assert np.abs(O.high_band_attention(Q, K, V, 0, 0.3) - V).max() < 1e-15


@pytest.mark.parametrize("n,w,chunk", [(45, 3, 256), (45, 3, 4), (100, 17, 16), (9, 32, 256)])
def test_high_matches_per_row_brute_force(n, w, chunk):
    Q, K, V = rand_qkv(n, 4, 7)
    want = brute_attention(Q, K, V, 0.5, lambda i, j: abs(i - j) <= w)
    assert np.abs(O.high_band_attention(Q, K, V, w, 0.5, chunk=chunk) - want).max() < 1e-12


def test_window_is_two_sided():
    # a causal (one-sided) window would ignore keys after the query: put all the value mass there
    n = 12
    Q = np.zeros((n, 2)); K = np.zeros((n, 2)); V = np.zeros((n, 1)); V[5, 0] = 1.0
    Y = O.high_band_attention(Q, K, V, 2, 1.0)
    assert Y[3, 0] == pytest.approx(1 / 5) and Y[7, 0] == pytest.approx(1 / 5) and Y[2, 0] == 0 and Y[8, 0] == 0
    assert Y[0, 0] == 0 and Y[4, 0] == pytest.approx(1 / 5)


# ------------------------------------------------------------------ summaries and exchange
def test_summary_chunks():
    Y = np.arange(10, dtype=np.float64)[:, None] * np.ones((1, 3))
    S = O.summary_tokens(Y, 4)     # bounds 0, 2, 5, 7, 10
    assert np.allclose(S[:, 0], [0.5, 3.0, 5.5, 8.0])
    assert np.allclose(O.summary_tokens(Y, 16), Y)          # m > n: one token per summary
    assert np.allclose(O.summary_tokens(Y, 1)[0], Y.mean(axis=0))
    # the weighted mean of the summaries is the mean of the band
    n, m = 37, 5
    Z = np.random.default_rng(8).standard_normal((n, 2))
    sizes = np.diff([(u * n) // m for u in range(m + 1)])
    assert np.allclose((O.summary_tokens(Z, m) * sizes[:, None]).sum(axis=0) / n, Z.mean(axis=0))


def test_exchange_invariants():
    rng = np.random.default_rng(9)
    Y = rng.standard_normal((30, 6)); C = rng.standard_normal((8, 6))
    D = O.cross_band_exchange(Y, C, 0.4)
    assert np.all(D <= C.max(axis=0) + 1e-12) and np.all(D >= C.min(axis=0) - 1e-12)     # convex hull of C's rows
    assert np.abs(O.cross_band_exchange(Y, C[rng.permutation(8)], 0.4) - D).max() < 1e-12  # order of C is immaterial
    assert np.abs(D - brute_attention(Y, C, C, 0.4, lambda i, j: True)).max() < 1e-12
    # one summary token: delta is that token for every query
    assert np.abs(O.cross_band_exchange(Y, C[:1], 0.4) - C[0]).max() < 1e-14
