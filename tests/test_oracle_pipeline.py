"""Pins for the whole per-head path (paper sections 3.2-3.7) and the pair counter (section 4.2)."""
import numpy as np
import pytest

from oracle import freqformer as O

GRID = (4, 8, 8)
D = 8


def rand_head(seed, grid=GRID, d=D):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal(grid + (d,)) for _ in range(3)]


def cfg_tiny(**kw):
    base = dict(mid_block=16, mid_diag=1, mid_stride=4, mid_block0=1, high_window=32, n_summary=4)
    base.update(kw)
    return O.BandConfig(**base)


def test_no_active_band_returns_v():
    q, k, v = rand_head(0)
    assert np.abs(O.head_forward(q, k, v, cfg_tiny(), 0) - v).max() < 1e-10


@pytest.mark.parametrize("mask", [1, 2, 4, 3, 7])
def test_linear_in_v_without_exchange(mask):
    q, k, v1 = rand_head(1)
    v2 = rand_head(2)[2]
    cfg = cfg_tiny(n_summary=0)
    f = lambda v: O.head_forward(q, k, v, cfg, mask)
    assert np.abs(f(v1 + 2.5 * v2) - (f(v1) + 2.5 * f(v2))).max() < 1e-10


@pytest.mark.parametrize("mask,band", [(1, 0), (2, 1), (4, 2)])
def test_one_hot_mask_changes_only_its_band(mask, band):
    q, k, v = rand_head(3)
    cfg = cfg_tiny()
    diff = O.spectral_forward(O.head_forward(q, k, v, cfg, mask) - v).reshape(-1, D)
    bands = O.band_partition(*GRID, cfg)
    for l, idx in enumerate(bands):
        if l == band:
            assert np.abs(diff[idx]).max() > 1e-3
        else:
            assert np.abs(diff[idx]).max() < 1e-10


def test_full_pipeline_by_hand_from_parts():
    """Re-assemble the output from independently computed pieces (library DCT, per-band operators, explicit exchange)."""
    from scipy.fft import dctn, idctn
    q, k, v = rand_head(4)
    cfg = cfg_tiny()
    mask = 7
    scale = 1 / np.sqrt(D)
    N = int(np.prod(GRID))
    spec = lambda x: dctn(x, type=2, norm="ortho", axes=(0, 1, 2)).reshape(N, D)
    qs, ks, vs = spec(q), spec(k), spec(v)
    bands = O.band_partition(*GRID, cfg)
    Y = [O.low_band_attention(qs[bands[0]], ks[bands[0]], vs[bands[0]], 4, scale),
         O.mid_band_attention(qs[bands[1]], ks[bands[1]], vs[bands[1]], cfg, scale),
         O.high_band_attention(qs[bands[2]], ks[bands[2]], vs[bands[2]], 32, scale)]
    S = [O.summary_tokens(y, 4) for y in Y]
    full = np.zeros((N, D))
    for l in range(3):
        C = np.concatenate([S[o] for o in range(3) if o != l])
        full[bands[l]] = Y[l] + O.dense_attention(Y[l], C, C, scale)
    want = idctn(full.reshape(GRID + (D,)), type=2, norm="ortho", axes=(0, 1, 2))
    got, parts = O.head_forward(q, k, v, cfg, mask, return_parts=True)
    assert np.abs(got - want).max() < 1e-10
    # summaries come from pre-exchange outputs of all bands, also of inactive ones (pass-through V~)
    got2, parts2 = O.head_forward(q, k, v, cfg, 4, return_parts=True)
    assert np.abs(parts2["Y"][0] - vs[bands[0]]).max() < 1e-10 and np.abs(parts2["Yhat"][1] - vs[bands[1]]).max() < 1e-10
    C = np.concatenate([O.summary_tokens(vs[bands[0]], 4), O.summary_tokens(vs[bands[1]], 4)])
    assert np.abs(parts2["Yhat"][2] - (Y[2] + O.dense_attention(Y[2], C, C, scale))).max() < 1e-10


def test_exchange_off_equals_m0_and_scale_override():
    q, k, v = rand_head(5)
    a = O.head_forward(q, k, v, cfg_tiny(n_summary=0), 7)
    b = O.head_forward(q, k, v, cfg_tiny(n_summary=4), 7)
    assert np.abs(a - b).max() > 1e-4
    c = O.head_forward(q, k, v, cfg_tiny(softmax_scale=1 / np.sqrt(D)), 7)
    assert np.abs(b - c).max() < 1e-12


def test_heads_and_batches_are_independent():
    rng = np.random.default_rng(6)
    N = int(np.prod(GRID))
    q, k, v = (rng.standard_normal((2, 3, N, D)) for _ in range(3))
    cfg = cfg_tiny()
    alloc = np.array([1, 2, 4])
    out = O.forward(q, k, v, GRID, cfg, alloc)
    perm = [2, 0, 1]
    outp = O.forward(q[:, perm], k[:, perm], v[:, perm], GRID, cfg, alloc[perm])
    assert np.abs(outp - out[:, perm]).max() < 1e-12
    assert np.abs(O.forward(q[::-1], k[::-1], v[::-1], GRID, cfg, alloc) - out[::-1]).max() < 1e-12
    one = O.head_forward(*(x[1, 2].reshape(GRID + (D,)) for x in (q, k, v)), cfg, 4).reshape(N, D)
    assert np.abs(one - out[1, 2]).max() < 1e-12


def test_degenerate_parameters_collapse_to_dense_attention_per_band():
    """Section 5: with c = 1, the full pattern and w >= N_high every band runs exact dense attention on its band."""
    q, k, v = rand_head(7)
    cfg = cfg_tiny(low_compress=1, mid_stride=1, high_window=10 ** 6, n_summary=0)
    out, parts = O.head_forward(q, k, v, cfg, 7, return_parts=True)
    scale = 1 / np.sqrt(D)
    for l, idx in enumerate(parts["bands"]):
        want = O.dense_attention(parts["qs"][idx], parts["ks"][idx], parts["vs"][idx], scale)
        assert np.abs(parts["Y"][l] - want).max() < 1e-12


@pytest.mark.parametrize("grid,kw", [((4, 8, 8), dict(mid_block=16, mid_diag=1, mid_stride=4, high_window=32)),
                                     ((16, 32, 32), dict(mid_block=64, mid_diag=1, mid_stride=8, high_window=256))])
def test_interaction_count_closed_form(grid, kw):
    cfg = O.BandConfig(**kw)
    n_low, n_mid, n_high = (len(b) for b in O.band_partition(*grid, cfg))
    nbar = -(-n_low // 4)
    B = cfg.mid_block
    nb = -(-n_mid // B)
    rp, ci = O.mid_block_csr(nb, cfg.mid_diag, cfg.mid_stride, 1)
    size = lambda J: min(B, n_mid - J * B)
    mid = sum(size(I) * size(int(J)) for I in range(nb) for J in ci[rp[I]:rp[I + 1]])
    w = cfg.high_window
    # sum_i (min(i+w, n-1) - max(i-w, 0) + 1) = n (2w+1) - w (w+1) when n > 2 w, else n^2 if w >= n - 1
    high = n_high * (2 * w + 1) - w * (w + 1) if n_high > 2 * w else None
    total = O.interaction_count(*grid, cfg, 7)
    if high is not None:
        assert total == nbar * nbar + mid + high
    assert O.interaction_count(*grid, cfg, 1) == nbar * nbar
    assert O.interaction_count(*grid, cfg, 2) == mid
    if grid == (16, 32, 32):   # 16K configuration: 64^2 low pairs, 177 full blocks, window average 508.4
        assert nbar == 64 and mid == 177 * 64 * 64 and abs((total - 4096 - mid) / n_high - 508.4) < 0.05


def test_projected_forward_pins():
    """Sections 3.1 / 3.7 around the path: (a) the transform commutes with a channel projection, F(X W) = F(X) W, which
    is what lets X be transformed once; (b) identity weights reduce the projected forward to the plain one on channel
    slices; (c) with no active band it is X W_V W_O; (d) per-head loops over explicitly sliced weights give the same."""
    grid, nh, d = (4, 8, 8), 3, 8
    N, dm = 256, 24
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, N, dm))
    wq, wk, wv = (rng.standard_normal((dm, nh * d)) / np.sqrt(dm) for _ in range(3))
    wo = rng.standard_normal((nh * d, dm)) / np.sqrt(nh * d)
    cfg = O.BandConfig(mid_block=16, mid_stride=4, high_window=32, n_summary=4)
    # (a)
    xs = O.spectral_forward(x[0].reshape(*grid, dm))
    assert np.abs(O.spectral_forward((x[0] @ wq).reshape(*grid, nh * d)) - xs @ wq).max() < 1e-10
    # (b)
    eye = np.eye(dm)
    alloc = (1, 6, 7)
    got = O.forward_projected(x, eye, eye, eye, eye, grid, cfg, alloc)
    heads = x.reshape(2, N, nh, d).transpose(0, 2, 1, 3)
    want = O.forward(heads, heads, heads, grid, cfg, alloc).transpose(0, 2, 1, 3).reshape(2, N, dm)
    assert np.abs(got - want).max() < 1e-12
    # (c)
    assert np.abs(O.forward_projected(x, wq, wk, wv, wo, grid, cfg, (0, 0, 0)) - x @ wv @ wo).max() < 1e-10
    # (d)
    got = O.forward_projected(x, wq, wk, wv, wo, grid, cfg, alloc)
    want = np.zeros((2, N, dm))
    for b in range(2):
        for h in range(nh):
            sl = slice(h * d, (h + 1) * d)
            f = lambda w: (x[b] @ w[:, sl]).reshape(*grid, d)
            want[b] += O.head_forward(f(wq), f(wk), f(wv), cfg, alloc[h]).reshape(N, d) @ wo[sl]
    assert np.abs(got - want).max() < 1e-10
    assert np.abs(got - x @ wv @ wo).max() > 1e-3


def cfg_four(**kw):
    return cfg_tiny(mid2_num=3, mid2_den=4, **kw)


def test_four_band_pipeline_by_hand_from_parts():
    """Four bands (the L = 4 of section 8): the output re-assembled from independently computed pieces - library DCT,
    the band operators (the block-sparse one on both middle bands), the exchange against the 3 m summary tokens of the
    other three bands - for all bands active and for a head that runs the second middle band alone."""
    from scipy.fft import dctn, idctn
    grid = (4, 8, 16)
    q, k, v = rand_head(14, grid=grid)
    cfg = cfg_four()
    scale = 1 / np.sqrt(D)
    N = int(np.prod(grid))
    spec = lambda x: dctn(x, type=2, norm="ortho", axes=(0, 1, 2)).reshape(N, D)
    qs, ks, vs = spec(q), spec(k), spec(v)
    bands = O.band_partition(*grid, cfg)
    assert [len(b) for b in bands] == [8, 56, 296, 152]     # 2*... boxes 1/4, 1/2, 3/4 of (4, 8, 16): 8, 64, 216 coefficients
    op = [lambda i: O.low_band_attention(qs[i], ks[i], vs[i], 4, scale),
          lambda i: O.mid_band_attention(qs[i], ks[i], vs[i], cfg, scale),
          lambda i: O.high_band_attention(qs[i], ks[i], vs[i], 32, scale),
          lambda i: O.mid_band_attention(qs[i], ks[i], vs[i], cfg, scale)]
    for mask in (15, 8, 9):
        Y = [op[l](bands[l]) if (mask >> l) & 1 else vs[bands[l]] for l in range(4)]
        S = [O.summary_tokens(y, 4) for y in Y]
        full = np.zeros((N, D))
        for l in range(4):
            if (mask >> l) & 1:
                C = np.concatenate([S[o] for o in range(4) if o != l])
                assert C.shape[0] == 12
                full[bands[l]] = Y[l] + O.dense_attention(Y[l], C, C, scale)
            else:
                full[bands[l]] = Y[l]
        want = idctn(full.reshape(grid + (D,)), type=2, norm="ortho", axes=(0, 1, 2))
        got = O.head_forward(q, k, v, cfg, mask)
        assert np.abs(got - want).max() < 1e-10, mask


def test_four_band_layout_with_an_empty_band_equals_three_bands():
    q, k, v = rand_head(15)
    three = O.head_forward(q, k, v, cfg_tiny(), 7)
    four = O.head_forward(q, k, v, cfg_tiny(mid2_num=1, mid2_den=2), 7 | 8)    # band 3 empty: its bit changes nothing
    assert np.abs(three - four).max() < 1e-12
    # the second middle band covering everything outside the mid edge, window wide enough to be dense, one block: both are
    # dense attention over the same rows
    a = O.head_forward(q, k, v, cfg_tiny(high_window=10**6, n_summary=0), 4)
    b = O.head_forward(q, k, v, cfg_tiny(mid2_num=1, mid2_den=1, mid_block=10**6, n_summary=0), 8)
    assert np.abs(a - b).max() < 1e-10


def test_four_band_interaction_count():
    cfg = cfg_four()
    n = [len(b) for b in O.band_partition(4, 8, 16, cfg)]
    both = O.interaction_count(4, 8, 16, cfg, mask=2 | 8)
    assert both == O.interaction_count(4, 8, 16, cfg, mask=2) + O.interaction_count(4, 8, 16, cfg, mask=8)
    nb = -(-n[3] // 16)                                  # 152 rows: nine full blocks of 16 and one of 8
    m = O.mid_block_mask(nb, 1, 4, 1)
    size = np.array([16] * 9 + [8])
    assert n[3] == 152 and O.interaction_count(4, 8, 16, cfg, mask=8) == int((m * np.outer(size, size)).sum())
