"""Pins for the band partition and the mid-band block pattern (paper sections 3.3, 3.4.2)."""
import numpy as np
import pytest

from oracle import freqformer as O

GRIDS = [(4, 8, 8), (16, 32, 32), (16, 64, 64), (3, 5, 7), (1, 1, 1), (2, 4, 4)]


def brute_bands(T, H, W, cfg):
    out = [[], [], []]
    for kt in range(T):
        for kh in range(H):
            for kw in range(W):
                flat = (kt * H + kh) * W + kw
                in_low = all(k * cfg.low_den < cfg.low_num * n for k, n in ((kt, T), (kh, H), (kw, W)))
                in_lm = all(k * cfg.mid_den < cfg.mid_num * n for k, n in ((kt, T), (kh, H), (kw, W)))
                out[0 if in_low else 1 if in_lm else 2].append(flat)
    return out


@pytest.mark.parametrize("grid", GRIDS)
def test_partition_is_disjoint_cover_and_matches_brute_force(grid):
    cfg = O.BandConfig()
    bands = O.band_partition(*grid, cfg)
    allidx = np.concatenate(bands)
    assert len(allidx) == np.prod(grid) and len(np.unique(allidx)) == np.prod(grid)
    for got, want in zip(bands, brute_bands(*grid, cfg)):
        assert got.dtype == np.int64 and list(got) == want       # ascending flat order, exact members


@pytest.mark.parametrize("grid", GRIDS)
def test_closed_form_counts(grid):
    T, H, W = grid
    c = lambda n, q: -(-n // q)
    n_low, n_mid, n_high = (len(b) for b in O.band_partition(T, H, W, O.BandConfig()))
    assert n_low == c(T, 4) * c(H, 4) * c(W, 4)
    assert n_low + n_mid == c(T, 2) * c(H, 2) * c(W, 2)
    assert n_low + n_mid + n_high == T * H * W


def test_benchmark_grid_counts():
    # power-of-two grids: N/64, 7N/64, 7N/8
    for grid in [(4, 8, 8), (16, 32, 32), (16, 64, 64), (64, 64, 64)]:
        N = int(np.prod(grid))
        assert [len(b) for b in O.band_partition(*grid, O.BandConfig())] == [N // 64, 7 * N // 64, 7 * N // 8]


def test_other_edges_and_r_is_max_norm():
    cfg = O.BandConfig(low_num=1, low_den=8, mid_num=3, mid_den=4)
    T, H, W = 8, 8, 8
    bands = O.band_partition(T, H, W, cfg)
    assert [list(b) for b in bands] == brute_bands(T, H, W, cfg)
    # (kt, kh, kw) = (0, 0, 6): r = 6/8 >= 3/4 -> high, although two axes are at DC
    assert 6 in bands[2] and (5 in bands[1])


def test_band_energies_sum_to_total():
    # section 5: the bands partition the transform domain, so band energies add up to ||x||^2
    rng = np.random.default_rng(3)
    T, H, W = 4, 8, 8
    x = rng.standard_normal((T, H, W, 5))
    c = O.spectral_forward(x).reshape(T * H * W, 5)
    parts = sum(np.sum(c[idx] ** 2) for idx in O.band_partition(T, H, W, O.BandConfig()))
    assert abs(parts - np.sum(x * x)) < 1e-10 * np.sum(x * x)


def test_mid_mask_rules():
    m = O.mid_block_mask(12, diag=1, stride=4, block0=1)
    for I in range(12):
        for J in range(12):
            want = abs(I - J) <= 1 or (I - J) % 4 == 0 or J == 0
            assert bool(m[I, J]) == want
    # relative stride: block (5, 1) is on, block (6, 4) is off (it would be on under an absolute stride)
    assert m[5, 1] and not m[6, 4]
    # no block0
    m0 = O.mid_block_mask(12, 1, 4, 0)
    assert not m0[6, 0] and m0[8, 0]
    # stride 1 is the all-ones mask
    assert O.mid_block_mask(7, 0, 1, 0).all()


@pytest.mark.parametrize("nb,d", [(1, 1), (5, 0), (9, 2), (28, 1), (224, 2)])
def test_diag_only_nnz_closed_form(nb, d):
    # stride larger than nb leaves only the diagonal band (and the main diagonal): nnz = (2d+1) nb - d (d+1)
    if d >= nb:
        pytest.skip("closed form needs d < nb")
    rp, ci = O.mid_block_csr(nb, d, stride=10 ** 6, block0=0)
    assert rp[-1] == (2 * d + 1) * nb - d * (d + 1) == len(ci)


def test_csr_agrees_with_mask_and_is_sorted():
    nb = 28
    m = O.mid_block_mask(nb, 1, 8, 1)
    rp, ci = O.mid_block_csr(nb, 1, 8, 1)
    assert rp.dtype == np.int32 and ci.dtype == np.int32 and rp[0] == 0
    for I in range(nb):
        cols = ci[rp[I]:rp[I + 1]]
        assert list(cols) == sorted(set(cols)) == list(np.nonzero(m[I])[0])
    assert rp[-1] == 177      # 16K benchmark configuration: 28 blocks, 177 active


def test_two_band_layouts_are_the_three_band_rule_with_an_empty_band():
    """Band count L = 2 (ablation list, section 8): mid edge == low edge empties the mid band, mid edge == 1 empties the
    high band; the partition still covers the grid, and a head allocated to the empty band changes nothing."""
    grid = (4, 8, 8)
    two = O.BandConfig(low_num=1, low_den=4, mid_num=1, mid_den=4, mid_block=16, mid_stride=4, high_window=32, n_summary=4)
    low, mid, high = O.band_partition(*grid, two)
    ref = O.band_partition(*grid, O.BandConfig())
    assert len(mid) == 0 and np.array_equal(low, ref[0])
    assert np.array_equal(high, np.sort(np.concatenate([ref[1], ref[2]])))
    no_high = O.BandConfig(low_num=1, low_den=4, mid_num=1, mid_den=1, mid_block=16, mid_stride=4, high_window=32, n_summary=4)
    low2, mid2, high2 = O.band_partition(*grid, no_high)
    assert len(high2) == 0 and len(low2) + len(mid2) == 256
    rng = np.random.default_rng(2)
    q, k, v = (rng.standard_normal((1, 1, 256, 8)) for _ in range(3))
    assert np.abs(O.forward(q, k, v, grid, two, [2]) - v).max() < 1e-10          # the empty band's operator is a no-op
    assert np.abs(O.forward(q, k, v, grid, two, [7]) - O.forward(q, k, v, grid, two, [5])).max() < 1e-12
    assert np.abs(O.forward(q, k, v, grid, two, [5]) - v).max() > 1e-3
    assert np.abs(O.forward(q, k, v, grid, no_high, [4]) - v).max() < 1e-10


def _cfg4(**kw):
    base = dict(low_num=1, low_den=4, mid_num=1, mid_den=2, mid2_num=3, mid2_den=4)
    base.update(kw)
    return O.BandConfig(**base)


@pytest.mark.parametrize("grid", [(4, 8, 8), (8, 12, 20), (16, 16, 16)])
def test_four_band_partition_brute_force_and_counts(grid):
    """Four bands (section 8's L = 4; the reading cuts the range between the mid edge and the new edge out of the high
    band): a triple loop over the max-norm rule, a disjoint cover, closed-form counts, public order low, mid, high, mid2."""
    T, H, W = grid
    cfg = _cfg4()
    bands = O.band_partition(T, H, W, cfg)
    assert len(bands) == 4
    want = [[], [], [], []]
    for kt in range(T):
        for kh in range(H):
            for kw in range(W):
                r = max(kt / T, kh / H, kw / W)
                l = 0 if r < 0.25 else 1 if r < 0.5 else 3 if r < 0.75 else 2
                want[l].append((kt * H + kh) * W + kw)
    for l in range(4):
        assert bands[l].tolist() == want[l]
    allidx = np.sort(np.concatenate(bands))
    assert np.array_equal(allidx, np.arange(T * H * W))
    box = lambda num, den: int(np.prod([-(-num * n // den) for n in grid]))
    assert [len(b) for b in bands] == [box(1, 4), box(1, 2) - box(1, 4), T * H * W - box(3, 4), box(3, 4) - box(1, 2)]


def test_four_band_layout_with_an_empty_fourth_band_is_the_three_band_layout():
    three = O.band_partition(8, 8, 16, O.BandConfig())
    four = O.band_partition(8, 8, 16, _cfg4(mid2_num=1, mid2_den=2))     # third edge on the mid edge: band 3 is empty
    assert len(four) == 4 and len(four[3]) == 0
    for a, b in zip(three, four[:3]):
        assert np.array_equal(a, b)
    four = O.band_partition(8, 8, 16, _cfg4(mid2_num=1, mid2_den=1))     # third edge at 1: the high band is empty
    assert len(four[2]) == 0 and np.array_equal(np.sort(np.concatenate([four[0], four[1], four[3]])), np.arange(8 * 8 * 16))
