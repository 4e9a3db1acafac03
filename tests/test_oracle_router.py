"""Pins for the router stand-in (paper section 3.5).  Only the counts are printed by the paper."""
import numpy as np

from oracle import freqformer as O
from paper_2604_22808_amd import workloads as WL


def test_paper_router_counts():
    assert O.router_param_count(256, 128, 3) == 33283       # section 3.5
    assert O.router_flops(256, 128, 3) == 66304             # section 3.5
    assert 3 * O.ROUTER_DR + O.ROUTER_DT == 256


def test_apportionment():
    for nh in (1, 2, 3, 8, 16, 24):
        for pi in ([1 / 3, 1 / 3, 1 / 3], [0.7, 0.2, 0.1], [0.0, 0.0, 1.0], [0.5, 0.5, 0.0]):
            c = O.apportion_heads(pi, nh)
            assert c.sum() == nh and (c >= (1 if nh >= 3 else 0)).all()
    assert list(O.apportion_heads([0.7, 0.2, 0.1], 8)) == [5, 2, 1]       # 1 + LR(3.5, 1.0, 0.5) -> 1+(3+1), 1+1, 1+0
    assert list(O.apportion_heads([0.5, 0.5, 0.0], 4)) == [2, 1, 1]       # tie goes to the lower band
    assert list(O.route_fixed(8, 2, 3, 3)) == [1, 1, 2, 2, 2, 4, 4, 4]


def test_statistics_and_probabilities():
    grid, d = (4, 8, 8), 64
    rng = np.random.default_rng(0)
    q, k, v = (rng.standard_normal((1, 2, 256, d)) for _ in range(3))
    cfg = O.BandConfig(mid_block=16, mid_stride=4, high_window=32, n_summary=4)
    g = O.band_statistics(q, k, v, grid, cfg)
    assert g.shape == (192,)
    # white unit-variance input has the same mean energy in every band: centred logs vanish within sampling noise
    assert abs(g.sum()) < 1e-9 and np.abs(g.reshape(3, 64).mean(axis=1)).max() < 0.2
    # a common gain on the inputs adds the same constant to every log statistic, which the centring removes
    g10 = O.band_statistics(10 * q, 10 * k, 10 * v, grid, cfg)
    assert np.abs(g10 - g).max() < 1e-4
    # more energy in the low band only raises the low-band statistics relative to the others
    idx = O.band_partition(*grid, cfg)[0]
    from scipy.fft import dctn, idctn
    c = dctn(q.reshape(1, 2, 4, 8, 8, d), type=2, norm="ortho", axes=(2, 3, 4)).reshape(1, 2, 256, d)
    c[:, :, idx] *= 10
    qb = idctn(c.reshape(1, 2, 4, 8, 8, d), type=2, norm="ortho", axes=(2, 3, 4)).reshape(1, 2, 256, d)
    gb = O.band_statistics(qb, k, v, grid, cfg).reshape(3, 64).mean(axis=1)
    assert gb[0] > gb[1] + 1 and abs(gb[1] - gb[2]) < 0.3
    w1, b1, w2, b2 = WL.router_weights(64, 1)
    for t in (0.1, 0.5, 0.9):
        pi = O.router_probabilities(g, t, w1, b1, w2, b2)
        assert abs(pi.sum() - 1) < 1e-12 and (pi > 0).all()
    # zero weights leave only the timestep prior
    z = lambda t: O.router_probabilities(g, t, 0 * w1, b1, 0 * w2, b2)
    assert np.allclose(z(0.5), 1 / 3) and z(0.9)[0] > z(0.9)[1] > z(0.9)[2] and z(0.1)[2] > z(0.1)[0]
    e = O.timestep_embedding(0.0)
    assert np.allclose(e[:32], 0) and np.allclose(e[32:], 1)
