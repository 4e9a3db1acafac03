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


# ---- pins written as explicit scalar loops, independent of the oracle's vector code ----------------------------
def _loop_embedding(t):
    """Section 3.5 reading: e(t)[i] = sin(1000 t / 10000^(2i/64)), e(t)[32 + i] = cos(same angle), i = 0..31."""
    e = [0.0] * 64
    for i in range(32):
        ang = 1000.0 * t / (10000.0 ** (2.0 * i / 64.0))
        e[i] = np.sin(ang)
        e[32 + i] = np.cos(ang)
    return e


def test_timestep_embedding_hand_angles():
    t = 0.37
    e = O.timestep_embedding(t)
    assert e.shape == (64,)
    # i = 0: angle 1000 t = 370; i = 16: 10000^(-2*16/64) = 10000^(-1/2) = 0.01 -> angle 3.7; i = 31: 10000^(-31/32)
    assert abs(e[0] - np.sin(370.0)) < 1e-12 and abs(e[32] - np.cos(370.0)) < 1e-12
    assert abs(e[16] - np.sin(3.7)) < 1e-12 and abs(e[48] - np.cos(3.7)) < 1e-12
    a31 = 370.0 * 10000.0 ** (-31.0 / 32.0)
    assert abs(e[31] - np.sin(a31)) < 1e-12 and abs(e[63] - np.cos(a31)) < 1e-12
    assert np.abs(e - np.array(_loop_embedding(t))).max() < 1e-12
    # a different frequency base or a sin/cos swap moves these entries by O(1)
    assert abs(np.sin(3.7) - np.sin(370.0 * 1000.0 ** (-0.5))) > 0.1 and abs(np.sin(3.7) - np.cos(3.7)) > 0.1


def test_router_probabilities_scalar_loops():
    rng = np.random.default_rng(7)
    hidden = 24
    g = rng.standard_normal(192)
    w1 = rng.standard_normal((256, hidden)) / 16.0
    b1 = rng.standard_normal(hidden) * 0.3
    w2 = rng.standard_normal((hidden, 3)) / 4.0
    b2 = rng.standard_normal(3) * 0.2
    for t in (0.15, 0.8):
        e = _loop_embedding(t)
        x = [float(g[i]) for i in range(192)] + e          # [g; e(t)]: statistics first, embedding behind them
        hdn, n_neg = [], 0
        for j in range(hidden):
            s = float(b1[j])
            for i in range(256):
                s += x[i] * float(w1[i, j])
            n_neg += s < 0
            hdn.append(max(s, 0.0))
        assert 0 < n_neg < hidden                           # the ReLU matters for this input
        prior = (1.0, 0.0, -1.0)
        z = []
        for o in range(3):
            s = float(b2[o])
            for j in range(hidden):
                s += hdn[j] * float(w2[j, o])
            z.append(s + 1.5 * (2.0 * t - 1.0) * prior[o])
        den = sum(np.exp(zz) for zz in z)
        want = np.array([np.exp(zz) / den for zz in z])
        got = O.router_probabilities(g, t, w1, b1, w2, b2)
        assert np.abs(got - want).max() < 1e-12
        # the planted mistakes the loop has to tell apart from the right answer
        x_sw = e + [float(g[i]) for i in range(192)]
        no_relu = np.array(x) @ w1 + b1
        for wrong_h in (no_relu, np.maximum(np.array(x_sw) @ w1 + b1, 0)):
            zz = wrong_h @ w2 + b2 + 1.5 * (2 * t - 1) * np.array(prior)
            pw = np.exp(zz - zz.max()); pw /= pw.sum()
            assert np.abs(pw - want).max() > 1e-3


def test_band_statistics_coefficient_loop():
    from scipy.fft import dctn
    grid, d = (2, 4, 4), 128                               # d_k / d_r = 2 adjacent channels per group
    T, H, W = grid
    rng = np.random.default_rng(3)
    Bsz, nh = 2, 3
    chan_gain = 1.0 + np.arange(d) % 7                      # channels differ, so the grouping is visible
    q, k, v = (rng.standard_normal((Bsz, nh, T * H * W, d)) * chan_gain * s for s in (1.0, 0.5, 2.0))
    cfg = O.BandConfig(mid_block=4, mid_stride=2, high_window=4, n_summary=2)
    n_band = [0, 0, 0]
    ssq = np.zeros((3, d))
    for x in (q, k, v):
        for b in range(Bsz):
            for h in range(nh):
                c = dctn(x[b, h].reshape(T, H, W, d), type=2, norm="ortho", axes=(0, 1, 2))
                for kt in range(T):
                    for kh in range(H):
                        for kw in range(W):
                            low = 4 * kt < T and 4 * kh < H and 4 * kw < W
                            lowmid = 2 * kt < T and 2 * kh < H and 2 * kw < W
                            l = 0 if low else (1 if lowmid else 2)
                            ssq[l] += c[kt, kh, kw] ** 2
                            if x is q and b == 0 and h == 0:
                                n_band[l] += 1
    assert n_band == [1, 3, 28]
    logs = np.zeros((3, 64))
    for l in range(3):
        for r in range(64):
            mean_sq = (ssq[l, 2 * r] + ssq[l, 2 * r + 1]) / 2.0 / (3 * Bsz * nh * n_band[l])
            logs[l, r] = np.log(1e-6 + mean_sq)
    want = (logs - logs.mean()).reshape(-1)
    got = O.band_statistics(q, k, v, grid, cfg)
    assert np.abs(got - want).max() < 1e-10
    # interleaved channel groups (r, r + 64) or another epsilon would not pass
    inter = np.array([[np.log(1e-6 + (ssq[l, r] + ssq[l, r + 64]) / 2.0 / (3 * Bsz * nh * n_band[l])) for r in range(64)]
                      for l in range(3)])
    assert np.abs((inter - inter.mean()).reshape(-1) - want).max() > 1e-2
    tiny = 1e-4
    g_small = O.band_statistics(tiny * q, tiny * k, tiny * v, grid, cfg)      # energies near eps: eps is visible
    logs_s = np.log(1e-6 + (np.exp(logs) - 1e-6) * tiny ** 2)
    assert np.abs(g_small - (logs_s - logs_s.mean()).reshape(-1)).max() < 1e-9
    assert np.abs(g_small - want).max() > 1e-3


def test_load_balance_term():
    """Section 3.5: L_lb = lambda * sum_l (mean_h pi[h, l] - 1/3)^2."""
    assert O.load_balance_loss(np.full((8, 3), 1 / 3), 0.01) == 0.0
    one_band = np.tile([1.0, 0.0, 0.0], (5, 1))
    assert abs(O.load_balance_loss(one_band, 0.5) - 0.5 * (4 / 9 + 1 / 9 + 1 / 9)) < 1e-15
    pi = np.array([[0.2, 0.3, 0.5], [0.6, 0.1, 0.3]])      # column means 0.4, 0.2, 0.4
    want = 2.0 * ((0.4 - 1 / 3) ** 2 + (0.2 - 1 / 3) ** 2 + (0.4 - 1 / 3) ** 2)
    assert abs(O.load_balance_loss(pi, 2.0) - want) < 1e-15
    # hard one-hot allocations: 16/6/2 heads of 24
    alloc = O.route_fixed(24, 16, 6, 2)
    hard = np.array([[float(m >> l & 1) for l in range(3)] for m in alloc])
    want = sum((c / 24 - 1 / 3) ** 2 for c in (16, 6, 2))
    assert abs(O.load_balance_loss(hard, 1.0) - want) < 1e-15
