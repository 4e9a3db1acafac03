"""Checks of the shared input generators and of the few constants the paper prints (tests/golden/paper_constants.txt)."""
import os

import numpy as np
from scipy.fft import idctn

from oracle import freqformer as O
from paper_2604_22808_amd import workloads as WL

HERE = os.path.dirname(os.path.abspath(__file__))


def golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_constants.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def test_paper_constants():
    g = golden()
    assert O.router_param_count() == g["router_params"]
    assert O.router_flops() == g["router_flops"]
    assert 3 * O.ROUTER_DR + O.ROUTER_DT == g["router_input_width"]
    assert O.BandConfig().low_compress == g["low_compression_ratio"]
    # section 4.1 with the paper's fractions: (0.03125 N)^2 + 0.375 N * 256 + 0.5 N * 64
    assert 0.03125 ** 2 == g["attn_quadratic_coeff"] and 0.375 * 256 + 0.5 * 64 == g["attn_linear_coeff"]


def test_host_generator_recipe():
    grid, d = (4, 8, 8), 16
    x = WL.field_numpy(grid, d, seed=0, stream=1, index=3)
    assert x.shape == (256, d)
    assert np.array_equal(x, WL.field_numpy(grid, d, 0, 1, 3))                 # seeded
    assert not np.array_equal(x, WL.field_numpy(grid, d, 0, 2, 3))             # streams differ
    # spectral variance follows (1 + rho)^-3 + 0.01: DC coefficients have variance ~1.01, far ones ~0.01
    c = O.spectral_forward(np.stack([WL.field_numpy(grid, 64, 0, 0, i) for i in range(8)]).reshape(8, *grid, 64)[0])
    xs = np.concatenate([O.spectral_forward(WL.field_numpy(grid, 64, 0, 0, i).reshape(*grid, 64)).reshape(256, 64)
                         for i in range(8)], axis=1)
    assert 0.6 < xs[0].var() < 1.6 and 0.005 < xs[-1].var() < 0.02


def test_device_generator_synthesis_matches_library_idct():
    import torch
    for n in (4, 16, 64):
        M = WL._idct_matrix_torch(n, "cpu", torch.float64).numpy()
        c = np.random.default_rng(n).standard_normal(n)
        assert np.abs(M @ c - idctn(c, type=2, norm="ortho")).max() < 1e-12
    wl = WL.Workload("t", "bf16", 1, 2, 64, (4, 8, 8), WL.WORKLOADS["tiny_f32"].band, {"kind": "masks", "masks": (1, 4)})
    q, k, v = WL.qkv_torch(wl, device="cpu")
    assert q.shape == (1, 2, 256, 64) and q.dtype == torch.bfloat16 and not torch.equal(q, k)
    q2, _, _ = WL.qkv_torch(wl, device="cpu")
    assert torch.equal(q, q2)


def test_router_weights_are_seeded_float32():
    w1, b1, w2, b2 = WL.router_weights(64, 1)
    assert w1.shape == (256, 64) and w2.shape == (64, 3) and w1.dtype == np.float32
    assert np.array_equal(w1, WL.router_weights(64, 1)[0]) and not b1.any() and not b2.any()
