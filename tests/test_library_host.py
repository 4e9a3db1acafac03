"""Host-side checks of libfreqattn that need no GPU: the library loads, exports every declared symbol, rejects bad
arguments, and its integer tables (paper sections 3.3, 3.4.2) equal the oracle's bit for bit."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import freqformer as O
from paper_2604_22808_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "freqattn.h")).read()
    declared = set(re.findall(r"\b(freqattn_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    raw = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(raw, name), name


def tables_ctx(grid, d=64, dtype=B.F32, **kw):
    return B.Context(1, 2, d, grid, dtype, B.make_cfg(**kw), path=B.PATH_TABLES_ONLY)


@pytest.mark.parametrize("grid", [(4, 8, 8), (16, 32, 32), (3, 5, 7), (1, 1, 1), (16, 64, 64), (2, 6, 10)])
def test_band_lists_bit_exact(grid):
    ctx = tables_ctx(grid)
    want = O.band_partition(*grid, O.BandConfig())
    assert ctx.band_sizes() == [len(w) for w in want]
    for l in range(3):
        got = ctx.band_index(l)
        assert got.dtype == np.int32 and np.array_equal(got.astype(np.int64), want[l])


def test_band_lists_other_edges():
    kw = dict(low_num=1, low_den=8, mid_num=3, mid_den=4)
    ctx = tables_ctx((8, 8, 16), **kw)
    want = O.band_partition(8, 8, 16, O.BandConfig(**kw))
    for l in range(3):
        assert np.array_equal(ctx.band_index(l).astype(np.int64), want[l])


@pytest.mark.parametrize("grid,block,diag,stride,b0", [((4, 8, 8), 16, 1, 4, 1), ((16, 32, 32), 64, 1, 8, 1),
                                                       ((16, 64, 64), 64, 1, 8, 1), ((64, 64, 64), 128, 2, 16, 1),
                                                       ((8, 8, 8), 5, 0, 3, 0), ((8, 8, 8), 7, 3, 1, 0)])
def test_mid_block_list_bit_exact(grid, block, diag, stride, b0):
    ctx = tables_ctx(grid, mid_block=block, mid_diag=diag, mid_stride=stride, mid_block0=b0)
    n_mid = ctx.band_sizes()[1]
    nb = -(-n_mid // block)
    rp, ci = ctx.mid_blocks()
    wrp, wci = O.mid_block_csr(nb, diag, stride, b0)
    assert np.array_equal(rp, wrp) and np.array_equal(ci, wci)


def test_mid_block_counts_of_the_benchmark_configurations():
    for grid, block, diag, stride, nnz in [((16, 32, 32), 64, 1, 8, 177), ((16, 64, 64), 64, 1, 8, 1887),
                                           ((64, 64, 64), 128, 2, 16, 4234)]:
        ctx = tables_ctx(grid, mid_block=block, mid_diag=diag, mid_stride=stride)
        assert len(ctx.mid_blocks()[1]) == nnz


@pytest.mark.parametrize("n", [1, 4, 8, 16, 64, 128])
def test_dct_matrix_matches_oracle(n):
    ctx = tables_ctx((n, 4, 4))
    assert np.abs(ctx.dct_matrix(0) - O.dct_matrix(n)).max() < 1e-14


@pytest.mark.parametrize("n", [1, 2, 8, 64, 128])
def test_haar_matrix_matches_oracle(n):
    ctx = tables_ctx((n, 4, 8), transform=B.TRANSFORM_HAAR)
    assert np.abs(ctx.dct_matrix(0) - O.haar_matrix(n)).max() < 1e-15
    assert np.abs(ctx.dct_matrix(2) - O.haar_matrix(8)).max() < 1e-15


def test_haar_needs_power_of_two_axes_and_known_transform():
    with pytest.raises(B.FreqAttnError):
        tables_ctx((12, 4, 4), transform=B.TRANSFORM_HAAR)
    with pytest.raises(B.FreqAttnError):
        tables_ctx((8, 4, 4), transform=2)


def test_route_fixed():
    assert list(B.route_fixed(8, 2, 3, 3)) == list(O.route_fixed(8, 2, 3, 3))
    with pytest.raises(B.FreqAttnError):
        B.route_fixed(8, 2, 3, 4)


@pytest.mark.parametrize("bad", [dict(low_compress=0), dict(mid_block=0), dict(mid_stride=0), dict(mid_diag=-1),
                                 dict(high_window=-1), dict(n_summary=-1), dict(low_num=3, low_den=4, mid_num=1, mid_den=2),
                                 dict(mid_num=3, mid_den=2), dict(low_num=0)])
def test_create_rejects_bad_band_cfg(bad):
    with pytest.raises(B.FreqAttnError) as e:
        tables_ctx((4, 8, 8), **bad)
    assert e.value.status == B.EINVAL


def test_create_rejects_bad_shapes_and_paths():
    for shape in [(0, 2, 64, (4, 8, 8), B.F32), (1, 2, 64, (4, 0, 8), B.F32), (1, 2, 64, (4, 8, 8), 7)]:
        with pytest.raises(B.FreqAttnError) as e:
            B.Context(*shape, B.make_cfg(), path=B.PATH_TABLES_ONLY)
        assert e.value.status == B.EINVAL
    with pytest.raises(B.FreqAttnError) as e:      # MFMA path cannot take fp32 I/O or a 4x8x8 grid
        B.Context(1, 2, 64, (4, 8, 8), B.F32, B.make_cfg(), path=B.PATH_MFMA)
    assert e.value.status == B.EUNSUPPORTED
    assert B.lib().freqattn_create(None, None, 0, None) == B.EINVAL
    B.lib().freqattn_destroy(None)   # no-op


def test_tables_only_context_refuses_compute():
    ctx = tables_ctx((4, 8, 8))
    cfg = ctx.cfg
    ha = (C.c_int32 * 2)(1, 4)
    dummy = C.c_void_p(16)
    st = B.lib().freqattn_forward(ctx._h, dummy, dummy, dummy, C.byref(cfg), ha, C.c_void_p(32), None)
    assert st == B.EUNSUPPORTED and b"tables-only" in B.lib().freqattn_last_error(ctx._h)


@pytest.mark.parametrize("grid,m,transform", [((4, 8, 8), 4, 0), ((16, 32, 32), 16, 0), ((3, 5, 7), 7, 0),
                                              ((2, 6, 10), 200, 0), ((8, 16, 16), 5, 1)])
def test_summary_weights_pool_the_spectrum_of_the_input(grid, m, transform):
    """Section 3.6 (U = I) through linearity: the weights applied to x in token space give the mean-pooled summary
    tokens of x's coefficients, band by band (the oracle transforms first and pools afterwards)."""
    T, H, W = grid
    ctx = tables_ctx(grid, n_summary=m, transform=transform)
    cfg = O.BandConfig(n_summary=m, transform=transform)
    rng = np.random.default_rng(5)
    x = rng.standard_normal((T, H, W, 3))
    xs = O.spectral_forward(x, transform=transform).reshape(-1, 3)
    for l, idx in enumerate(O.band_partition(T, H, W, cfg)):
        w = ctx.summary_weights(l)
        if len(idx) == 0:
            assert w.shape[0] == 0
            continue
        want = O.summary_tokens(xs[idx], m)
        n, me = len(idx), min(m, len(idx))
        assert w.shape == (me, T * H * W)
        sizes = np.array([((u + 1) * n) // me - (u * n) // me for u in range(me)], np.float64)
        got = (w.astype(np.float64) @ x.reshape(-1, 3)) / sizes[:, None]
        assert np.abs(got - want).max() < 2e-6, (l, np.abs(got - want).max())


def test_binding_rejects_tensors_the_kernels_could_not_address(monkeypatch):
    """The C side only sees addresses; the binding refuses host tensors, other types, shapes and layouts, and a
    head_alloc of the wrong length, before any pointer is taken."""
    import torch
    ctx = B.Context(1, 2, 64, (4, 8, 8), B.BF16, B.make_cfg(mid_block=16, mid_stride=4, high_window=32, n_summary=4),
                    path=B.PATH_TABLES_ONLY)
    good = torch.zeros(1, 2, 256, 64, dtype=torch.bfloat16)

    class FakeDevice(torch.Tensor):      # a host tensor that claims to live on the device: reaches the later checks
        is_cuda = True

    dev = lambda t: t.as_subclass(FakeDevice)
    with pytest.raises(ValueError, match="device tensor"):
        ctx.forward(good, good, good, [1, 4], good.clone())
    with pytest.raises(ValueError, match="dtype"):
        ctx.forward(dev(good.float()), dev(good), dev(good), [1, 4], dev(good.clone()))
    with pytest.raises(ValueError, match="shape"):
        ctx.forward(dev(good[:, :1]), dev(good), dev(good), [1, 4], dev(good.clone()))
    with pytest.raises(ValueError, match="contiguous"):
        ctx.forward(dev(good.transpose(2, 3).contiguous().transpose(2, 3)), dev(good), dev(good), [1, 4], dev(good.clone()))
    with pytest.raises(ValueError, match="head_alloc"):
        ctx.forward(dev(good), dev(good), dev(good), [1], dev(good.clone()))
    with pytest.raises(TypeError):
        ctx.forward(np.zeros((1, 2, 256, 64)), good, good, [1, 4], good)
    w1, b1, w2, b2 = np.zeros((256, 8)), np.zeros(8), np.zeros((8, 3)), np.zeros(3)
    with pytest.raises(ValueError, match="router weights"):
        ctx.route_mlp(dev(good), dev(good), dev(good), 0.5, w1[:100], b1, w2, b2)
    with pytest.raises(ValueError, match="device tensor"):
        ctx.dense_forward(good, good, good, good.clone())
    # with everything in order the call reaches the library, which refuses a tables-only context itself
    monkeypatch.setattr(B, "_stream", lambda: C.c_void_p(0))       # no device here: the default stream's handle
    with pytest.raises(B.FreqAttnError) as ei:
        ctx.forward(dev(good), dev(good), dev(good), [1, 4], dev(good.clone()))
    assert ei.value.status == B.EUNSUPPORTED


def test_two_band_tables_and_load_balance_term():
    """L = 2 band layouts (an empty mid or high band) give the oracle's lists; the load-balancing term of section 3.5
    equals the oracle's."""
    for kw in (dict(mid_num=1, mid_den=4), dict(mid_num=1, mid_den=1)):
        ctx = tables_ctx((8, 16, 16), **kw)
        want = O.band_partition(8, 16, 16, O.BandConfig(**kw))
        assert ctx.band_sizes() == [len(w) for w in want] and 0 in ctx.band_sizes()
        for l in range(3):
            assert np.array_equal(ctx.band_index(l).astype(np.int64), want[l])
    with pytest.raises(B.FreqAttnError):
        tables_ctx((8, 16, 16), low_num=1, low_den=2, mid_num=1, mid_den=4)      # low edge above the mid edge
    rng = np.random.default_rng(4)
    pi = rng.random((24, 3)); pi /= pi.sum(axis=1, keepdims=True)
    assert abs(B.load_balance(pi, 0.01) - O.load_balance_loss(pi.astype(np.float32), 0.01)) < 1e-9
    hard = np.eye(3)[[0] * 16 + [1] * 6 + [2] * 2]
    assert abs(B.load_balance(hard, 1.0) - O.load_balance_loss(hard, 1.0)) < 1e-7


def test_four_band_tables():
    """L = 4 (the band-count ablation of section 8): a third edge splits what lies beyond the mid edge into a second
    block-sparse band (index 3, rows after the high band) and the windowed rest; lists and block patterns are the oracle's,
    and without the third edge the context is the three-band one."""
    for grid, kw in [((8, 16, 16), dict(mid2_num=3, mid2_den=4)), ((4, 8, 16), dict(mid2_num=3, mid2_den=4, mid_block=16)),
                     ((3, 5, 7), dict(mid2_num=2, mid2_den=3, mid_block=5, mid_stride=3)),
                     ((8, 8, 8), dict(mid2_num=1, mid2_den=1, mid_block=16))]:
        ctx = tables_ctx(grid, **kw)
        cfg = O.BandConfig(**kw)
        want = O.band_partition(*grid, cfg)
        assert len(want) == 4 and ctx.band_sizes() == [len(w) for w in want]
        for l in range(4):
            assert np.array_equal(ctx.band_index(l).astype(np.int64), want[l])
        for band, (rp, ci) in ((1, ctx.mid_blocks()), (3, ctx.mid2_blocks())):
            nb = -(-len(want[band]) // cfg.mid_block)
            wrp, wci = O.mid_block_csr(nb, cfg.mid_diag, cfg.mid_stride, cfg.mid_block0)
            assert np.array_equal(rp, wrp) and np.array_equal(ci, wci)
    three = tables_ctx((8, 16, 16))
    assert three.band_sizes() == [len(w) for w in O.band_partition(8, 16, 16, O.BandConfig())]
    assert len(three.mid2_blocks()[1]) == 0
    with pytest.raises(B.FreqAttnError):
        tables_ctx((8, 16, 16), mid2_num=1, mid2_den=4)      # third edge below the mid edge
    with pytest.raises(B.FreqAttnError):
        tables_ctx((8, 16, 16), mid2_num=5, mid2_den=4)      # third edge beyond the grid
