"""GPU parity: the HIP library (through its C ABI) against the fp64 oracle on the same seeded inputs.

Tolerances: bf16 I/O with fp16 matrix-core operands and fp32 accumulation: max-abs <= 2e-2 and relative L2 <= 5e-3;
fp32 configuration: 1e-5 for both.  Integer tables must be bit-exact.
"""
import numpy as np
import pytest

from oracle import freqformer as O
from paper_2604_22808_amd import binding as B
from paper_2604_22808_amd import workloads as WL
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _inputs(wl, heads=None):
    q, k, v = WL.qkv_numpy(wl, heads=heads)
    return [WL.round_to_io(x, wl.dtype) for x in (q, k, v)]


def _check(got, want, dtype, what=""):
    mx, rl = U.errors(got, want)
    tol_abs, tol_rel = U.TOL[dtype]
    print(f"{what}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= tol_abs and rl <= tol_rel, (what, mx, rl)


# ------------------------------------------------------------------ fp32 configuration (generic kernels)
@pytest.mark.parametrize("masks", [(1, 4), (2, 7), (0, 3), (5, 6)])
def test_tiny_f32_matches_oracle(masks):
    wl = WL.WORKLOADS["tiny_f32"]
    q, k, v = _inputs(wl)
    ctx, band = U.make_ctx(wl)
    assert ctx.get_path() == B.PATH_GENERIC
    got = U.run_forward(ctx, q, k, v, wl.dtype, masks)
    want = O.forward(q, k, v, wl.grid, U.oracle_cfg(band), masks)
    _check(got, want, "f32", f"tiny_f32 masks={masks}")


def test_tiny_f32_unit_rms_stress():
    """Inputs rescaled to unit RMS: the low band becomes argmax-like (DC variance ~86); fp32 only."""
    wl = WL.WORKLOADS["tiny_f32"]
    q, k, v = (x / x.std() for x in WL.qkv_numpy(wl))
    q, k, v = (WL.round_to_io(x, "f32") for x in (q, k, v))
    ctx, band = U.make_ctx(wl)
    got = U.run_forward(ctx, q, k, v, "f32", (7, 7))
    want = O.forward(q, k, v, wl.grid, U.oracle_cfg(band), (7, 7))
    mx, rl = U.errors(got, want)
    print(f"unit-rms stress: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 1e-4 and rl <= 1e-4   # logits reach O(100): fp32 products lose ~1e-5 absolute before the exponential


@pytest.mark.parametrize("grid,d,band", [
    ((3, 5, 7), 8, dict(mid_block=5, mid_diag=1, mid_stride=3, mid_block0=0, high_window=4, n_summary=3, low_compress=2)),
    ((2, 4, 4), 16, dict(mid_block=4, mid_diag=0, mid_stride=2, mid_block0=1, high_window=100, n_summary=50, low_compress=1)),
    ((1, 1, 1), 4, dict(mid_block=4, high_window=1, n_summary=2)),
    ((4, 8, 8), 64, dict(mid_block=16, mid_diag=1, mid_stride=1, high_window=0, n_summary=0)),
    ((4, 8, 8), 160, dict(mid_block=16, mid_diag=1, mid_stride=4, high_window=32, n_summary=4, softmax_scale=0.2)),
])
def test_generic_edge_shapes_f32(grid, d, band):
    """Ragged grids, empty bands (1x1x1 has only a low band), m larger than a band, window 0 and >= N, all-ones mask."""
    rng = np.random.default_rng(11)
    N = int(np.prod(grid))
    q, k, v = (WL.round_to_io(rng.standard_normal((2, 3, N, d)), "f32") for _ in range(3))
    cfgd = dict(WL.WORKLOADS["tiny_f32"].band)
    cfgd.update(band)
    ctx = B.Context(2, 3, d, grid, B.F32, B.make_cfg(**cfgd))
    alloc = (7, 2, 5)
    got = U.run_forward(ctx, q, k, v, "f32", alloc)
    want = O.forward(q, k, v, grid, O.BandConfig(**cfgd), alloc)
    _check(got, want, "f32", f"edge {grid} d={d}")


def test_no_active_band_returns_v_on_gpu():
    wl = WL.WORKLOADS["tiny_f32"]
    q, k, v = _inputs(wl)
    ctx, _ = U.make_ctx(wl)
    got = U.run_forward(ctx, q, k, v, "f32", (0, 0))
    assert np.abs(got - v).max() < 1e-5


def test_forward_rejects_bad_arguments():
    import torch
    wl = WL.WORKLOADS["tiny_f32"]
    ctx, band = U.make_ctx(wl)
    q = torch.zeros((1, 2, 256, 64), device="cuda")
    out = torch.empty_like(q)
    with pytest.raises(B.FreqAttnError) as e:
        ctx.forward(q, q, q, (1, 9), out)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.FreqAttnError) as e:
        ctx.forward(q, q, q, (1, 4), q)            # out aliases an input
    assert e.value.status == B.EINVAL
    other = dict(band); other["high_window"] = 31
    with pytest.raises(B.FreqAttnError) as e:
        ctx.forward(q, q, q, (1, 4), out, cfg=B.make_cfg(**other))
    assert e.value.status == B.EINVAL
    ctx.forward(q, q, q, (1, 4), out)              # the context is still usable
    torch.cuda.synchronize()


# ------------------------------------------------------------------ bf16 configurations (MFMA kernels)
def _stagewise(ctx, wl, band, q, k, v, alloc, out_gpu, tol_rel=2e-3):
    """Per-slice, per-stage comparison with the oracle's intermediate results: spectral Q~, K~ (active bands), V~ and the
    band outputs after the exchange must each be within tol_rel (relative L2) - an error in one stage cannot hide behind
    the pass-through of the inactive bands in the final output."""
    cfg = U.oracle_cfg(band)
    T, H, W = wl.grid
    for s in range(q.shape[1]):
        f = lambda a: a[0, s].reshape(T, H, W, -1)
        want, parts = O.head_forward(f(q), f(k), f(v), cfg, int(alloc[s]), return_parts=True)
        for l in range(3):
            idx = parts["bands"][l]
            if (alloc[s] >> l) & 1:
                for which, name in ((0, "qs"), (1, "ks")):
                    mx, rl = U.errors(ctx.read_spectral(which, s, l), parts[name][idx])
                    print(f"  slice {s} band {l} {name}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
                    assert rl <= tol_rel, (s, l, name, rl)
            try:   # a slice that does not run the high band has no V~ rows there (its V~ stops at the low+mid box)
                mx, rl = U.errors(ctx.read_spectral(2, s, l), parts["vs"][idx])
                print(f"  slice {s} band {l} vs: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
                assert rl <= tol_rel, (s, l, "vs", rl)
                mx, rl = U.errors(ctx.read_spectral(3, s, l), parts["Yhat"][l])
                print(f"  slice {s} band {l} Yhat: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
                assert rl <= tol_rel, (s, l, "Yhat", rl)
            except B.FreqAttnError as e:
                assert e.status == B.EUNSUPPORTED and l == 2 and not (alloc[s] >> 2) & 1
        mx, rl = U.errors(out_gpu[0, s], want.reshape(-1, want.shape[-1]))
        print(f"  slice {s} mask {alloc[s]} out: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)


@pytest.mark.parametrize("path", [B.PATH_MFMA, B.PATH_GENERIC])
def test_16k_bf16_matches_oracle(path):
    wl = WL.WORKLOADS["16k"]
    heads = [0, 2, 5, 7]                       # one low, one mid, two high heads of the 2/3/3 allocation
    alloc_full = B.route_fixed(wl.heads, *wl.alloc["counts"])
    alloc = [int(alloc_full[h]) for h in heads]
    alloc[3] = 7                               # and one head that runs every band (the paper's literal equations)
    q, k, v = _inputs(wl, heads=heads)
    ctx, band = U.make_ctx(wl, path=path, heads=len(heads))
    assert ctx.get_path() == path
    got = U.run_forward(ctx, q, k, v, wl.dtype, alloc)
    _stagewise(ctx, wl, band, q, k, v, alloc, got)
    want = O.forward(q, k, v, wl.grid, U.oracle_cfg(band), alloc)
    _check(got, want, "bf16", f"16k path={path}")
    for s in range(len(heads)):
        _check(got[0, s], want[0, s], "bf16", f"16k path={path} slice {s}")


def test_16k_tables_bit_exact_on_device_context():
    wl = WL.WORKLOADS["16k"]
    ctx, band = U.make_ctx(wl)
    want = O.band_partition(*wl.grid, U.oracle_cfg(band))
    for l in range(3):
        assert np.array_equal(ctx.band_index(l).astype(np.int64), want[l])
    rp, ci = ctx.mid_blocks()
    wrp, wci = O.mid_block_csr(len(rp) - 1, band["mid_diag"], band["mid_stride"], band["mid_block0"])
    assert np.array_equal(rp, wrp) and np.array_equal(ci, wci)


def test_16k_fused_and_separate_launches_agree():
    import torch
    wl = WL.WORKLOADS["16k"]
    q, k, v = (U.to_device(x, "bf16") for x in _inputs(wl, heads=[0, 3, 6]))
    ctx, _ = U.make_ctx(wl, heads=3)
    a = torch.empty_like(q); b = torch.empty_like(q)
    ctx.forward(q, k, v, (1, 2, 4), a)
    ctx.set_launch_mode(B.LAUNCH_SEPARATE)
    ctx.forward(q, k, v, (1, 2, 4), b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)                      # same kernels, same per-item arithmetic: bitwise equal
    ctx.set_launch_mode(B.LAUNCH_FUSED)
    ctx.forward(q, k, v, (1, 2, 4), b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)                      # and run-to-run deterministic


@pytest.mark.parametrize("band", [
    dict(mid_stride=1, high_window=20000, low_compress=1, n_summary=0),     # every branch degenerates to dense attention
    dict(mid_block=128, mid_diag=0, mid_stride=3, mid_block0=0, high_window=100, n_summary=5, low_compress=3),
    dict(mid_block=192, mid_diag=1, mid_stride=2, high_window=0, n_summary=300),
])
@pytest.mark.parametrize("v_box", ["0", "1"])
def test_16k_bf16_parameter_edges(band, v_box, monkeypatch):
    """Degenerate and odd band parameters, with V~ on the whole grid and with V~ of slices without the high band on the
    low+mid box (no summaries at all; more summary tokens than the summing kernel takes, where the library keeps the
    whole-grid V~ by itself)."""
    monkeypatch.setenv("FREQATTN_V_BOX", v_box)
    wl = WL.WORKLOADS["16k"]
    q, k, v = _inputs(wl, heads=[1, 4])
    ctx, bandd = U.make_ctx(wl, heads=2, **band)
    assert ctx.get_path() == B.PATH_MFMA
    assert ctx.get_v_box() == (int(v_box) if band["n_summary"] <= 64 else 0)
    alloc = (3, 6)
    got = U.run_forward(ctx, q, k, v, wl.dtype, alloc)
    want = O.forward(q, k, v, wl.grid, U.oracle_cfg(bandd), alloc)
    _check(got, want, "bf16", f"16k edges {band}")


@pytest.mark.parametrize("v_box,alloc", [("0", (7, 4)), ("1", (7, 4)), ("1", (1, 2, 3))])
def test_mfma_ragged_grid_bf16(v_box, alloc, monkeypatch):
    """Grid 16x48x80 (axis lengths that are not powers of two), head_dim 128, ragged tails in every band; also with V~ of
    the heads without the high band on the low+mid box, wherever the kernels' granularity gives a smaller box."""
    monkeypatch.setenv("FREQATTN_V_BOX", v_box)
    grid, d = (16, 48, 80), 128
    rng = np.random.default_rng(5)
    N = int(np.prod(grid))
    q, k, v = (WL.round_to_io(0.3 * rng.standard_normal((1, len(alloc), N, d)), "bf16") for _ in range(3))
    band = dict(WL.WORKLOADS["16k"].band)
    band.update(mid_block=128, mid_diag=1, mid_stride=5, high_window=200, n_summary=7, low_compress=4)
    ctx = B.Context(1, len(alloc), d, grid, B.BF16, B.make_cfg(**band))
    assert ctx.get_path() == B.PATH_MFMA
    print(f"ragged grid: V on the box = {ctx.get_v_box()}", flush=True)
    got = U.run_forward(ctx, q, k, v, "bf16", alloc)
    want = O.forward(q, k, v, grid, O.BandConfig(**band), alloc)
    _check(got, want, "bf16", "ragged 16x48x80")


def test_64k_router_in_the_loop_matches_oracle():
    """64K configuration, four of its heads: the device router (statistics on fp16 spectra, MLP on the host) must give
    the oracle's probabilities and the same integer allocation; the routed forward must match the oracle run with it."""
    import torch
    wl = WL.WORKLOADS["64k"]
    heads = [0, 1, 2, 3]
    q, k, v = _inputs(wl, heads=heads)
    ctx, band = U.make_ctx(wl, heads=len(heads))
    cfg = U.oracle_cfg(band)
    w = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
    dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
    for t in (0.9, 0.1):
        want_alloc, want_pi = O.route_mlp(q, k, v, wl.grid, cfg, t, *w)
        got_alloc, got_pi, got_stats = ctx.route_mlp(dq, dk, dv, t, *w)
        want_stats = O.band_statistics(q, k, v, wl.grid, cfg)
        print(f"t={t}: pi gpu {got_pi} oracle {want_pi} alloc {got_alloc}; stats max diff "
              f"{np.abs(got_stats - want_stats).max():.2e}", flush=True)
        assert np.abs(got_stats - want_stats).max() < 5e-3
        assert np.abs(got_pi - want_pi).max() < 2e-3
        assert np.array_equal(got_alloc, want_alloc)
    out = torch.empty_like(dq)
    alloc, pi = ctx.forward_routed(dq, dk, dv, 0.9, *w, out)
    torch.cuda.synchronize()
    want_alloc, _ = O.route_mlp(q, k, v, wl.grid, cfg, 0.9, *w)
    assert np.array_equal(alloc, want_alloc)
    want = O.forward(q, k, v, wl.grid, cfg, want_alloc)
    _check(U.to_host64(out), want, "bf16", f"64k routed alloc={list(alloc)}")
    # the same allocation through the plain entry point gives the same bits
    out2 = torch.empty_like(dq)
    ctx.forward(dq, dk, dv, alloc, out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_16k_mask_classes_bf16():
    """Every class of band mask on the MFMA path: idle head (out = V exactly), low+high, low+mid, mid+high, and the
    one-hot masks, in one context (heads that only run the low / low+mid bands take the pruned transforms)."""
    wl = WL.WORKLOADS["16k"]
    heads = [0, 1, 2, 3, 4, 5, 6]
    alloc = (0, 5, 3, 6, 1, 2, 4)
    q, k, v = _inputs(wl, heads=heads)
    ctx, band = U.make_ctx(wl, heads=len(heads))
    assert ctx.get_path() == B.PATH_MFMA
    got = U.run_forward(ctx, q, k, v, wl.dtype, alloc)
    want = O.forward(q, k, v, wl.grid, U.oracle_cfg(band), alloc)
    assert np.array_equal(got[0, 0], v[0, 0])          # nothing active: the library returns V itself
    for s in range(len(heads)):
        _check(got[0, s], want[0, s], "bf16", f"16k mask {alloc[s]}")


@pytest.mark.parametrize("name,heads,alloc,routed", [
    ("16k", [0, 1, 2, 3, 4, 5, 6], (0, 5, 3, 6, 1, 2, 4), False),   # head_dim 64, every class of mask
    ("16k", [0, 1, 2, 3], None, True),                               # router in the loop
    ("256k", [0, 5, 11], (1, 2, 3), False),                          # head_dim 128, no head runs the high band
])
def test_v_on_the_low_mid_box_matches_oracle_and_whole_grid_path(name, heads, alloc, routed, monkeypatch):
    """Slices without the high band: V~ on the low+mid box and their high-band summary tokens summed from the
    untransformed V (forced on here, whatever the size), against the oracle and against the same library with the
    whole-grid V~ (the two differ by rounding only)."""
    import torch
    wl = WL.WORKLOADS[name]
    q, k, v = _inputs(wl, heads=heads)
    outs = []
    for flag in ("1", "0"):
        monkeypatch.setenv("FREQATTN_V_BOX", flag)
        ctx, band = U.make_ctx(wl, path=B.PATH_MFMA, heads=len(heads))
        if routed:
            w = WL.router_weights(64, 1)
            dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
            out = torch.empty_like(dq)
            for t in (0.9, 0.1, 0.5):   # from the second call on, the previous allocation serves as the prediction
                al, pi = ctx.forward_routed(dq, dk, dv, t, *w, out)
            torch.cuda.synchronize()
            outs.append((out.to(torch.float64).cpu().numpy(), tuple(int(a) for a in al)))
        else:
            outs.append((U.run_forward(ctx, q, k, v, wl.dtype, alloc), alloc))
        ctx.destroy()
    (got, al), (ref, al_ref) = outs
    assert tuple(al) == tuple(al_ref)
    if name == "16k":
        want = O.forward(q, k, v, wl.grid, U.oracle_cfg(band), al)
        for s in range(len(heads)):
            _check(got[0, s], want[0, s], "bf16", f"{name} V on the box, mask {al[s]}")
    mx, rl = U.errors(got, ref)
    print(f"{name}: box vs whole grid max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 1e-2 and rl <= 2e-3, (mx, rl)


@pytest.mark.parametrize("grid,band_kw", [
    ((16, 32, 32), dict(mid_block=128, mid_diag=1, mid_stride=4, high_window=96, n_summary=8)),
    ((16, 16, 48), dict(mid_block=64, mid_diag=2, mid_stride=3, high_window=40, n_summary=5)),
])
@pytest.mark.parametrize("v_box", ["0", "1"])
def test_mfma_head_dim_64_bf16(grid, band_kw, v_box, monkeypatch):
    """head_dim 64 instantiations of the matrix-core kernels (transform passes with one 64-column chunk per token,
    attention with four channel steps), one head per band plus one head that runs all bands; with V~ on the whole grid
    and with V~ of the heads without the high band on the low+mid box (summary weights over ragged chunks, white-noise
    inputs: nothing is small in the high band)."""
    monkeypatch.setenv("FREQATTN_V_BOX", v_box)
    d = 64
    rng = np.random.default_rng(11)
    N = int(np.prod(grid))
    q, k, v = (WL.round_to_io(0.3 * rng.standard_normal((1, 4, N, d)), "bf16") for _ in range(3))
    band = dict(WL.WORKLOADS["16k"].band)
    band.update(low_compress=4, **band_kw)
    ctx = B.Context(1, 4, d, grid, B.BF16, B.make_cfg(**band))
    assert ctx.get_path() == B.PATH_MFMA
    if grid == (16, 32, 32):       # (the 16x16x48 grid has no smaller low+mid box in the kernels' granularity)
        assert ctx.get_v_box() == int(v_box)
    alloc = (1, 2, 4, 7)
    got = U.run_forward(ctx, q, k, v, "bf16", alloc)
    want = O.forward(q, k, v, grid, O.BandConfig(**band), alloc)
    for s in range(4):
        _check(got[0, s], want[0, s], "bf16", f"d=64 grid {grid} mask {alloc[s]}")


@pytest.mark.parametrize("d,grid", [(128, (16, 16, 32)), (64, (16, 16, 16))])
def test_dense_baseline_matches_dense_reference(d, grid):
    """The dense comparison kernel (same attention kernel over the untransformed sequence, bf16 in and out) against
    the oracle's plain softmax attention."""
    import torch
    rng = np.random.default_rng(13)
    N = int(np.prod(grid))
    q, k, v = (WL.round_to_io(0.5 * rng.standard_normal((1, 2, N, d)), "bf16") for _ in range(3))
    band = dict(WL.WORKLOADS["16k"].band)
    band.update(mid_block=128)
    ctx = B.Context(1, 2, d, grid, B.BF16, B.make_cfg(**band))
    assert ctx.get_path() == B.PATH_MFMA
    dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
    out = torch.empty_like(dq)
    ctx.dense_forward(dq, dk, dv, out)
    torch.cuda.synchronize()
    got = U.to_host64(out)
    for s in range(2):
        want = O.dense_reference(q[0, s], k[0, s], v[0, s])
        _check(got[0, s], want, "bf16", f"dense d={d} slice {s}")


# ------------------------------------------------------------------ Haar wavelet as the per-axis transform (section 3.2)
def test_haar_tiny_f32_matches_oracle():
    wl = WL.WORKLOADS["tiny_f32"]
    q, k, v = _inputs(wl)
    ctx, band = U.make_ctx(wl, transform=B.TRANSFORM_HAAR)
    alloc = (2, 7)
    got = U.run_forward(ctx, q, k, v, wl.dtype, alloc)
    want = O.forward(q, k, v, wl.grid, U.oracle_cfg(band), alloc)
    _check(got, want, "f32", "haar tiny f32")
    dct = O.forward(q, k, v, wl.grid, U.oracle_cfg(dict(band, transform=0)), alloc)
    assert np.abs(want - dct).max() > 1e-3       # the variant really computes something else


def test_haar_16k_bf16_matches_oracle_on_the_matrix_cores():
    """Same kernels, other matrix: pruned transforms, delta-form inverse and the Parseval statistics only rely on the
    transform being orthonormal and on bands being index boxes, which the Haar ordering (coarse to fine) keeps."""
    wl = WL.WORKLOADS["16k"]
    heads = [0, 2, 5, 7]
    q, k, v = _inputs(wl, heads=heads)
    ctx, band = U.make_ctx(wl, path=B.PATH_MFMA, heads=len(heads), transform=B.TRANSFORM_HAAR)
    alloc = (1, 2, 4, 7)
    got = U.run_forward(ctx, q, k, v, wl.dtype, alloc)
    want = O.forward(q, k, v, wl.grid, U.oracle_cfg(band), alloc)
    for s in range(len(heads)):
        _check(got[0, s], want[0, s], "bf16", f"haar 16k mask {alloc[s]}")
    for which, x in ((0, q), (2, v)):            # spectral coefficients of head 3 (all bands computed)
        xs = O.spectral_forward(x[0, 3].reshape(wl.grid + (wl.head_dim,)), transform=1).reshape(-1, wl.head_dim)
        for l, idx in enumerate(O.band_partition(*wl.grid, U.oracle_cfg(band))):
            mx, rl = U.errors(ctx.read_spectral(which, 3, l), xs[idx])
            assert rl < 2e-3, (which, l, rl)


def test_haar_64k_router_statistics_and_routed_forward():
    import torch
    wl = WL.WORKLOADS["64k"]
    heads = [0, 1, 2, 3]
    q, k, v = _inputs(wl, heads=heads)
    ctx, band = U.make_ctx(wl, heads=len(heads), transform=B.TRANSFORM_HAAR)
    cfg = U.oracle_cfg(band)
    w = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
    dq, dk, dv = (U.to_device(x, wl.dtype) for x in (q, k, v))
    got_alloc, got_pi, got_stats = ctx.route_mlp(dq, dk, dv, 0.5, *w)
    want_alloc, want_pi = O.route_mlp(q, k, v, wl.grid, cfg, 0.5, *w)
    assert np.abs(got_stats - O.band_statistics(q, k, v, wl.grid, cfg)).max() < 5e-3
    assert np.abs(got_pi - want_pi).max() < 2e-3
    assert np.array_equal(got_alloc, want_alloc)
    out = torch.empty_like(dq)
    alloc2, _ = ctx.forward_routed(dq, dk, dv, 0.5, *w, out)
    torch.cuda.synchronize()
    assert np.array_equal(alloc2, want_alloc)
    want = O.forward(q, k, v, wl.grid, cfg, want_alloc)
    _check(U.to_host64(out), want, "bf16", f"haar 64k routed alloc={list(alloc2)}")


def test_measure_peaks_reports_machine_rates():
    wl = WL.WORKLOADS["64k"]
    ctx, _ = U.make_ctx(wl)
    copy_bps, mfma_fps = ctx.measure_peaks()
    print(f"copy {copy_bps / 1e9:.0f} GB/s, mfma loop {mfma_fps / 1e12:.0f} TFLOP/s", flush=True)
    assert 1e11 < copy_bps < 3e13 and 1e14 < mfma_fps < 5.1e15


def test_routed_forward_with_allocation_prediction():
    """The routed forward transforms Q/K of the heads that were high in the previous call in full at once and completes
    only newly high heads after routing: whatever was predicted, allocation and output bits are those of the plain
    forward with the routed allocation (and of the routed forward with prediction switched off)."""
    import torch
    wl = WL.WORKLOADS["64k"]
    heads = [0, 1, 2, 3, 4, 5]
    q, k, v = _inputs(wl, heads=heads)
    ctx, band = U.make_ctx(wl, heads=len(heads))
    ref, _ = U.make_ctx(wl, heads=len(heads))
    ref.set_alloc_prediction(False)
    cfg = U.oracle_cfg(band)
    w = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
    dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
    out, out_ref, out_plain = (torch.empty_like(dq) for _ in range(3))
    seen = set()
    for t in (0.9, 0.9, 0.1, 0.1, 0.5, 0.9):          # first call: nothing to predict from; then right and wrong guesses
        alloc, pi = ctx.forward_routed(dq, dk, dv, t, *w, out)
        alloc_ref, _ = ref.forward_routed(dq, dk, dv, t, *w, out_ref)
        want_alloc, _ = O.route_mlp(q, k, v, wl.grid, cfg, t, *w)
        torch.cuda.synchronize()
        assert np.array_equal(alloc, want_alloc) and np.array_equal(alloc_ref, want_alloc), (t, alloc, alloc_ref, want_alloc)
        ref.forward(dq, dk, dv, alloc, out_plain)
        torch.cuda.synchronize()
        assert torch.equal(out, out_plain) and torch.equal(out_ref, out_plain), t
        seen.add(tuple(int(a) for a in alloc))
    assert len(seen) >= 2                                # the sequence really changes the allocation
    want = O.forward(q, k, v, wl.grid, cfg, alloc)
    _check(U.to_host64(out), want, "bf16", f"64k routed with prediction, alloc={list(alloc)}")


def test_batch_of_two_on_a_side_stream():
    """batch 2 x 3 heads (slice = batch index * heads + head, the allocation repeats per batch entry), both paths, with
    the forward queued on a non-default stream."""
    import torch
    grid, d = (16, 16, 32), 128
    rng = np.random.default_rng(21)
    N = int(np.prod(grid))
    q, k, v = (WL.round_to_io(0.4 * rng.standard_normal((2, 3, N, d)), "bf16") for _ in range(3))
    band = dict(WL.WORKLOADS["16k"].band)
    band.update(mid_block=64, mid_diag=1, mid_stride=4, high_window=100, n_summary=6)
    alloc = (4, 1, 2)
    want = O.forward(q, k, v, grid, O.BandConfig(**band), alloc)
    assert np.abs(want[0] - want[1]).max() > 1e-3      # the two batch entries really differ
    for path in (B.PATH_MFMA, B.PATH_GENERIC):
        ctx = B.Context(2, 3, d, grid, B.BF16, B.make_cfg(**band), path=path)
        dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
        out = torch.empty_like(dq)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            ctx.forward(dq, dk, dv, alloc, out)
        side.synchronize()
        got = U.to_host64(out)
        for b in range(2):
            for h in range(3):
                _check(got[b, h], want[b, h], "bf16", f"path {path} batch {b} head {h} mask {alloc[h]}")


def test_contexts_release_their_device_memory():
    """freqattn_destroy gives back everything freqattn_create took (tables, scratch, summary weights, partial-sum
    buffers): free device memory after twenty create/forward/destroy rounds is what it was after the first."""
    import torch
    wl = WL.WORKLOADS["64k"]
    heads = [0, 1, 2]
    q, k, v = _inputs(wl, heads=heads)
    dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
    out = torch.empty_like(dq)
    free = []
    for it in range(20):
        ctx, _ = U.make_ctx(wl, path=B.PATH_MFMA, heads=len(heads))
        ctx.forward(dq, dk, dv, (1, 2, 4), out)
        torch.cuda.synchronize()
        ctx.destroy()
        free.append(torch.cuda.mem_get_info()[0])
    assert free[0] - free[-1] < (64 << 20), (free[0], free[-1])   # (a context of this size holds over a gigabyte)
