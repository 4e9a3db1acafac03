"""GPU parity at the full benchmark sizes (256K and 1M tokens, head_dim 128) in the launch configuration bench.py times
(MFMA path, fused branch launch, exchange on): one head per band mask, every output element against the fp64 oracle.

Inputs come from the device variant of the seeded field recipe and are copied to the host as stored (bf16) values, so
the oracle and the library see the same numbers.  Tolerance: max-abs <= 2e-2, relative L2 <= 5e-3."""
import dataclasses

import numpy as np
import pytest

from oracle import freqformer as O
from paper_2604_22808_amd import binding as B
from paper_2604_22808_amd import workloads as WL
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _one_head(name, mask):
    import torch
    wl = dataclasses.replace(WL.WORKLOADS[name], heads=1, seed=100 + mask)
    q, k, v = WL.qkv_torch(wl, "cuda")
    ctx = B.Context(1, 1, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**wl.band))
    assert ctx.get_path() == B.PATH_MFMA
    out = torch.empty_like(q)
    ctx.forward(q, k, v, [mask], out)
    torch.cuda.synchronize()
    T, H, W = wl.grid
    host = [U.to_host64(x)[0, 0].reshape(T, H, W, wl.head_dim) for x in (q, k, v)]
    want, parts = O.head_forward(host[0], host[1], host[2], O.BandConfig(**wl.band), mask, return_parts=True)
    want = want.reshape(-1, wl.head_dim)
    got = U.to_host64(out)[0, 0]
    mx, rl = U.errors(got, want)
    print(f"{name} mask {mask}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 2e-2 and rl <= 5e-3, (name, mask, mx, rl)
    # For a one-hot mask most of the output is V passed through, which dilutes the bound above: the active bands'
    # outputs before the inverse transform (fp16, no output rounding) are compared on their own.
    for l in range(3):
        if (mask >> l) & 1:
            _, rl = U.errors(ctx.read_spectral(3, 0, l), parts["Yhat"][l])
            print(f"{name} mask {mask} band {l} Y^: rel-L2 {rl:.3e}", flush=True)
            assert rl <= 3e-3, (name, mask, l, rl)
    return ctx, q, k, v, out


@pytest.mark.parametrize("mask", [1, 2, 4, 7])
def test_256k_head_matches_oracle(mask):
    _one_head("256k", mask)


@pytest.mark.parametrize("mask", [1, 2, 4])
def test_1m_head_matches_oracle(mask):
    _one_head("1m", mask)


def test_1m_launch_modes_agree_and_idle_head_returns_v():
    """Properties that hold at any size: fused and per-branch launches give the same bits; a head with no active band
    returns V up to the transforms' rounding."""
    import torch
    wl = dataclasses.replace(WL.WORKLOADS["1m"], heads=4, seed=7)
    q, k, v = WL.qkv_torch(wl, "cuda")
    ctx = B.Context(1, 4, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**wl.band))
    a = torch.empty_like(q); b = torch.empty_like(q)
    alloc = [1, 2, 4, 0]
    ctx.forward(q, k, v, alloc, a)
    ctx.set_launch_mode(B.LAUNCH_SEPARATE)
    ctx.forward(q, k, v, alloc, b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    diff = (a[0, 3].float() - v[0, 3].float())
    rel = float(diff.norm() / v[0, 3].float().norm())
    print(f"1m idle head: max-abs {float(diff.abs().max()):.3e} rel-L2 {rel:.3e}", flush=True)
    assert float(diff.abs().max()) <= 2e-2 and rel <= 5e-3


def test_1m_benchmark_configuration_routed_with_prediction():
    """The configuration bench.py times: 16 heads, router in the loop at t = 0.5, second call with the first call's
    allocation as the prediction (V~ of heads without the high band on the low+mid box, their high-band summaries from
    the untransformed V).  The routed output must equal the plain forward with the same allocation bit for bit, and
    one head per band is compared with the oracle on every element."""
    import torch
    wl = WL.WORKLOADS["1m"]
    q, k, v = WL.qkv_torch(wl, "cuda")
    cfg = B.make_cfg(**wl.band)
    ctx = B.Context(wl.batch, wl.heads, wl.head_dim, wl.grid, B.BF16, cfg)
    assert ctx.get_path() == B.PATH_MFMA and ctx.get_v_box() == 1
    w = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
    out = torch.empty_like(q); plain = torch.empty_like(q)
    for _ in range(2):
        alloc, pi = ctx.forward_routed(q, k, v, wl.alloc["t"], *w, out)
    torch.cuda.synchronize()
    alloc = [int(a) for a in alloc]
    print(f"1m routed allocation {alloc} pi {pi}", flush=True)
    stats = U.band_statistics_library_transform(U.HeadsOnDemand(q), U.HeadsOnDemand(k), U.HeadsOnDemand(v), wl.grid, wl.band)
    want_alloc, want_pi = U.expected_route(stats, wl.alloc["t"], w, wl.heads)
    print(f"1m oracle allocation {list(want_alloc)} pi {want_pi}", flush=True)
    assert np.abs(pi - want_pi).max() < 2e-3 and alloc == [int(a) for a in want_alloc]
    ctx.forward(q, k, v, alloc, plain)
    torch.cuda.synchronize()
    assert torch.equal(out, plain)
    T, H, W = wl.grid
    seen = set()
    for h, mask in enumerate(alloc):
        if mask in seen or mask == 0:
            continue
        seen.add(mask)
        host = [U.to_host64(x[:, h:h + 1])[0, 0].reshape(T, H, W, wl.head_dim) for x in (q, k, v)]
        want = O.head_forward(host[0], host[1], host[2], O.BandConfig(**wl.band), mask).reshape(-1, wl.head_dim)
        got = U.to_host64(out[:, h:h + 1])[0, 0]
        mx, rl = U.errors(got, want)
        print(f"1m routed head {h} mask {mask}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
        assert mx <= 2e-2 and rl <= 5e-3, (h, mask, mx, rl)


def _one_head_on(grid, head_dim, mask, seed, band=None):
    """One head on an arbitrary grid in the bench's launch configuration, every output element against the oracle."""
    import torch
    base = WL.WORKLOADS["1m"]
    wl = dataclasses.replace(base, grid=tuple(grid), head_dim=head_dim, heads=1, seed=seed, band=dict(band or base.band))
    q, k, v = WL.qkv_torch(wl, "cuda")
    ctx = B.Context(1, 1, head_dim, wl.grid, B.BF16, B.make_cfg(**wl.band))
    assert ctx.get_path() == B.PATH_MFMA
    out = torch.empty_like(q)
    ctx.forward(q, k, v, [mask], out)
    torch.cuda.synchronize()
    T, H, W = wl.grid
    host = [U.to_host64(x)[0, 0].reshape(T, H, W, head_dim) for x in (q, k, v)]
    want, parts = O.head_forward(host[0], host[1], host[2], O.BandConfig(**wl.band), mask, return_parts=True)
    got = U.to_host64(out)[0, 0]
    mx, rl = U.errors(got, want.reshape(-1, head_dim))
    print(f"grid {grid} d {head_dim} mask {mask}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 2e-2 and rl <= 5e-3, (grid, mask, mx, rl)
    for l in range(3):
        if (mask >> l) & 1:
            _, rl = U.errors(ctx.read_spectral(3, 0, l), parts["Yhat"][l])
            print(f"grid {grid} mask {mask} band {l} Y^: rel-L2 {rl:.3e}", flush=True)
            assert rl <= 3e-3, (grid, mask, l, rl)


@pytest.mark.parametrize("mask", [3, 4])
def test_largest_grid_the_matrix_core_path_takes(mask):
    """128 x 128 x 128 = 2,097,152 tokens, the largest grid of the MFMA path (every axis at its 128-row limit, so the
    T-axis passes run their 128-row variants): low + mid on one head, the window branch on another."""
    band = dict(WL.WORKLOADS["1m"].band, high_window=128, mid_stride=64)   # (narrower patterns: the oracle's time)
    _one_head_on((128, 128, 128), 64, mask, seed=300 + mask, band=band)


@pytest.mark.parametrize("mask", [1, 6])
def test_axis_lengths_that_are_not_powers_of_two(mask):
    """32 x 96 x 112 tokens (344,064): axis lengths whose passes cannot be pruned to a coefficient box (96- and 112-row
    variants of the transform passes), head_dim 128."""
    _one_head_on((32, 96, 112), 128, mask, seed=310 + mask)


def test_routed_forward_on_an_odd_grid_matches_the_plain_forward():
    """Router in the loop on 32 x 96 x 112 with 4 heads: statistics from the passes' own sums against the oracle's
    statistics of the same spectra, and the routed output against the plain forward with that allocation (same bits)."""
    import torch
    base = WL.WORKLOADS["1m"]
    wl = dataclasses.replace(base, grid=(32, 96, 112), head_dim=128, heads=4, seed=77)
    q, k, v = WL.qkv_torch(wl, "cuda")
    ctx = B.Context(1, 4, 128, wl.grid, B.BF16, B.make_cfg(**wl.band))
    assert ctx.get_path() == B.PATH_MFMA
    w = WL.router_weights(64, 1)
    out = torch.empty_like(q); plain = torch.empty_like(q)
    for _ in range(2):
        alloc, pi = ctx.forward_routed(q, k, v, 0.5, *w, out)
    torch.cuda.synchronize()
    alloc = [int(a) for a in alloc]
    stats = U.band_statistics_library_transform(U.HeadsOnDemand(q), U.HeadsOnDemand(k), U.HeadsOnDemand(v), wl.grid, wl.band)
    want_alloc, want_pi = U.expected_route(stats, 0.5, w, 4)
    print(f"odd grid routed allocation {alloc} pi {pi} oracle {list(want_alloc)} {want_pi}", flush=True)
    assert np.abs(pi - want_pi).max() < 2e-3 and alloc == [int(a) for a in want_alloc]
    ctx.forward(q, k, v, alloc, plain)
    torch.cuda.synchronize()
    assert torch.equal(out, plain)
