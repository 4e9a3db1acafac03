"""GPU parity of the benchmark configurations as a whole: all heads of the 64K and 256K configurations with the router
in the loop, allocation compared with the oracle's on every head, outputs on one head per band mask.

Tolerance: max-abs <= 2e-2 and relative L2 <= 5e-3 on outputs; band outputs before the inverse transform (fp16, no bf16
output rounding) relative L2 <= 3e-3; router statistics 5e-3, probabilities 2e-3, allocations exact."""
import numpy as np
import pytest

from oracle import freqformer as O
from paper_2604_22808_amd import binding as B
from paper_2604_22808_amd import workloads as WL
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _check_heads(ctx, wl, q, k, v, out, alloc, heads, what):
    """Heads `heads` of device tensors against the oracle: output, and the band outputs Y^ of the active bands."""
    T, H, W = wl.grid
    cfg = O.BandConfig(**wl.band)
    for h in heads:
        mask = int(alloc[h])
        host = [U.to_host64(x[0, h]).reshape(T, H, W, wl.head_dim) for x in (q, k, v)]
        want, parts = O.head_forward(host[0], host[1], host[2], cfg, mask, return_parts=True)
        mx, rl = U.errors(U.to_host64(out[0, h]), want.reshape(-1, wl.head_dim))
        print(f"{what} head {h} mask {mask}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
        assert mx <= 2e-2 and rl <= 5e-3, (what, h, mask, mx, rl)
        for l in range(3):
            if (mask >> l) & 1:
                _, rl = U.errors(ctx.read_spectral(3, h, l), parts["Yhat"][l])
                print(f"{what} head {h} band {l} Y^: rel-L2 {rl:.3e}", flush=True)
                assert rl <= 3e-3, (what, h, l, rl)


def _one_head_per_mask(alloc):
    seen, heads = set(), []
    for h, m in enumerate(alloc):
        if int(m) and int(m) not in seen:
            seen.add(int(m))
            heads.append(h)
    return heads


def test_64k_configuration_all_24_heads_routed():
    """Configuration 3 in full: 24 heads, MLP router (hidden 64, seed 1) at t = 0.9.  Statistics are means over all
    heads, so only the whole configuration checks the allocation the benchmark reports."""
    import torch
    wl = WL.WORKLOADS["64k"]
    q, k, v = (WL.round_to_io(x, wl.dtype) for x in WL.qkv_numpy(wl))
    cfg = O.BandConfig(**wl.band)
    w = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
    t = wl.alloc["t"]
    want_stats = O.band_statistics(q, k, v, wl.grid, cfg)
    assert np.abs(U.band_statistics_library_transform(q, k, v, wl.grid, wl.band) - want_stats).max() < 1e-9
    want_alloc, want_pi = O.route_mlp(q, k, v, wl.grid, cfg, t, *w)
    ctx, _ = U.make_ctx(wl)
    dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
    got_alloc, got_pi, got_stats = ctx.route_mlp(dq, dk, dv, t, *w)
    print(f"64k x24: pi gpu {got_pi} oracle {want_pi}; alloc counts "
          f"{[int((got_alloc == m).sum()) for m in (1, 2, 4)]}", flush=True)
    assert np.abs(got_stats - want_stats).max() < 5e-3 and np.abs(got_pi - want_pi).max() < 2e-3
    assert np.array_equal(got_alloc, want_alloc)
    out = torch.empty_like(dq)
    for _ in range(2):          # the second call runs with the first call's allocation as its prediction
        alloc, _ = ctx.forward_routed(dq, dk, dv, t, *w, out)
        assert np.array_equal(alloc, want_alloc)
    torch.cuda.synchronize()
    _check_heads(ctx, wl, dq, dk, dv, out, alloc, _one_head_per_mask(alloc), "64k x24 routed")


@pytest.mark.parametrize("t", [0.9, 0.1])
def test_256k_configuration_routed_allocation_and_outputs(t):
    """Configuration 4 in full (24 heads, head_dim 128, 262,144 tokens), routed at t = 0.9 (low-heavy) and t = 0.1
    (high-heavy): the library's allocation equals the oracle's on all 24 heads; one head per mask against the oracle."""
    import torch
    wl = WL.WORKLOADS["256k"]
    q, k, v = WL.qkv_torch(wl, "cuda")
    w = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
    stats = U.band_statistics_library_transform(U.HeadsOnDemand(q), U.HeadsOnDemand(k), U.HeadsOnDemand(v), wl.grid, wl.band)
    want_alloc, want_pi = U.expected_route(stats, t, w, wl.heads)
    ctx = B.Context(wl.batch, wl.heads, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**wl.band))
    out = torch.empty_like(q)
    for _ in range(2):
        alloc, pi = ctx.forward_routed(q, k, v, t, *w, out)
    torch.cuda.synchronize()
    print(f"256k t={t}: pi gpu {pi} oracle {want_pi}; counts {[int((alloc == m).sum()) for m in (1, 2, 4)]}", flush=True)
    assert np.abs(pi - want_pi).max() < 2e-3
    assert np.array_equal(alloc, want_alloc)
    heads = _one_head_per_mask(alloc) if t == 0.9 else [int(np.flatnonzero(alloc == 4)[-1])]
    _check_heads(ctx, wl, q, k, v, out, alloc, heads, f"256k t={t}")
    plain = torch.empty_like(q)
    ctx.forward(q, k, v, alloc, plain)
    torch.cuda.synchronize()
    assert torch.equal(out, plain)


def test_band_limited_field_routes_like_the_oracle():
    """Noise-free input whose coefficients vanish outside the low+mid box: the high band holds no energy at all.  Total
    minus low minus mid is then pure rounding; the library must notice, take the statistics from whole-grid transforms
    and arrive at the oracle's numbers."""
    import torch
    from scipy.fft import idctn
    wl = WL.WORKLOADS["64k"]
    T, H, W = wl.grid
    d, nh = wl.head_dim, 4
    rng = np.random.default_rng(17)
    coef = rng.standard_normal((3, nh, T, H, W, d)) * WL.amplitude(T, H, W)[..., None]
    coef[:, :, T // 2:] = 0; coef[:, :, :, H // 2:] = 0; coef[:, :, :, :, W // 2:] = 0
    x = idctn(coef, type=2, norm="ortho", axes=(2, 3, 4)).reshape(3, 1, nh, T * H * W, d)
    q, k, v = (WL.round_to_io(x[i], "bf16") for i in range(3))
    cfg = O.BandConfig(**wl.band)
    w = WL.router_weights(64, 1)
    ctx, _ = U.make_ctx(wl, heads=nh)
    dq, dk, dv = (U.to_device(a, "bf16") for a in (q, k, v))
    want_stats = O.band_statistics(q, k, v, wl.grid, cfg)
    for t in (0.9, 0.1):
        got_alloc, got_pi, got_stats = ctx.route_mlp(dq, dk, dv, t, *w)
        want_alloc, want_pi = O.route_mlp(q, k, v, wl.grid, cfg, t, *w)
        print(f"band-limited t={t}: stats max diff {np.abs(got_stats - want_stats).max():.2e} pi {got_pi} / {want_pi}", flush=True)
        assert np.isfinite(got_pi).all()
        # the high band's statistic is log(1e-6 + rounding noise of bf16 inputs): compare it loosely, the others tightly
        assert np.abs(got_stats - want_stats)[:128].max() < 2e-2
        assert np.abs(got_pi - want_pi).max() < 2e-2
        assert np.array_equal(got_alloc, want_alloc)
    out = torch.empty_like(dq)
    alloc, _ = ctx.forward_routed(dq, dk, dv, 0.9, *w, out)
    torch.cuda.synchronize()
    want = O.forward(q, k, v, wl.grid, cfg, alloc)
    mx, rl = U.errors(U.to_host64(out), want)
    assert mx <= 2e-2 and rl <= 5e-3, (mx, rl)


@pytest.mark.parametrize("mid_block", [1, 5, 16])
def test_generic_path_small_mid_blocks_at_16k(mid_block):
    """Mid-band blocks far below the matrix-core tile on a 16K-token grid (1,792 mid tokens: up to 1,792 query blocks):
    the generic kernels walk the block list directly and need no work-item lists."""
    wl = WL.WORKLOADS["16k"]
    q, k, v = (WL.round_to_io(x, "bf16") for x in WL.qkv_numpy(wl, heads=[3]))
    band = dict(wl.band, mid_block=mid_block, mid_stride=8 if mid_block > 1 else 64, n_summary=4)
    ctx = B.Context(1, 1, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**band))
    assert ctx.get_path() == B.PATH_GENERIC
    got = U.run_forward(ctx, q, k, v, "bf16", [2])
    want = O.forward(q, k, v, wl.grid, O.BandConfig(**band), [2])
    mx, rl = U.errors(got, want)
    print(f"generic mid_block={mid_block}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 2e-2 and rl <= 5e-3


@pytest.mark.parametrize("edges", [dict(mid_num=1, mid_den=4), dict(mid_num=1, mid_den=1)])
def test_two_band_layouts_on_both_paths(edges):
    """Band count L = 2: the mid band empty (low + windowed rest) or the high band empty (low + block-sparse rest), on
    the matrix-core path at 16K tokens and on the generic fp32 path."""
    wl = WL.WORKLOADS["16k"]
    q, k, v = (WL.round_to_io(x, "bf16") for x in WL.qkv_numpy(wl, heads=[0, 4, 7]))
    band = dict(wl.band, **edges)
    ctx = B.Context(1, 3, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**band))
    assert ctx.get_path() == B.PATH_MFMA and 0 in ctx.band_sizes()
    alloc = (1, 6, 7)
    got = U.run_forward(ctx, q, k, v, "bf16", alloc)
    want = O.forward(q, k, v, wl.grid, O.BandConfig(**band), alloc)
    for s in range(3):
        mx, rl = U.errors(got[0, s], want[0, s])
        print(f"two bands {edges} mask {alloc[s]}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
        assert mx <= 2e-2 and rl <= 5e-3
    tiny = WL.WORKLOADS["tiny_f32"]
    q, k, v = (WL.round_to_io(x, "f32") for x in WL.qkv_numpy(tiny))
    bandt = dict(tiny.band, **edges)
    ctx = B.Context(1, 2, tiny.head_dim, tiny.grid, B.F32, B.make_cfg(**bandt))
    got = U.run_forward(ctx, q, k, v, "f32", (7, 3))
    want = O.forward(q, k, v, tiny.grid, O.BandConfig(**bandt), (7, 3))
    mx, rl = U.errors(got, want)
    assert mx <= 1e-5 and rl <= 1e-5


def test_paper_dimension_router_hidden_128():
    """The router at the paper's dimensions (256 -> 128 -> 3: 33,283 parameters, section 3.5) on the 64K grid."""
    wl = WL.WORKLOADS["64k"]
    heads = [0, 5, 11, 17, 23]
    q, k, v = (WL.round_to_io(x, "bf16") for x in WL.qkv_numpy(wl, heads=heads))
    w = WL.router_weights(128, 3)
    assert sum(a.size for a in w) == 33283
    w = (w[0], (0.1 * np.random.default_rng(5).standard_normal(128)).astype(np.float32), w[2], np.array([0.2, -0.1, 0.05], np.float32))
    ctx, band = U.make_ctx(wl, heads=len(heads))
    dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
    for t in (0.9, 0.3):
        got_alloc, got_pi, got_stats = ctx.route_mlp(dq, dk, dv, t, *w)
        want_alloc, want_pi = O.route_mlp(q, k, v, wl.grid, U.oracle_cfg(band), t, *w)
        assert np.abs(got_pi - want_pi).max() < 2e-3 and np.array_equal(got_alloc, want_alloc)
        lb = B.load_balance(np.tile(got_pi, (len(heads), 1)), 0.01)
        assert abs(lb - O.load_balance_loss(np.tile(want_pi, (len(heads), 1)), 0.01)) < 1e-5


def test_inputs_beyond_the_fp16_range_are_reported():
    """sqrt(N) * mean = 256 * 300 > 65504 at 64K tokens: the DC coefficient does not fit fp16.  The plain forward marks
    it on the device (freqattn_check_range), the routed forward refuses by itself; the context stays usable, and the same
    input is fine on the fp32 kernels."""
    import torch
    wl = WL.WORKLOADS["64k"]
    ctx, band = U.make_ctx(wl, heads=2)
    g = torch.Generator(device="cuda").manual_seed(3)
    x = torch.randn((1, 2, wl.n_tokens, wl.head_dim), device="cuda", generator=g)
    ok = (0.5 * x).to(torch.bfloat16)
    big = (300.0 + x).to(torch.bfloat16)
    out = torch.empty_like(ok)
    ctx.forward(ok, ok, ok.clone(), (2, 4), out)
    assert ctx.check_range() == 0
    ctx.forward(big, big, big.clone(), (2, 4), out)
    with pytest.raises(B.FreqAttnError) as e:
        ctx.check_range()
    assert e.value.status == B.ERANGE
    assert ctx.check_range() == 0                       # the mark is cleared by the check
    w = WL.router_weights(64, 1)
    with pytest.raises(B.FreqAttnError) as e:
        ctx.forward_routed(big, big, big.clone(), 0.5, *w, out)
    assert e.value.status == B.ERANGE
    alloc, pi = ctx.forward_routed(ok, ok, ok.clone(), 0.5, *w, out)      # still usable
    torch.cuda.synchronize()
    assert np.isfinite(pi).all() and torch.isfinite(out.float()).all()


def test_ablation_speed_sweep_helper():
    """The speed sweep over the paper's ablation dimensions (section 8's list) times real forwards: its helper must run a
    changed configuration end to end and report the mid band's keys per query from the library's own block list."""
    import torch
    from paper_2604_22808_amd import sweep
    wl = WL.WORKLOADS["16k"]
    sweep.time_forward.inputs = WL.qkv_torch(wl, "cuda")
    sweep.time_forward.out = torch.empty_like(sweep.time_forward.inputs[0])
    ms0, keys0 = sweep.time_forward(wl, dict(wl.band), steps=2, warmup=1)
    ms1, keys1 = sweep.time_forward(wl, dict(wl.band, mid_stride=4, high_window=64), steps=2, warmup=1)
    assert ms0 > 0 and ms1 > 0 and keys1 > keys0 > 0
    assert torch.isfinite(sweep.time_forward.out.float()).all()
    ms4, _ = sweep.time_forward(wl, dict(wl.band, mid2_num=3, mid2_den=4), steps=2, warmup=1,
                                alloc=[1, 1, 2, 2, 8, 8, 4, 4])     # the band-count rows: a four-band context, given allocation
    assert ms4 > 0 and torch.isfinite(sweep.time_forward.out.float()).all()


@pytest.mark.parametrize("name,heads,alloc,extra", [("16k", 8, (1, 1, 2, 2, 2, 4, 4, 7), {}), ("64k", 6, (1, 2, 4, 3, 0, 6), {}),
                                                   ("16k", 8, (8, 9, 15, 6, 12, 10, 0, 1), dict(mid2_num=3, mid2_den=4))])
def test_projected_forward_matches_oracle(name, heads, alloc, extra, monkeypatch):
    """Projections folded around the path (sections 3.1, 3.7): X transformed once, Q~/K~/V~ projected from spectral rows
    of the bands a head runs (what it passes through goes from X~ straight into the output projection, its summary tokens
    from pooled rows of X~), W_O applied before one inverse transform of model width - against the oracle's
    project-then-forward definition."""
    import torch
    wl = WL.WORKLOADS[name]
    d, N = wl.head_dim, wl.n_tokens
    dm = heads * d
    rng = np.random.default_rng(23)
    xs = np.stack([WL.field_numpy(wl.grid, d, 5, 0, h) for h in range(heads)], axis=1).reshape(1, N, dm)   # field per channel group
    x = WL.round_to_io(xs, "bf16")
    wq, wk, wv = (WL.round_to_io(rng.standard_normal((dm, dm)) / np.sqrt(dm), "bf16") for _ in range(3))
    wo = WL.round_to_io(rng.standard_normal((dm, dm)) / np.sqrt(dm), "bf16")
    band = dict(wl.band, **extra)      # (the third case: a four-band context)
    ctx = B.Context(1, heads, d, wl.grid, B.BF16, B.make_cfg(**band))
    dev = lambda a: U.to_device(a, "bf16")
    dx, dwq, dwk, dwv, dwo = dev(x), dev(wq), dev(wk), dev(wv), dev(wo)
    out = torch.empty_like(dx)
    for _ in range(2):           # second call: buffers and tables exist
        ctx.forward_projected(dx, dwq, dwk, dwv, dwo, alloc, out)
    torch.cuda.synchronize()
    assert ctx.check_range() == 0
    got = U.to_host64(out)
    want = O.forward_projected(x, wq, wk, wv, wo, wl.grid, O.BandConfig(**band), alloc)
    mx, rl = U.errors(got, want)
    print(f"projected {name}: max-abs {mx:.3e} rel-L2 {rl:.3e} (|want| max {np.abs(want).max():.2f})", flush=True)
    assert mx <= 2e-2 and rl <= 5e-3
    # the same without the pass-through folding (V~ projected on every row, pooled and sent through W_O per head)
    monkeypatch.setenv("FREQATTN_PROJ_FOLD", "0")
    ctx.forward_projected(dx, dwq, dwk, dwv, dwo, alloc, out)
    torch.cuda.synchronize()
    mx, rl = U.errors(U.to_host64(out), want)
    print(f"projected {name} without pass-through folding: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 2e-2 and rl <= 5e-3
    monkeypatch.delenv("FREQATTN_PROJ_FOLD")
    # another allocation on the same context: new product tables
    alloc2 = tuple(reversed(alloc))
    ctx.forward_projected(dx, dwq, dwk, dwv, dwo, alloc2, out)
    torch.cuda.synchronize()
    want2 = O.forward_projected(x, wq, wk, wv, wo, wl.grid, O.BandConfig(**band), alloc2)
    mx, rl = U.errors(U.to_host64(out), want2)
    print(f"projected {name} second allocation: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 2e-2 and rl <= 5e-3


@pytest.mark.parametrize("name,heads,alloc", [("16k", [0, 1, 2, 3, 4, 5, 6], (1, 2, 4, 3, 5, 7, 0)), ("256k", [0, 7, 19], (1, 2, 4))])
def test_exchange_inside_the_band_items_is_bit_identical(name, heads, alloc):
    """Slices that run one band carry the cross-band exchange inside their band items (the output tile never leaves the
    registers between the band operator and the exchange); slices that run several bands use the separate launch.  Same
    arithmetic on the same fp16 values: the outputs must equal those of the all-separate route bit for bit, in both
    launch modes; m = 5 gives a ragged summary tile."""
    import torch
    wl = WL.WORKLOADS[name]
    q, k, v = (U.to_device(WL.round_to_io(x, "bf16"), "bf16") for x in WL.qkv_numpy(wl, heads=heads)) if name == "16k" else \
        [t[:, heads].contiguous() for t in WL.qkv_torch(wl, "cuda")]
    for extra in (dict(), dict(n_summary=5)):
        ctx, _ = U.make_ctx(wl, heads=len(heads), **extra)
        a, b, c2 = (torch.empty_like(q) for _ in range(3))
        ctx.forward(q, k, v, alloc, a)
        ctx.set_exchange_fusion(False)
        ctx.forward(q, k, v, alloc, b)
        ctx.set_exchange_fusion(True)
        ctx.set_launch_mode(B.LAUNCH_SEPARATE)
        ctx.forward(q, k, v, alloc, c2)
        torch.cuda.synchronize()
        assert torch.equal(a, b) and torch.equal(a, c2), (name, extra)
        ctx.destroy()


def test_forward_replays_from_a_hip_graph():
    """The plain forward enqueues kernels only (no synchronisation, no allocation, no memset nodes) once its allocation
    is known, so it can be captured in a HIP graph - what a launch-bound sampling loop at 16K-64K tokens wants.  The
    graph is replayed several times with eager work and synchronisations in between; every replay must give the eager
    result bit for bit."""
    import torch
    wl = WL.WORKLOADS["16k"]
    q, k, v = (U.to_device(WL.round_to_io(x, "bf16"), "bf16") for x in WL.qkv_numpy(wl))
    alloc = B.route_fixed(wl.heads, *wl.alloc["counts"])
    ctx, _ = U.make_ctx(wl)
    eager = torch.empty_like(q)
    ctx.forward(q, k, v, alloc, eager)           # also uploads the work lists of this allocation
    torch.cuda.synchronize()
    out = torch.empty_like(q)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        ctx.forward(q, k, v, alloc, out)
    for rep in range(4):
        out.zero_()
        q2 = (q.float() * (1.0 + 0.25 * rep)).to(torch.bfloat16)     # eager work between the replays, new inputs
        q.copy_(q2)
        ctx.forward(q, k, v, alloc, eager)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep


def test_batch_of_two_router_in_the_loop():
    """batch 2 x 4 heads on the 16K grid, router in the loop: the statistics are means over both batch entries (section
    3.5), the allocation repeats per batch entry, and the routed output must equal the plain forward with it bit for bit
    and the oracle within the tolerance."""
    import torch
    wl = WL.WORKLOADS["16k"]
    d, N = wl.head_dim, wl.n_tokens
    q, k, v = (np.stack([np.stack([WL.field_numpy(wl.grid, d, 40 + b, s, h) for h in range(4)]) for b in range(2)]).reshape(2, 4, N, d)
               for s in range(3))
    q, k, v = (WL.round_to_io(x, "bf16") for x in (q, k, v))
    band = dict(wl.band)
    cfg = O.BandConfig(**band)
    w = WL.router_weights(64, 1)
    ctx = B.Context(2, 4, d, wl.grid, B.BF16, B.make_cfg(**band))
    assert ctx.get_path() == B.PATH_MFMA
    dq, dk, dv = (U.to_device(x, "bf16") for x in (q, k, v))
    out = torch.empty_like(dq); plain = torch.empty_like(dq)
    for t in (0.8, 0.2):
        for _ in range(2):     # second call: the prediction from the first
            alloc, pi = ctx.forward_routed(dq, dk, dv, t, *w, out)
        torch.cuda.synchronize()
        alloc = [int(a) for a in alloc]
        stats = U.band_statistics_library_transform(q, k, v, wl.grid, band)
        want_alloc, want_pi = U.expected_route(stats, t, w, 4)
        print(f"batch 2 routed t={t}: allocation {alloc} pi {pi} oracle {list(want_alloc)} {want_pi}", flush=True)
        assert np.abs(pi - want_pi).max() < 2e-3 and alloc == [int(a) for a in want_alloc]
        ctx.forward(dq, dk, dv, alloc, plain)
        torch.cuda.synchronize()
        assert torch.equal(out, plain)
        want = O.forward(q, k, v, wl.grid, cfg, alloc)
        mx, rl = U.errors(U.to_host64(out), want)
        print(f"batch 2 routed t={t}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
        assert mx <= 2e-2 and rl <= 5e-3


def test_projected_forward_batch_of_two():
    """The folded layer with batch 2 (the product launches group by batch entry)."""
    import torch
    wl = WL.WORKLOADS["16k"]
    heads, alloc = 4, (1, 2, 4, 6)
    d, N = wl.head_dim, wl.n_tokens
    dm = heads * d
    rng = np.random.default_rng(29)
    xs = np.stack([np.stack([WL.field_numpy(wl.grid, d, 50 + b, 0, h) for h in range(heads)], axis=1).reshape(N, dm) for b in range(2)])
    x = WL.round_to_io(xs, "bf16")
    wq, wk, wv, wo = (WL.round_to_io(rng.standard_normal((dm, dm)) / np.sqrt(dm), "bf16") for _ in range(4))
    band = dict(wl.band)
    ctx = B.Context(2, heads, d, wl.grid, B.BF16, B.make_cfg(**band))
    dev = lambda a: U.to_device(a, "bf16")
    dx, dwq, dwk, dwv, dwo = dev(x), dev(wq), dev(wk), dev(wv), dev(wo)
    out = torch.empty_like(dx)
    ctx.forward_projected(dx, dwq, dwk, dwv, dwo, alloc, out)
    torch.cuda.synchronize()
    assert ctx.check_range() == 0
    want = O.forward_projected(x, wq, wk, wv, wo, wl.grid, O.BandConfig(**band), alloc)
    assert np.abs(want[0] - want[1]).max() > 1e-3
    mx, rl = U.errors(U.to_host64(out), want)
    print(f"projected batch 2: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 2e-2 and rl <= 5e-3


def test_projected_forward_on_a_ragged_grid():
    """Grid 16 x 48 x 80 (61,440 tokens; bands of 960 / 6,720 / 53,760 rows, none a multiple of the products' 256-row
    tiles), head_dim 128, 3 heads: the last row tile of every product launch is partly empty."""
    import torch
    grid, d, heads, alloc = (16, 48, 80), 128, 3, (1, 2, 4)
    N = int(np.prod(grid))
    dm = heads * d
    rng = np.random.default_rng(31)
    xs = np.stack([WL.field_numpy(grid, d, 60, 0, h) for h in range(heads)], axis=1).reshape(1, N, dm)
    x = WL.round_to_io(xs, "bf16")
    wq, wk, wv, wo = (WL.round_to_io(rng.standard_normal((dm, dm)) / np.sqrt(dm), "bf16") for _ in range(4))
    band = dict(WL.WORKLOADS["16k"].band)
    band.update(mid_block=128, mid_diag=1, mid_stride=5, high_window=200, n_summary=7, low_compress=4)
    ctx = B.Context(1, heads, d, grid, B.BF16, B.make_cfg(**band))
    assert ctx.get_path() == B.PATH_MFMA
    assert any(n % 256 for n in ctx.band_sizes())
    dev = lambda a: U.to_device(a, "bf16")
    dx, dwq, dwk, dwv, dwo = dev(x), dev(wq), dev(wk), dev(wv), dev(wo)
    out = torch.empty_like(dx)
    ctx.forward_projected(dx, dwq, dwk, dwv, dwo, alloc, out)
    torch.cuda.synchronize()
    assert ctx.check_range() == 0
    want = O.forward_projected(x, wq, wk, wv, wo, grid, O.BandConfig(**band), alloc)
    mx, rl = U.errors(U.to_host64(out), want)
    print(f"projected ragged grid: bands {ctx.band_sizes()} max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
    assert mx <= 2e-2 and rl <= 5e-3


def test_four_band_layout_on_both_paths():
    """Band count L = 4 (the band-count ablation of section 8): a second block-sparse band between the mid edge and a
    third edge at 3/4 of every axis.  Matrix-core path at 16K tokens (bands of 256 / 1,792 / 9,472 / 4,864 coefficients),
    one head per mask: each band alone, pairs across the new band, all four, and a head that passes everything through;
    band outputs of the new band are compared before the inverse transform as well.  Then the generic fp32 path on the
    tiny grid.  The routed entry points refuse such a context (section 3.5 scores three bands)."""
    wl = WL.WORKLOADS["16k"]
    alloc = (8, 9, 15, 6, 12, 10, 0, 1, 4)
    heads = list(range(len(alloc)))
    q, k, v = (WL.round_to_io(x, "bf16") for x in WL.qkv_numpy(wl, heads=[h % wl.heads for h in heads]))
    band = dict(wl.band, mid2_num=3, mid2_den=4)
    cfg = O.BandConfig(**band)
    ctx = B.Context(1, len(alloc), wl.head_dim, wl.grid, B.BF16, B.make_cfg(**band))
    assert ctx.get_path() == B.PATH_MFMA and ctx.band_sizes() == [256, 1792, 9472, 4864]
    T, H, W = wl.grid
    wants = []
    for s, mask in enumerate(alloc):
        host = [x[0, s].astype(np.float64).reshape(T, H, W, wl.head_dim) for x in (q, k, v)]
        wants.append(O.head_forward(host[0], host[1], host[2], cfg, mask, return_parts=True))
    for fusion in (1, 0):
        ctx.set_exchange_fusion(fusion)
        got = U.run_forward(ctx, q, k, v, "bf16", alloc)
        for s, mask in enumerate(alloc):
            want, parts = wants[s]
            mx, rl = U.errors(got[0, s], want.reshape(-1, wl.head_dim))
            print(f"four bands fusion={fusion} mask {mask}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
            assert mx <= 2e-2 and rl <= 5e-3, (mask, mx, rl)
            for l in range(4):
                if (mask >> l) & 1:
                    _, rl = U.errors(ctx.read_spectral(3, s, l), parts["Yhat"][l])
                    assert rl <= 3e-3, (mask, l, rl)
    with pytest.raises(B.FreqAttnError):
        U.run_forward(ctx, q, k, v, "bf16", (16,) + alloc[1:])     # a fifth band does not exist
    import torch
    qd, kd, vd = (U.to_device(x, "bf16") for x in (q, k, v))
    w = WL.router_weights(64, 1)
    for call in (lambda: ctx.forward_routed(qd, kd, vd, 0.5, *w, torch.empty_like(qd)),
                 lambda: ctx.route_mlp(qd, kd, vd, 0.5, *w)):
        with pytest.raises(B.FreqAttnError) as e:
            call()
        assert e.value.status == B.EUNSUPPORTED
    tiny = WL.WORKLOADS["tiny_f32"]
    q, k, v = (WL.round_to_io(x, "f32") for x in WL.qkv_numpy(tiny))
    bandt = dict(tiny.band, mid2_num=3, mid2_den=4)
    ctx = B.Context(1, 2, tiny.head_dim, tiny.grid, B.F32, B.make_cfg(**bandt))
    assert ctx.get_path() == B.PATH_GENERIC and len(ctx.band_sizes()) == 4 and min(ctx.band_sizes()) > 0
    for allocs in ((15, 9), (8, 14), (5, 10)):
        got = U.run_forward(ctx, q, k, v, "f32", allocs)
        want = O.forward(q, k, v, tiny.grid, O.BandConfig(**bandt), allocs)
        mx, rl = U.errors(got, want)
        print(f"four bands fp32 {allocs}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
        assert mx <= 1e-5 and rl <= 1e-5


@pytest.mark.parametrize("edges,m", [(dict(mid2_num=3, mid2_den=4), 8), (dict(mid2_num=1, mid2_den=2), 8),
                                      (dict(mid2_num=1, mid2_den=1), 8), (dict(mid2_num=2, mid2_den=3), 0),
                                      (dict(mid2_num=3, mid2_den=4), 100)])
def test_four_band_edge_cases_on_a_ragged_grid(edges, m):
    """Four-band contexts where the layout degenerates - the second mid band empty (third edge = mid edge), the high band
    empty (third edge = 1) - without exchange (m = 0), with an edge that cuts the axes at non-integers (2/3 of 16, 32,
    48) and with m = 100 summary tokens per band (300 summary keys per query: five key tiles in the exchange, chunks of
    unequal length); head_dim 128 with 128-token
    blocks (128 query rows per work item) on a grid whose bands are no multiples of the tiles."""
    grid, d = (16, 32, 48), 128
    band = dict(low_num=1, low_den=4, mid_num=1, mid_den=2, low_compress=4, mid_block=128, mid_diag=1, mid_stride=4,
                mid_block0=1, high_window=128, n_summary=m, **edges)
    alloc = (8, 15, 12, 3, 5)
    rng = np.random.default_rng(77)
    N = int(np.prod(grid))
    q, k, v = (WL.round_to_io(0.5 * rng.standard_normal((1, len(alloc), N, d)), "bf16") for _ in range(3))
    ctx = B.Context(1, len(alloc), d, grid, B.BF16, B.make_cfg(**band))
    cfg = O.BandConfig(**band)
    sizes = [len(ix) for ix in O.band_partition(*grid, cfg)]
    assert ctx.get_path() == B.PATH_MFMA and ctx.band_sizes() == sizes
    got = U.run_forward(ctx, q, k, v, "bf16", alloc)
    want = O.forward(q, k, v, grid, cfg, alloc)
    for s, mask in enumerate(alloc):
        mx, rl = U.errors(got[0, s], want[0, s])
        print(f"four bands {edges} m={m} sizes {sizes} mask {mask}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
        assert mx <= 2e-2 and rl <= 5e-3, (edges, m, mask, mx, rl)


def test_block_sparse_items_with_more_than_64_key_blocks():
    """The matrix-core kernel holds a work item's key-block list in one register, 64 entries at a time: a pattern
    dense enough to give every query block about 130 key blocks (the block-sparse band over 63/64 of a 16K grid, every
    second block strided in) walks through several refills."""
    wl = WL.WORKLOADS["16k"]
    band = dict(wl.band, mid_num=1, mid_den=1, mid_stride=2)
    q, k, v = (WL.round_to_io(x, "bf16") for x in WL.qkv_numpy(wl, heads=[1, 6]))
    ctx = B.Context(1, 2, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**band))
    rp, ci = ctx.mid_blocks()
    assert ctx.get_path() == B.PATH_MFMA and int(np.diff(rp).max()) > 2 * 64
    alloc = (2, 3)
    got = U.run_forward(ctx, q, k, v, "bf16", alloc)
    want = O.forward(q, k, v, wl.grid, O.BandConfig(**band), alloc)
    for s in range(2):
        mx, rl = U.errors(got[0, s], want[0, s])
        print(f"dense block pattern mask {alloc[s]}: max-abs {mx:.3e} rel-L2 {rl:.3e}", flush=True)
        assert mx <= 2e-2 and rl <= 5e-3
