"""freqattn_forward_static (all device buffers inside the library's static device array, no allocation) against
freqattn_forward: same kernels, same layout, so the outputs must agree bit for bit.  Two calls in a row, the second
with a smaller input, then back to the first shape; a shape that does not fit is refused with a clear error."""
import numpy as np
import pytest

from paper_2604_22808_amd import binding as B
from paper_2604_22808_amd import workloads as WL
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _case(grid, heads, d, dtype, band, alloc, seed):
    import torch
    rng = np.random.default_rng(seed)
    N = int(np.prod(grid))
    io = "bf16" if dtype == B.BF16 else "f32"
    q, k, v = (U.to_device(WL.round_to_io(0.4 * rng.standard_normal((1, heads, N, d)), io), io) for _ in range(3))
    ref_ctx = B.Context(1, heads, d, grid, dtype, B.make_cfg(**band))
    want = torch.empty_like(q)
    ref_ctx.forward(q, k, v, alloc, want)
    torch.cuda.synchronize()
    # the context handed to the static entry point never touched the device: no allocation anywhere on this route
    ctx = B.Context(1, heads, d, grid, dtype, B.make_cfg(**band), path=B.PATH_TABLES_ONLY)
    return ctx, (q, k, v), want, ref_ctx.get_path()


def test_forward_static_matches_forward_on_two_calls_in_a_row():
    import torch
    band = dict(WL.WORKLOADS["16k"].band)
    band.update(mid_block=64, mid_diag=1, mid_stride=3, high_window=100, n_summary=6)
    big = _case((16, 16, 32), 4, 64, B.BF16, band, (1, 2, 4, 7), 31)        # 8,192 tokens, matrix-core kernels
    small = _case((4, 8, 8), 2, 64, B.F32, dict(WL.WORKLOADS["tiny_f32"].band), (3, 4), 32)   # 256 tokens, fp32 kernels
    assert big[3] == B.PATH_MFMA and small[3] == B.PATH_GENERIC
    torch.cuda.synchronize()
    for rnd, (ctx, (q, k, v), want, _) in enumerate((big, small, big, small)):
        alloc = (1, 2, 4, 7) if ctx is big[0] else (3, 4)
        got = torch.full_like(q, float("nan"))
        got2 = torch.full_like(q, float("nan"))
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        ctx.forward_static(q, k, v, alloc, got)
        ctx.forward_static(q, k, v, alloc, got2)         # steady state: same context again, kernels only
        torch.cuda.synchronize()
        if rnd > 0:    # (the very first call of the process may load code objects)
            assert torch.cuda.mem_get_info()[0] == free_before, "device memory in use changed across static calls"
        assert torch.equal(got, want), f"call {rnd}"
        assert torch.equal(got2, want), f"call {rnd} repeated"
    # another allocation on the same context: new work lists inside the same array
    ctx, (q, k, v), _, _ = big
    ref = B.Context(1, 4, 64, (16, 16, 32), B.BF16, B.make_cfg(**band))
    want2 = torch.empty_like(q); got = torch.empty_like(q)
    ref.forward(q, k, v, (4, 4, 0, 3), want2)
    ctx.forward_static(q, k, v, (4, 4, 0, 3), got)
    torch.cuda.synchronize()
    assert torch.equal(got, want2)


def test_forward_static_refuses_shapes_beyond_the_array():
    import torch
    wl = WL.WORKLOADS["64k"]                                   # 24 heads x 65,536 tokens: far more than 128 MiB of scratch
    ctx = B.Context(1, wl.heads, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**wl.band), path=B.PATH_TABLES_ONLY)
    q = torch.zeros((1, wl.heads, wl.n_tokens, wl.head_dim), dtype=torch.bfloat16, device="cuda")
    out = torch.empty_like(q)
    with pytest.raises(B.FreqAttnError) as e:
        ctx.forward_static(q, q, q, [1] * wl.heads, out)
    assert e.value.status == B.ENOMEM and "static array holds" in str(e.value)
    # the array stays usable for a shape that fits
    band = dict(WL.WORKLOADS["tiny_f32"].band)
    small = B.Context(1, 2, 64, (4, 8, 8), B.F32, B.make_cfg(**band), path=B.PATH_TABLES_ONLY)
    ref = B.Context(1, 2, 64, (4, 8, 8), B.F32, B.make_cfg(**band))
    x = torch.randn((1, 2, 256, 64), device="cuda")
    a = torch.empty_like(x); b = torch.empty_like(x)
    small.forward_static(x, x, x.clone(), (1, 4), a)
    ref.forward(x, x, x.clone(), (1, 4), b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_forward_static_on_a_four_band_context():
    """A context with a second block-sparse band (four bands) through the static entry point: its second block list and
    the wider summary layout are carved out of the array too."""
    import torch
    band = dict(WL.WORKLOADS["16k"].band)
    band.update(mid_block=64, mid_stride=3, high_window=100, n_summary=6, mid2_num=3, mid2_den=4)
    alloc = (8, 9, 15, 6)
    ctx, (q, k, v), want, path = _case((16, 16, 32), 4, 64, B.BF16, band, alloc, 33)
    assert path == B.PATH_MFMA and len(ctx.band_sizes()) == 4
    got = torch.full_like(q, float("nan"))
    ctx.forward_static(q, k, v, alloc, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
