"""Helpers shared by the GPU parity tests (not a test module)."""
import numpy as np

from oracle import freqformer as O
from paper_2604_22808_amd import binding as B
from paper_2604_22808_amd import workloads as WL


def to_device(x64, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x64))
    return t.to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda().contiguous()


def to_host64(t):
    import torch
    return t.detach().to(torch.float64).cpu().numpy()


def oracle_cfg(band: dict) -> O.BandConfig:
    return O.BandConfig(**band)


def errors(got, want):
    """max-abs error and relative L2 error (paper-independent metrics named by the benchmark's tolerance)."""
    diff = np.asarray(got, dtype=np.float64) - np.asarray(want, dtype=np.float64)
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(want), 1e-300))


def make_ctx(wl: WL.Workload, path=B.PATH_AUTO, heads=None, **band_override):
    band = dict(wl.band)
    band.update(band_override)
    nh = wl.heads if heads is None else heads
    ctx = B.Context(wl.batch, nh, wl.head_dim, wl.grid, B.BF16 if wl.dtype == "bf16" else B.F32, B.make_cfg(**band),
                    path=path)
    return ctx, band


def run_forward(ctx, q64, k64, v64, dtype, alloc):
    import torch
    q, k, v = (to_device(x, dtype) for x in (q64, k64, v64))
    out = torch.empty_like(q)
    ctx.forward(q, k, v, alloc, out)
    torch.cuda.synchronize()
    return to_host64(out)


TOL = {"bf16": (2e-2, 5e-3), "f32": (1e-5, 1e-5)}   # (max-abs, relative L2) per I/O type


class HeadsOnDemand:
    """A [batch, heads, N, d] device tensor that hands the oracle one (batch, head) slice at a time as fp64 host data,
    so that a 24-head, million-token configuration never sits on the host in fp64 as a whole."""

    def __init__(self, t):
        self._t = t
        self.shape = tuple(t.shape)

    def __getitem__(self, bh):
        b, h = bh
        return to_host64(self._t[b, h])


def band_statistics_library_transform(q, k, v, grid, band: dict):
    """Router statistics (paper section 3.5, same reading as the oracle's band_statistics) with the transform taken by
    scipy's orthonormal DCT-II - the routine the oracle's transform is pinned against - because the oracle's plain
    matrix products need minutes for 48 to 72 head-tensors of 256K to 1M tokens.  The 64K test checks that the two
    agree to 1e-9 on a whole 24-head configuration; everything after the statistics is the oracle's own code."""
    from scipy.fft import dctn
    T, H, W = grid
    Bsz, nh, N, d = q.shape
    bands = O.band_partition(T, H, W, oracle_cfg(band))
    acc = np.zeros((3, d))
    for x in (q, k, v):
        for b in range(Bsz):
            for h in range(nh):
                c = dctn(np.asarray(x[b, h], dtype=np.float64).reshape(T, H, W, d), type=2, norm="ortho",
                         axes=(0, 1, 2), workers=16).reshape(N, d)
                for l, idx in enumerate(bands):
                    acc[l] += np.einsum("nc,nc->c", c[idx], c[idx]) if len(idx) else 0.0
    g = np.empty((3, O.ROUTER_DR))
    for l, idx in enumerate(bands):
        g[l] = (acc[l] / max(1, 3 * Bsz * nh * len(idx))).reshape(O.ROUTER_DR, d // O.ROUTER_DR).mean(axis=1)
    logs = np.log(O.ROUTER_EPS + g).reshape(-1)
    return logs - logs.mean()


def expected_route(stats, t, weights, heads):
    """Oracle allocation from given statistics: probabilities, integer head counts, one-hot masks."""
    pi = O.router_probabilities(stats, t, *weights)
    counts = O.apportion_heads(pi, heads)
    return O.route_fixed(heads, *[int(c) for c in counts]), pi
