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
