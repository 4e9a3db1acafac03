"""Synthetic workloads: the five benchmark configurations and the seeded input generators.

This module is shared *data* plumbing for the tests, the benchmark and the smoke check.  It holds
none of the attention method's arithmetic and imports neither the HIP binding nor the CPU checker:
the random fields are synthesised with a library inverse DCT (scipy on the host, plain torch
matmuls on the device for the large cases).

Recipe (stands in for video-latent Q/K/V with strong low-frequency structure, paper section 1.2):
for every tensor X in {Q, K, V} (stream 0, 1, 2), batch*head index h and channel c,
    C[kt, kh, kw] = g * (1 + sqrt(kt^2 + kh^2 + kw^2))^(-1.5),  g ~ N(0, 1)
    X = IDCT-II-orthonormal(C) + 0.1 * N(0, 1)
so spectral variances are (1 + rho)^-3 + 0.01 <= 1.01 and attention logits stay O(1).
"""
from __future__ import annotations

from dataclasses import dataclass, field
import math

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                 # "f32" or "bf16" (I/O type)
    batch: int
    heads: int
    head_dim: int
    grid: tuple                # (T, H, W)
    band: dict                 # band-operator parameters (keys as in the C struct)
    alloc: dict                # {"kind": "fixed", "counts": (l, m, h)} or {"kind": "mlp", "t": ..., "hidden": 64, "seed": 1}
    seed: int = 0

    @property
    def n_tokens(self) -> int:
        T, H, W = self.grid
        return T * H * W


def _band(block, diag, stride, window, m):
    return dict(low_num=1, low_den=4, mid_num=1, mid_den=2, low_compress=4, mid_block=block, mid_diag=diag,
                mid_stride=stride, mid_block0=1, high_window=window, n_summary=m, softmax_scale=0.0)


WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", "f32", 1, 2, 64, (4, 8, 8), _band(16, 1, 4, 32, 4),
                         {"kind": "masks", "masks": (1, 4)}),
    "16k": Workload("16k", "bf16", 1, 8, 64, (16, 32, 32), _band(64, 1, 8, 256, 16),
                    {"kind": "fixed", "counts": (2, 3, 3)}),
    "64k": Workload("64k", "bf16", 1, 24, 64, (16, 64, 64), _band(64, 1, 8, 256, 16),
                    {"kind": "mlp", "t": 0.9, "hidden": 64, "seed": 1}),
    "256k": Workload("256k", "bf16", 1, 24, 128, (64, 64, 64), _band(128, 2, 16, 512, 32),
                     {"kind": "mlp", "t": 0.9, "hidden": 64, "seed": 1}),
    "1m": Workload("1m", "bf16", 1, 16, 128, (64, 128, 128), _band(128, 2, 32, 512, 64),
                   {"kind": "mlp", "t": 0.5, "hidden": 64, "seed": 1}),
}


def amplitude(T: int, H: int, W: int) -> np.ndarray:
    kt = np.arange(T, dtype=np.float64)[:, None, None]
    kh = np.arange(H, dtype=np.float64)[None, :, None]
    kw = np.arange(W, dtype=np.float64)[None, None, :]
    return (1.0 + np.sqrt(kt * kt + kh * kh + kw * kw)) ** -1.5


def field_numpy(grid, d: int, seed: int, stream: int, index: int) -> np.ndarray:
    """One head-tensor [N, d] in fp64, generator numpy.random.default_rng([seed, stream, index])."""
    from scipy.fft import idctn
    T, H, W = grid
    rng = np.random.default_rng([seed, stream, index])
    coef = rng.standard_normal((T, H, W, d)) * amplitude(T, H, W)[..., None]
    x = idctn(coef, type=2, norm="ortho", axes=(0, 1, 2))
    x += 0.1 * rng.standard_normal((T, H, W, d))
    return x.reshape(T * H * W, d)


def qkv_numpy(wl: Workload, heads=None):
    """q, k, v as fp64 arrays [batch, heads, N, d] (host recipe).  `heads` restricts to a list of heads
    (the returned arrays then have len(heads) heads, generated with the original head indices)."""
    hs = list(range(wl.heads)) if heads is None else list(heads)
    out = []
    for stream in range(3):
        x = np.empty((wl.batch, len(hs), wl.n_tokens, wl.head_dim), dtype=np.float64)
        for b in range(wl.batch):
            for i, h in enumerate(hs):
                x[b, i] = field_numpy(wl.grid, wl.head_dim, wl.seed, stream, b * wl.heads + h)
        out.append(x)
    return out


def _idct_matrix_torch(n: int, device, dtype):
    """Columns are the orthonormal DCT-II basis vectors: x = M @ c synthesises a signal from coefficients c."""
    import torch
    j = torch.arange(n, device=device, dtype=torch.float64)[:, None]
    k = torch.arange(n, device=device, dtype=torch.float64)[None, :]
    M = math.sqrt(2.0 / n) * torch.cos(math.pi * (2.0 * j + 1.0) * k / (2.0 * n))
    M[:, 0] *= 1.0 / math.sqrt(2.0)
    return M.to(dtype)


def qkv_torch(wl: Workload, device="cuda", out_dtype=None):
    """Device variant of the recipe for the large workloads (same distribution, torch's generator, seeded
    per tensor and head): returns q, k, v as torch tensors [batch, heads, N, d] of the workload's I/O type."""
    import torch
    T, H, W = wl.grid
    d = wl.head_dim
    if out_dtype is None:
        out_dtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    amp = torch.from_numpy(amplitude(T, H, W)).to(device=device, dtype=torch.float32)[..., None]
    Mt, Mh, Mw = (_idct_matrix_torch(n, device, torch.float32) for n in (T, H, W))
    gen = torch.Generator(device=device)
    out = []
    for stream in range(3):
        x = torch.empty((wl.batch, wl.heads, T * H * W, d), device=device, dtype=out_dtype)
        for b in range(wl.batch):
            for h in range(wl.heads):
                gen.manual_seed((wl.seed * 3 + stream) * 1_000_003 + b * wl.heads + h)
                c = torch.randn((T, H, W, d), device=device, dtype=torch.float32, generator=gen) * amp
                c = torch.einsum("ta,ahwc->thwc", Mt, c)
                c = torch.einsum("hb,tbwc->thwc", Mh, c)
                c = torch.einsum("wg,thgc->thwc", Mw, c)
                c += 0.1 * torch.randn((T, H, W, d), device=device, dtype=torch.float32, generator=gen)
                x[b, h] = c.reshape(T * H * W, d).to(out_dtype)
        out.append(x)
    return out


def router_weights(hidden: int = 64, seed: int = 1, d_in: int = 256):
    """Random-initialised router weights (the trained router is not available): W ~ N(0, 1/fan_in), zero
    biases, numpy.random.default_rng(seed).  Returned as float32 so that every consumer sees identical values."""
    rng = np.random.default_rng(seed)
    w1 = (rng.standard_normal((d_in, hidden)) / math.sqrt(d_in)).astype(np.float32)
    w2 = (rng.standard_normal((hidden, 3)) / math.sqrt(hidden)).astype(np.float32)
    return w1, np.zeros(hidden, np.float32), w2, np.zeros(3, np.float32)


def round_to_io(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 host data to the workload's I/O type and widen back to fp64: the stored values both the
    checker and the device path see."""
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x)).to(torch.bfloat16)
    return t.to(torch.float64).numpy()
