"""Speed sweep over the ablation dimensions the paper lists (its section on ablation dimensions): transform choice,
low-band compression ratio, mid-band sparse degree, high-band window, number of summary tokens, number of bands.  Quality columns stay
empty - there is no trained model here - so this prints time per forward only.

    python -m paper_2604_22808_amd.sweep [--workload 256k] [--steps 5]

One parameter is varied at a time around the workload's own configuration; the head allocation is the workload's
(router in the loop where the workload says so); the band-count rows give every head one band, heads split evenly
over the bands that exist.  Prints one markdown table row per configuration.
"""
from __future__ import annotations

import argparse
import dataclasses
import time


def time_forward(wl, band, steps, warmup=2, alloc=None):
    import torch
    from . import binding as B
    from . import workloads as WL
    q, k, v = time_forward.inputs
    out = time_forward.out
    ctx = B.Context(wl.batch, wl.heads, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**band))
    if alloc is not None:
        step = lambda: ctx.forward(q, k, v, alloc, out)
    elif wl.alloc["kind"] == "mlp":
        w = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
        step = lambda: ctx.forward_routed(q, k, v, wl.alloc["t"], *w, out)
    else:
        alloc = B.route_fixed(wl.heads, *wl.alloc["counts"])
        step = lambda: ctx.forward(q, k, v, alloc, out)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / steps
    rp, ci = ctx.mid_blocks()
    n_mid = ctx.band_sizes()[1]
    keys_mid = len(ci) * band["mid_block"] ** 2 / max(n_mid, 1)
    del ctx
    return ms, keys_mid


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="256k")
    ap.add_argument("--steps", type=int, default=5)
    args = ap.parse_args()
    import torch
    from . import binding as B
    from . import workloads as WL
    B.lib()
    wl = WL.WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    time_forward.inputs = WL.qkv_torch(wl, "cuda")
    time_forward.out = torch.empty_like(time_forward.inputs[0])
    base = dict(wl.band)
    rows = [("workload's configuration", {})]
    rows += [("transform = Haar", {"transform": B.TRANSFORM_HAAR})]
    rows += [(f"low compression c = {c}", {"low_compress": c}) for c in (2, 4, 8)]
    rows += [(f"mid stride = {s} (sparser for larger)", {"mid_stride": s}) for s in (base["mid_stride"] // 2, base["mid_stride"] * 2)]
    rows += [(f"mid diagonal = +-{dg}", {"mid_diag": dg}) for dg in (1, 4)]
    rows += [(f"high window w_h = {w}", {"high_window": w}) for w in (32, 64, 128, 256, 1024)]
    rows += [(f"summary tokens m = {m}", {"n_summary": m}) for m in (0, 4, 8, 16)]
    def one_band_per_head(bits):
        return [bits[h * len(bits) // wl.heads] for h in range(wl.heads)]
    rows += [("L = 2: low + windowed rest, one band per head", {"mid_num": base["low_num"], "mid_den": base["low_den"], "_alloc": one_band_per_head([1, 4])}),
             ("L = 2: low + block-sparse rest, one band per head", {"mid_num": 1, "mid_den": 1, "_alloc": one_band_per_head([1, 2])}),
             ("L = 3, one band per head", {"_alloc": one_band_per_head([1, 2, 4])}),
             ("L = 4: second block-sparse band up to 3/4 of every axis, one band per head", {"mid2_num": 3, "mid2_den": 4, "_alloc": one_band_per_head([1, 2, 8, 4])})]
    print(f"| configuration ({wl.name}: {wl.n_tokens} tokens, {wl.heads} heads, head_dim {wl.head_dim}) | mid keys per query | ms per forward | tokens/s |")
    print("|---|---|---|---|")
    for name, change in rows:
        change = dict(change)
        alloc = change.pop("_alloc", None)
        band = dict(base, **change)
        ms, keys_mid = time_forward(wl, band, args.steps, alloc=alloc)
        print(f"| {name} | {keys_mid:.0f} | {ms:.3f} | {wl.batch * wl.n_tokens / (ms * 1e-3):.3e} |", flush=True)


if __name__ == "__main__":
    main()
