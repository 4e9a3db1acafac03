#!/usr/bin/env python3
"""Benchmark of the freqattn hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic Q/K/V already resident in HBM: head
allocation (router MLP in the loop for the MLP workloads), forward transforms, band split, the three band
operators, summary exchange, inverse transform.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1m|256k|64k|16k] [--dense] [--separate]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0   # dense fp16/bf16 matrix-core peak


def measured_traffic(workload: str, stage: str):
    """HBM bytes per launch of a stage's kernels from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (scaled by the
    plain-copy calibration), read from the figures file written next to the counter summary of that workload
    (profiles/hbm_traffic_bench_<workload>.txt: `key: value` lines, among them `<stage>_bytes_per_step`,
    `<stage>_launches` and the commit the counters were taken at).  None where no counter run exists."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_bench_{workload}.txt")
    if not os.path.exists(path):
        return None, None
    vals = {}
    for line in open(path):
        if ":" in line and not line.startswith("#"):
            key, val = line.split(":", 1)
            vals[key.strip()] = val.strip()
    try:
        return float(vals[f"{stage}_bytes_per_step"]) / float(vals[f"{stage}_launches"]), vals.get("commit")
    except (KeyError, ValueError, ZeroDivisionError):
        return None, vals.get("commit")


def algorithmic_work(wl, ctx, alloc):
    """Algorithmic bytes / flops per stage of one forward (what the method itself must move or multiply)."""
    N, d, S = wl.n_tokens, wl.head_dim, wl.batch * wl.heads
    n_low, n_mid, n_high = ctx.band_sizes()
    band = wl.band
    c = band["low_compress"]
    nbar = -(-n_low // c)
    rp, ci = ctx.mid_blocks()
    B = band["mid_block"]
    nb = len(rp) - 1
    size = lambda J: min(B, n_mid - J * B)
    mid_pairs = sum(size(I) * size(int(J)) for I in range(nb) for J in ci[rp[I]:rp[I + 1]])
    w = band["high_window"]
    high_pairs = n_high * (2 * w + 1) - w * (w + 1) if n_high > 2 * w else n_high * n_high
    pairs = [nbar * nbar, mid_pairs, high_pairs]
    m = band["n_summary"]
    m_eff = [min(m, n) for n in (n_low, n_mid, n_high)]
    n_c = [sum(m_eff) - m_eff[l] for l in range(3)]
    attn_flops = [0.0, 0.0, 0.0]
    xchg_flops = 0.0
    for b in range(wl.batch):
        for h in range(wl.heads):
            for l, n in enumerate((n_low, n_mid, n_high)):
                if (int(alloc[h]) >> l) & 1:
                    attn_flops[l] += 4.0 * d * pairs[l]
                    xchg_flops += 4.0 * d * n * n_c[l]
    io = 2  # bytes per bf16 element
    # What the pruned scheme strictly needs for the forward transforms: every input element read once, and only the
    # coefficients somebody uses written (Q~, K~ on the box of the bands a head runs; V~ on the low+mid box for heads
    # without the high band when the context sums their high-band summaries from V, else everywhere).
    box = {0: n_low, 1: n_low + n_mid, 2: N}
    fwd_min = 0.0
    for h in range(wl.heads):
        mk = int(alloc[h])
        top = 2 if mk & 4 else (1 if mk & 2 else (0 if mk & 1 else -1))
        qk_rows = box[top] if top >= 0 else 0
        v_rows = N if (top == 2 or not ctx.get_v_box()) else box[1]
        fwd_min += wl.batch * d * io * (3 * N + 2 * qk_rows + v_rows)
    work_min = {"forward_transform": fwd_min}
    return work_min, {
        "forward_transform": ("hbm", 3 * S * N * d * io * 2.0, 9),     # 3 tensors, one read + one write each; 9 launches
        "inverse_transform": ("hbm", S * N * d * io * 2.0, 3),
        "band_attention_fused": ("mfma", sum(attn_flops), 1),
        "low_attention": ("mfma", attn_flops[0], 1),
        "mid_attention": ("mfma", attn_flops[1], 1),
        "high_attention": ("mfma", attn_flops[2], 1),
        "exchange": ("mfma", xchg_flops, 1),
        "summaries": ("hbm", S * N * d * io * 1.0, 1),
        "dense_attention": ("mfma", 4.0 * d * float(N) * N * S, 1),
    }


def cpu_baseline(wl, alloc, q, k, v):
    """Times the fp64 oracle on the host cores on a bounded sample of the workload itself: one whole head (the
    workload's own token grid, head_dim and band parameters, the benchmark's own input tensors) per distinct band mask of
    the allocation.  The whole-forward figure charges every head of the allocation the seconds measured for its mask."""
    from oracle import freqformer as O
    T, H, W = wl.grid
    cfg = O.BandConfig(**wl.band)
    masks = [int(a) for a in alloc]
    per_mask, sampled = {}, []
    for h, mk in enumerate(masks):
        if mk in per_mask:
            continue
        x = [t[0, h].to("cpu").double().numpy().reshape(T, H, W, wl.head_dim) for t in (q, k, v)]
        t0 = time.perf_counter()
        O.head_forward(x[0], x[1], x[2], cfg, mk)
        per_mask[mk] = time.perf_counter() - t0
        sampled.append(h)
    total_s = sum(per_mask[mk] for mk in masks) * wl.batch
    cores = len(os.sched_getaffinity(0))
    return {"value": wl.batch * wl.n_tokens / total_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "measured_s": {str(mk): round(sec, 2) for mk, sec in per_mask.items()},
            "sample": f"fp64 numpy oracle, heads {sampled} of the benchmark's own tensors (one whole head per distinct band "
                      f"mask {sorted(per_mask)}, full {T}x{H}x{W} grid, {sum(per_mask.values()):.1f} s of CPU work); the "
                      f"forward's time is extrapolated over the {wl.heads} heads, each charged its mask's measured seconds "
                      f"({total_s:.1f} s)"}


def dense_comparison_256k(steps=3):
    """The path against plain dense attention on the same tensors at 256K tokens (the 256k workload, router at its
    t): both through the library's own kernels, in this run."""
    import torch
    from paper_2604_22808_amd import binding as B
    from paper_2604_22808_amd import workloads as WL
    wl = WL.WORKLOADS["256k"]
    q, k, v = WL.qkv_torch(wl, "cuda")
    out = torch.empty_like(q)
    ctx = B.Context(wl.batch, wl.heads, wl.head_dim, wl.grid, B.BF16, B.make_cfg(**wl.band))
    router = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
    for _ in range(3):
        alloc, _ = ctx.forward_routed(q, k, v, wl.alloc["t"], *router, out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ctx.forward_routed(q, k, v, wl.alloc["t"], *router, out)
    torch.cuda.synchronize()
    path_ms = 1e3 * (time.perf_counter() - t0) / steps
    ctx.dense_forward(q, k, v, out)          # warm-up: clocks under matrix load
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.dense_forward(q, k, v, out)
    torch.cuda.synchronize()
    dense_ms = 1e3 * (time.perf_counter() - t0)
    flops = 4.0 * wl.head_dim * float(wl.n_tokens) ** 2 * wl.batch * wl.heads
    ctx.destroy()
    return {"workload": "256k", "tokens": wl.n_tokens, "heads": wl.heads, "head_dim": wl.head_dim,
            "head_alloc_counts": [int((alloc == m).sum()) for m in (1, 2, 4)],
            "freqattn_ms": round(path_ms, 3), "dense_ms": round(dense_ms, 2),
            "dense_achieved_TFLOPs": round(flops / (dense_ms * 1e-3) / 1e12, 1),
            "speedup_of_freqattn": round(dense_ms / path_ms, 1)}


def projected_comparison(wl, alloc, steps=3):
    """The layer around the path (sections 3.1, 3.7) at the workload's shape, two ways, same tensors, same run:
    unfolded - Q, K, V projected in token space (torch.matmul, i.e. the vendor GEMM a model would call), the q/k/v path,
    output projection; folded - freqattn_forward_projected (X transformed once, projections on spectral rows)."""
    import torch
    from paper_2604_22808_amd import binding as B
    from paper_2604_22808_amd import workloads as WL
    N, heads, d = wl.n_tokens, wl.heads, wl.head_dim
    dm = heads * d
    gen = torch.Generator(device="cuda").manual_seed(11)
    q, _, _ = WL.qkv_torch(wl, "cuda")                         # [1, heads, N, d]: used as X's channel groups
    x = q.permute(0, 2, 1, 3).reshape(wl.batch, N, dm).contiguous()
    del q
    w = [(torch.randn((dm, dm), device="cuda", generator=gen) / dm ** 0.5).to(torch.bfloat16) for _ in range(4)]
    ctx = B.Context(wl.batch, heads, d, wl.grid, B.BF16, B.make_cfg(**wl.band))
    out = torch.empty_like(x)

    def folded():
        ctx.forward_projected(x, w[0], w[1], w[2], w[3], alloc, out)

    def timed(fn):
        fn(); fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / steps

    folded_ms = timed(folded)
    ctx.set_stage_timing(True)
    for _ in range(steps):
        folded()
    torch.cuda.synchronize()
    stages = {name: round(ms, 3) for name, ms in ctx.stage_times()}
    ctx.set_stage_timing(False)
    y = torch.empty((wl.batch, heads, N, d), device="cuda", dtype=torch.bfloat16)

    def heads_of(t):
        return t.reshape(wl.batch, N, heads, d).permute(0, 2, 1, 3).contiguous()

    parts = {}

    def unfolded():
        t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
        t2 = torch.cuda.Event(enable_timing=True); t3 = torch.cuda.Event(enable_timing=True)
        t0.record()
        qh, kh, vh = (heads_of(x @ w[i]) for i in range(3))
        t1.record()
        ctx.forward(qh, kh, vh, alloc, y)
        t2.record()
        torch.matmul(y.permute(0, 2, 1, 3).reshape(wl.batch, N, dm), w[3], out=out)
        t3.record()
        parts["ev"] = (t0, t1, t2, t3)

    unfolded_ms = timed(unfolded)
    torch.cuda.synchronize()
    t0, t1, t2, t3 = parts["ev"]
    res = {"workload": wl.name, "d_model": dm, "head_alloc": [int(a) for a in alloc],
           "folded_ms": round(folded_ms, 3), "folded_stages_ms": stages,
           "unfolded_ms": round(unfolded_ms, 3),
           "unfolded_stages_ms": {"qkv_projection_and_head_split (torch)": round(t0.elapsed_time(t1), 3),
                                  "freqattn_forward": round(t1.elapsed_time(t2), 3),
                                  "head_merge_and_o_projection (torch)": round(t2.elapsed_time(t3), 3)},
           "speedup_of_folding": round(unfolded_ms / folded_ms, 3)}
    ctx.destroy()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="1m")
    ap.add_argument("--dense", action="store_true", help="also time the dense flash-style baseline (one iteration)")
    ap.add_argument("--separate", action="store_true", help="one launch per branch instead of the fused launch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense-256k", action="store_true", help="skip the dense comparison at 256K tokens")
    ap.add_argument("--no-projected", action="store_true", help="skip the folded-projection comparison")
    ap.add_argument("--separate-exchange", action="store_true",
                    help="cross-band exchange as a launch of its own for every slice (A/B of the in-item exchange)")
    ap.add_argument("--t", type=float, default=None, help="timestep for the MLP head allocator (default: the workload's)")
    ap.add_argument("--transform", choices=("dct", "haar"), default="dct",
                    help="per-axis transform: the reference design's DCT-II or the Haar wavelet variant")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of q (known bytes) so that a counter run can be scaled by it")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (every (batch, head) is independent, so the path would shard "
                 "by heads without any exchange); run with --gpus 1")

    import numpy as np
    import torch
    from paper_2604_22808_amd import binding as B
    from paper_2604_22808_amd import workloads as WL

    B.lib()  # fails loudly when the HIP library has not been built
    wl = WL.WORKLOADS[args.workload]
    assert wl.dtype == "bf16", "the benchmark runs the bf16 workloads"
    torch.cuda.set_device(0)
    q, k, v = WL.qkv_torch(wl, "cuda")
    out = torch.empty_like(q)
    import dataclasses
    if args.transform == "haar":
        wl = dataclasses.replace(wl, band=dict(wl.band, transform=B.TRANSFORM_HAAR))
    if args.t is not None and wl.alloc["kind"] == "mlp":
        wl = dataclasses.replace(wl, alloc=dict(wl.alloc, t=args.t))
    cfg = B.make_cfg(**wl.band)
    ctx = B.Context(wl.batch, wl.heads, wl.head_dim, wl.grid, B.BF16, cfg)
    if args.separate:
        ctx.set_launch_mode(B.LAUNCH_SEPARATE)
    if args.separate_exchange:
        ctx.set_exchange_fusion(False)
    router = None
    if wl.alloc["kind"] == "mlp":
        router = WL.router_weights(wl.alloc["hidden"], wl.alloc["seed"])
        t_step = wl.alloc["t"]
        alloc, pi, _ = ctx.route_mlp(q, k, v, t_step, *router)
    else:
        alloc = B.route_fixed(wl.heads, *wl.alloc["counts"])
        pi = None

    def step():
        if router is not None:
            ctx.forward_routed(q, k, v, t_step, *router, out)
        else:
            ctx.forward(q, k, v, alloc, out)

    if args.calibrate_copy:
        out.copy_(q)          # plain copy kernel: reads and writes q.numel() * 2 bytes
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.set_stage_timing(True)       # HIP events on the launch stream around every stage of every timed step
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stages = ctx.stage_times()
    ctx.set_stage_timing(False)

    ms_per_step = 1e3 * elapsed / args.steps
    tokens = wl.batch * wl.n_tokens
    value = tokens / (elapsed / args.steps)

    # the same loop with the allocation prediction off: every forward transforms on the low+mid box first and completes
    # the heads routed to the high band afterwards (what a call pays whose previous allocation is no guide)
    ms_no_prediction = None
    if router is not None:
        ctx.set_alloc_prediction(False)
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms_no_prediction = 1e3 * (time.perf_counter() - t0) / args.steps
        ctx.set_alloc_prediction(True)

    # the plain forward with this allocation (no router, no host round trip), eagerly and replayed from a HIP graph
    ms_fixed = ms_graph = None
    try:
        ctx.set_stage_timing(False)
        for _ in range(2):
            ctx.forward(q, k, v, alloc, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ctx.forward(q, k, v, alloc, out)
        torch.cuda.synchronize()
        ms_fixed = 1e3 * (time.perf_counter() - t0) / args.steps
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ctx.forward(q, k, v, alloc, out)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = 1e3 * (time.perf_counter() - t0) / args.steps
        del graph
    except RuntimeError as e:      # capture is a convenience of the caller's runtime, not part of the measured path
        sys.stderr.write(f"bench.py: graph replay skipped: {e}\n")

    work_min, work = algorithmic_work(wl, ctx, alloc)
    # the forward transform may be split in two stages (completion of Q~/K~ for the heads routed to the high band)
    merged, extra = [], 0.0
    for name, ms in stages:
        if name == "forward_transform_high_qk":
            extra += ms
        else:
            merged.append([name, ms])
    for e in merged:
        if e[0] == "forward_transform":
            e[1] += extra
    stages = [tuple(e) for e in merged]
    masks = [int(a) for a in alloc]
    cls_present = [any((m & 4) == 0 and (m & 2) == 0 and (m & 1) for m in masks), any((m & 4) == 0 and (m & 2) for m in masks),
                   any(m & 4 for m in masks)]
    vbox = ctx.get_v_box()   # V~ of a slice without the high band on the low+mid box: V follows Q and K class by class
    nonhigh_present = cls_present[0] or cls_present[1] or any(m == 0 for m in masks)
    if router is not None:   # routed: slices split into "ran the high band last time" and the rest
        fwd_launches = (9 if nonhigh_present else 0) + ((9 if vbox else 6) if cls_present[2] else 0) + (0 if vbox else 3)
    elif vbox:
        fwd_launches = 6 * sum(cls_present) + (3 if nonhigh_present else 0) + (3 if cls_present[2] else 0)
    else:
        fwd_launches = 3 + 6 * sum(cls_present)
    inv_launches = 3 * sum(cls_present) + (1 if any(m == 0 for m in masks) else 0)
    # single-band slices run their exchange inside the band items: its flops then belong to the band attention launch
    one_band = [m in (1, 2, 4) for m in masks]
    if any(one_band):
        n_l = ctx.band_sizes()
        m_eff = [min(wl.band["n_summary"], n) for n in n_l]
        moved_band = [0.0, 0.0, 0.0]
        for m, ob in zip(masks, one_band):
            if ob:
                l = m.bit_length() - 1
                moved_band[l] += 4.0 * wl.head_dim * n_l[l] * (sum(m_eff) - m_eff[l]) * wl.batch
        moved = sum(moved_band) if not args.separate_exchange else 0.0
        if moved:
            work["band_attention_fused"] = ("mfma", work["band_attention_fused"][1] + moved, 1)
            for l, name in enumerate(("low_attention", "mid_attention", "high_attention")):
                work[name] = ("mfma", work[name][1] + moved_band[l], 1)
            work["exchange"] = ("mfma", max(work["exchange"][1] - moved, 0.0), 1)
    work["forward_transform"] = (work["forward_transform"][0], work["forward_transform"][1], fwd_launches)
    work["inverse_transform"] = (work["inverse_transform"][0], work["inverse_transform"][1], max(1, inv_launches))
    stage_report = {}
    for name, ms in stages:
        entry = {"ms": round(ms, 4)}
        if name in work and ms > 0 and work[name][1] > 0:   # (a stage with nothing left to do carries only its time)
            bound, amount, launches = work[name]
            if bound == "hbm":
                entry.update(bound="hbm", achieved_GBs=round(amount / (ms * 1e-3) / 1e9, 1), launches=launches)
            else:
                entry.update(bound="mfma", achieved_TFLOPs=round(amount / (ms * 1e-3) / 1e12, 2), launches=launches)
        stage_report[name] = entry
    dom = max((s for s in stages if s[0] in work), key=lambda s: s[1])
    bound, amount, launches = work[dom[0]]
    per_launch_s = dom[1] * 1e-3 / launches
    if bound == "hbm":
        achieved, peak, unit = amount / launches / per_launch_s / 1e9, HBM_PEAK_GBS, "GB/s"
    else:
        achieved, peak, unit = amount / launches / per_launch_s / 1e12, MFMA_PEAK_TFLOPS, "TFLOP/s"
    traffic, traffic_commit = measured_traffic(wl.name, dom[0]) if args.transform == "dct" and args.t is None else (None, None)
    # what this machine sustains for a plain streaming copy and for a loop of the MFMA instruction the kernels use
    copy_bps, mfma_fps = ctx.measure_peaks()
    measured = copy_bps / 1e9 if bound == "hbm" else mfma_fps / 1e12
    roofline = {"bound": bound, "kernel": dom[0], "launches_per_step": launches,
                "avg_launch_ms": round(per_launch_s * 1e3, 4), "achieved": round(achieved, 2), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic, "traffic_measured_at_commit": traffic_commit,
                "measured_peak": round(measured, 1), "frac_of_measured": round(achieved / measured, 4)}
    if traffic and bound == "hbm":   # what the stage's kernels really move (counter bytes of the committed profile) per second
        roofline["hbm_rate_at_measured_traffic"] = round(traffic / per_launch_s / 1e9, 1)
        roofline["frac_at_measured_traffic"] = round(traffic / per_launch_s / 1e9 / peak, 4)
    if dom[0] in work_min:   # the same stage against the bytes the pruned scheme strictly needs
        ach_min = work_min[dom[0]] / (dom[1] * 1e-3) / 1e9
        roofline["achieved_pruned_minimum"] = round(ach_min, 2)
        roofline["frac_pruned_minimum"] = round(ach_min / peak, 4)
        roofline["algorithmic_bytes_per_step"] = amount
        roofline["pruned_minimum_bytes_per_step"] = work_min[dom[0]]

    result = {
        "metric": "tokens/s per forward", "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_no_prediction": None if ms_no_prediction is None else round(ms_no_prediction, 4),
        "ms_per_step_given_allocation": None if ms_fixed is None else round(ms_fixed, 4),
        "ms_per_step_given_allocation_hip_graph": None if ms_graph is None else round(ms_graph, 4),
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "heads": wl.heads, "head_dim": wl.head_dim,
                   "grid": list(wl.grid), "tokens": wl.n_tokens, "band": wl.band, "alloc": wl.alloc,
                   "head_alloc": [int(a) for a in alloc], "pi": None if pi is None else [round(float(p), 4) for p in pi],
                   "launch": "separate" if args.separate else "fused",
                   "alloc_prediction": "previous forward's high heads (exact in this constant-t loop)" if router is not None else None,
                   "v_on_low_mid_box": bool(vbox),
                   "precision": "bf16 tensors in and out, fp16 MFMA operands and intermediates, fp32 accumulation"},
        "roofline": roofline, "stages": stage_report,
        "measured_peaks": {"copy_GBs": round(copy_bps / 1e9, 1), "mfma_f16_TFLOPs": round(mfma_fps / 1e12, 1)},
    }
    if args.dense:
        dout = torch.empty_like(q)
        ctx.set_stage_timing(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.dense_forward(q, k, v, dout)
        torch.cuda.synchronize()
        dense_s = time.perf_counter() - t0
        ctx.set_stage_timing(False)
        dflops = work["dense_attention"][1]
        result["dense_baseline"] = {"ms": round(dense_s * 1e3, 3), "tokens_per_s": round(tokens / dense_s, 1),
                                    "achieved_TFLOPs": round(dflops / dense_s / 1e12, 2),
                                    "speedup_of_freqattn": round(dense_s * 1e3 / ms_per_step, 2)}
    ctx.destroy()
    if not args.no_projected:
        del out
        torch.cuda.empty_cache()
        result["projected"] = projected_comparison(wl, alloc)
        out = None
    if not args.no_dense_256k:
        result["dense_256k"] = dense_comparison_256k()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, alloc, q, k, v)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
