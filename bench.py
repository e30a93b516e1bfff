#!/usr/bin/env python3
"""Benchmark of the neighbourhood-attention hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic tokens that are
already resident in HBM: affmae_cluster (curve order and clusters) -> affmae_knn
(neighbour table) -> affmae_pla_plan -> affmae_pla_fwd -> affmae_pla_bwd; exactly
--steps of them are timed by the wall clock (ms_per_step).  The headline value is
attention forward+backward tokens/s (the table is built once per encoder stage and
reused by every block, so the search is reported on its own), taken from loops that
time the forward and the backward call separately, each call starting with cold
caches: between two timed calls a 512 MiB buffer is read through the chip,
outside the timed events.  All phase times are medians.  The other bf16
configurations of the workload list get the same cold loops ("configs").
Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config ft_s1_1024]
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

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def algorithmic_bytes_per_token(C: int, H: int, K: int, elt: int = 2):
    """Compulsory HBM bytes per token, every tensor element touched once
    (bf16 storage: elt = 2; int32 indices; fp32 lse)."""
    row = C * elt
    bias = K * H * elt
    idx = K * 4
    lse = H * 4
    fwd = 3 * row + bias + idx + row + lse                       # q,k,v + bias + idx + out + lse
    bwd = 5 * row + bias + idx + lse + 3 * row + bias            # q,k,v,out,dout + bias + idx + lse + dq,dk,dv + dbias
    return fwd, bwd


def bench_virtual_tokens(aff, torch, np, dev, reps: int = 20):
    """The point decoder's virtual sampled tokens at the shape of the paper's decoder timing (batch 48, 2048 mask
    tokens x 4 sample points, 4 nearest visible tokens; 512px images at 25 % visible, stage-1 width 128, bf16):
    table build, fused lookup + weights + sum forward, backward.  Times are HIP-event medians."""
    rng = np.random.default_rng(2602016249 + 100)
    B, Nv, Mq, C, Hg, Wg, Kt, cell, p, eps = 48, 1024, 8192, 128, 64, 64, 4, 8.0, 0.5, 1e-6
    grid = (Hg, Wg, 0.0, 0.0, cell)
    vis = np.empty((B, Nv, 2), dtype=np.float32)
    for b in range(B):
        keep = np.sort(rng.permutation(Hg * Wg)[:Nv])
        vis[b, :, 0] = (keep % Wg + 0.5) * cell
        vis[b, :, 1] = (keep // Wg + 0.5) * cell
    q = torch.from_numpy(rng.uniform(0, Wg * cell, size=(B, Mq, 2)).astype(np.float32)).to(dev)
    vis = torch.from_numpy(vis).to(dev)
    feat = torch.randn((B, Nv, C), device=dev).bfloat16()
    dout = torch.randn((B, Mq, C), device=dev).bfloat16()
    table = aff.affmae_vts_table(vis, grid, Kt)
    out = aff.affmae_vts_fwd(q, vis, feat, table, grid, p, eps)
    ws = torch.empty(aff.load_library().affmae_vts_bwd_workspace_bytes(B, Mq, Nv, Kt), dtype=torch.uint8, device=dev)
    aff.affmae_vts_bwd(q, vis, feat, table, dout, grid, p, eps, workspace=ws)
    torch.cuda.synchronize()
    ts = [[], [], []]
    for _ in range(reps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        ev[0].record()
        aff.affmae_vts_table(vis, grid, Kt, table=table)
        ev[1].record()
        aff.affmae_vts_fwd(q, vis, feat, table, grid, p, eps, out=out)
        ev[2].record()
        aff.affmae_vts_bwd(q, vis, feat, table, dout, grid, p, eps, workspace=ws)
        ev[3].record()
        torch.cuda.synchronize()
        for i in range(3):
            ts[i].append(ev[i].elapsed_time(ev[i + 1]))
    t = [float(np.median(x)) for x in ts]
    samples = B * Mq
    # algorithmic bytes: every tensor element once (bf16 features; the gathered rows counted once, as stored)
    fwd_bytes = samples * (8 + 4 * Kt + 2 * C) + B * Nv * (8 + 2 * C)
    bwd_bytes = samples * (8 + 4 * Kt + 2 * C + 8) + B * Nv * (8 + 2 * C + 2 * C)
    return {"workload": "point decoder, batch 48 x 2048 mask tokens x 4 sample points, Nv=1024 of 64x64, C=128, Kt=4, bf16",
            "table_ms": t[0], "fwd_ms": t[1], "bwd_ms": t[2],
            "sample_points_per_s_fwd_bwd": samples / ((t[1] + t[2]) * 1e-3),
            "fwd_algorithmic_GBs": fwd_bytes / (t[1] * 1e-3) / 1e9, "bwd_algorithmic_GBs": bwd_bytes / (t[2] * 1e-3) / 1e9}


def bench_merging(aff, torch, np, cfg, s, flush, reps: int = 20):
    """Neighbourhood merging between two stages of the configuration: d_s = 0.25 of the tokens kept as anchors,
    every anchor aggregating its K neighbours (the stage's own table), forward and backward; cold medians."""
    dev = s["q"].device
    B, N, C, K = cfg.B, cfg.N, cfg.C, cfg.K
    n_keep = N // 4
    p = 0.25
    feat = s["q"].reshape(B, N, C)
    score = torch.randn((B, N), device=dev)
    dout = torch.randn((B, n_keep, C), device=dev).to(feat.dtype)
    anchors, axy = aff.affmae_merge_select(score, n_keep, s["coords"])
    out = aff.affmae_merge_fwd(feat, s["coords"], score, s["nbr"], anchors, p)
    ws = torch.empty(aff.load_library().affmae_merge_bwd_workspace_bytes(B, N, K, n_keep), dtype=torch.uint8, device=dev)
    grads = aff.affmae_merge_bwd(feat, s["coords"], score, s["nbr"], anchors, dout, p, want_dp=False, workspace=ws)
    one = [s]
    t_sel = float(np.median(cold_times(torch, lambda _: aff.affmae_merge_select(score, n_keep, s["coords"], anchors, axy), one, reps, flush)))
    t_fwd = float(np.median(cold_times(torch, lambda _: aff.affmae_merge_fwd(feat, s["coords"], score, s["nbr"], anchors, p, out=out), one, reps, flush)))
    t_bwd = float(np.median(cold_times(torch, lambda _: aff.affmae_merge_bwd(feat, s["coords"], score, s["nbr"], anchors, dout, p, want_dp=False, grads=grads, workspace=ws), one, reps, flush)))
    elt = 2 if cfg.dtype == "bf16" else 4
    tokens, anch = B * N, B * n_keep
    # every tensor element once; the gathered feature rows counted once, as stored
    fwd_bytes = anch * (4 * K + elt * C + 4) + tokens * (elt * C + 8 + 4)
    bwd_bytes = anch * (4 * K + elt * C + 4) + tokens * (elt * C + 8 + 4 + elt * C + 4)
    return {"workload": f"{cfg.name}: {B} x {N} tokens -> {n_keep} anchors each (d_s = 0.25), C = {C}, K = {K}, {cfg.dtype}",
            "select_ms": t_sel, "fwd_ms": t_fwd, "bwd_ms": t_bwd,
            "tokens_per_s_fwd_bwd": tokens / ((t_fwd + t_bwd) * 1e-3),
            "fwd_algorithmic_GBs": fwd_bytes / (t_fwd * 1e-3) / 1e9, "bwd_algorithmic_GBs": bwd_bytes / (t_bwd * 1e-3) / 1e9,
            "frac_of_hbm_peak": (fwd_bytes + bwd_bytes) / ((t_fwd + t_bwd) * 1e-3) / 1e9 / HBM_PEAK_GBS}


def bench_relpos(aff, torch, np, cfg, sets, scale, promise, flush, reps: int = 20):
    """The same attention with the bias taken from a relative-position table (9 x 9 bins of one 8-px patch per
    head) instead of a bias tensor: forward and backward through affmae_pla_*_relpos, timed like the headline
    (the same rotating tensor sets, every call on cold caches, medians)."""
    dev = sets[0]["q"].device
    R, rate = 4, 1.0 / 8.0
    table = (0.1 * torch.randn((cfg.H, 2 * R + 1, 2 * R + 1), device=dev)).to(sets[0]["q"].dtype)
    lib = aff.load_library()
    code = 1 if cfg.dtype == "bf16" else 0
    ws = torch.empty(max(lib.affmae_pla_fwd_relpos_workspace_bytes(cfg.B, cfg.N, cfg.H, cfg.d, cfg.K, cfg.S, cfg.M, code, int(promise)),
                         lib.affmae_pla_bwd_relpos_workspace_bytes(cfg.B, cfg.N, cfg.H, cfg.d, cfg.K, cfg.S, cfg.M, R, code, int(promise))),
                     dtype=torch.uint8, device=dev)

    def fwd(s):
        aff.affmae_pla_fwd_relpos(s["q"], s["k"], s["v"], s["coords"], table, s["nbr"], scale, rate,
                                  s["near"] if promise else None, cfg.S, cfg.M, out=s["out"], lse=s["lse"], workspace=ws,
                                  plan=s["plan"])

    def bwd(s):
        aff.affmae_pla_bwd_relpos(s["q"], s["k"], s["v"], s["coords"], table, s["nbr"], s["out"], s["lse"], s["dout"],
                                  scale, rate, s["near"] if promise else None, cfg.S, cfg.M, workspace=ws, plan=s["plan"])

    t_fwd = float(np.median(cold_times(torch, fwd, sets, reps, flush)))
    t_bwd = float(np.median(cold_times(torch, bwd, sets, reps, flush)))
    elt = 2 if cfg.dtype == "bf16" else 4
    fwd_b, bwd_b = algorithmic_bytes_per_token(cfg.C, cfg.H, cfg.K, elt)
    own = fwd_b + bwd_b - 3 * cfg.K * cfg.H * elt + 2 * 8   # no bias / dbias tensor; the coordinates instead
    tokens = cfg.B * cfg.N
    return {"table": f"{cfg.H} x {2 * R + 1} x {2 * R + 1}, bins of 8 px", "tensor_sets": len(sets), "fwd_ms": t_fwd,
            "bwd_ms": t_bwd, "tokens_per_s_fwd_bwd": tokens / ((t_fwd + t_bwd) * 1e-3),
            "algorithmic_bytes_per_token": own,
            "frac_of_hbm_peak": own * tokens / ((t_fwd + t_bwd) * 1e-3) / 1e9 / HBM_PEAK_GBS}


def bench_graphs(torch, sets, step, attn, steps: int):
    """The same work replayed from HIP graphs (one per tensor set, recorded once): the library's calls only
    enqueue kernels, so a caller can remove the launch gaps between the ~20 kernels of a step this way.
    Returns mean milliseconds per replay of the whole step and of attention forward + backward alone."""
    out = {}
    for name, fn in (("step_ms", step), ("attn_fwd_bwd_ms", attn)):
        side = torch.cuda.Stream()
        graphs = []
        for st in sets:
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                fn(st)  # warm-up outside the capture
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                fn(st)
            graphs.append(g)
        for g in graphs:
            g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            graphs[i % len(graphs)].replay()
        e1.record()
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1) / steps
        del graphs
    return out


def alloc_set(cfg, w, torch, dev, tdt):
    """One copy of every tensor of a configuration, resident on the device."""
    def up(x):
        return torch.from_numpy(x).to(dev).to(tdt)
    s = {n: up(w[n]) for n in ("q", "k", "v", "bias", "dout")}
    s["coords"] = torch.from_numpy(w["coords"]).to(dev)
    s["nbr"] = torch.empty((cfg.B, cfg.N, cfg.K), dtype=torch.int32, device=dev)
    s["near"] = torch.empty((cfg.B, cfg.G, cfg.M), dtype=torch.int32, device=dev)
    s["out"] = torch.empty_like(s["q"])
    s["lse"] = torch.empty((cfg.B, cfg.N, cfg.H), dtype=torch.float32, device=dev)
    s["plan"] = None
    s["order"] = torch.empty((cfg.B, cfg.N), dtype=torch.int32, device=dev)
    s["cid"] = torch.empty((cfg.B, cfg.N), dtype=torch.int32, device=dev)
    s["grads"] = {"dq": torch.empty_like(s["q"]), "dk": torch.empty_like(s["q"]), "dv": torch.empty_like(s["q"]),
                  "dbias": torch.empty_like(s["bias"])}
    return s


class Runner:
    """The calls of one configuration on its tensor sets."""

    def __init__(self, aff, torch, cfg, promise):
        self.aff, self.torch, self.cfg, self.promise = aff, torch, cfg, promise
        self.scale = 1.0 / float(cfg.d) ** 0.5
        self.frame = (0.0, 0.0, float(cfg.frame), float(cfg.frame))
        lib = aff.load_library()
        code = 1 if cfg.dtype == "bf16" else 0
        self.ws_bytes = max(lib.affmae_cluster_workspace_bytes(cfg.B, cfg.N),
                            lib.affmae_knn_workspace_bytes(cfg.B, cfg.N, cfg.S, cfg.M, cfg.K),
                            lib.affmae_pla_fwd_workspace_bytes(cfg.B, cfg.N, cfg.H, cfg.d, cfg.K, cfg.S, cfg.M, code, int(promise)),
                            lib.affmae_pla_bwd_workspace_bytes(cfg.B, cfg.N, cfg.H, cfg.d, cfg.K, cfg.S, cfg.M, code, int(promise)),
                            256)

    def tables(self, s):
        aff, cfg = self.aff, self.cfg
        # the generator hands the tokens over in curve order already: the clustering returns the identity
        # (its sorting network does the same work for any input), so nothing has to be gathered here
        aff.affmae_cluster(s["coords"], cfg.S, self.frame, order=s["order"], cluster_id=s["cid"], workspace=s["ws"])
        self.knn(s)

    def knn(self, s):
        aff, cfg = self.aff, self.cfg
        aff.affmae_knn(s["coords"], None, cfg.S, cfg.M, cfg.K, nbr_idx=s["nbr"], near_clusters=s["near"], workspace=s["ws"])
        if self.promise:  # the tiled kernels' view of the table: built once per table, like the table itself
            s["plan"] = aff.affmae_pla_plan(s["nbr"], s["near"], cfg.S, cfg.M, plan=s["plan"])

    def fwd(self, s):
        cfg = self.cfg
        self.aff.affmae_pla_fwd(s["q"], s["k"], s["v"], s["bias"], s["nbr"], self.scale, s["near"] if self.promise else None,
                                cfg.S, cfg.M, out=s["out"], lse=s["lse"], workspace=s["ws"], plan=s["plan"])

    def bwd(self, s):
        cfg = self.cfg
        self.aff.affmae_pla_bwd(s["q"], s["k"], s["v"], s["bias"], s["nbr"], s["out"], s["lse"], s["dout"], self.scale,
                                s["near"] if self.promise else None, cfg.S, cfg.M, grads=s["grads"], workspace=s["ws"],
                                plan=s["plan"])


def cold_times(torch, fn, sets, iters, flush):
    """Milliseconds of `iters` calls of fn, each after the flush buffer has been streamed through the chip
    (outside the timed events), rotating over the tensor sets."""
    ms = []
    for i in range(iters + 2):
        flush.sum()  # read only: a flush that writes would leave dirty lines for the timed call to push out
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn(sets[i % len(sets)])
        e1.record()
        torch.cuda.synchronize()
        if i >= 2:
            ms.append(e0.elapsed_time(e1))
    return ms


def bench_config(aff, torch, np, cfg, dev, flush, iters, promise=True):
    """Cold forward and backward times of one configuration (tables built once, outside the timing)."""
    from workloads import make_workload
    w = make_workload(cfg)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    run = Runner(aff, torch, cfg, promise)
    sets = [alloc_set(cfg, w, torch, dev, tdt) for _ in range(2)]
    for s in sets:
        s["ws"] = torch.empty(run.ws_bytes, dtype=torch.uint8, device=dev)
        run.tables(s)
        run.fwd(s)
    torch.cuda.synchronize()
    knn = float(np.median(cold_times(torch, run.knn, sets, max(iters // 2, 4), flush)))
    fwd = float(np.median(cold_times(torch, run.fwd, sets, iters, flush)))
    bwd = float(np.median(cold_times(torch, run.bwd, sets, iters, flush)))
    tokens = cfg.B * cfg.N
    fwd_b, bwd_b = algorithmic_bytes_per_token(cfg.C, cfg.H, cfg.K, 2 if cfg.dtype == "bf16" else 4)
    gbs = (fwd_b + bwd_b) * tokens / ((fwd + bwd) * 1e-3) / 1e9
    return {"workload": cfg.name, "B": cfg.B, "N": cfg.N, "C": cfg.C, "H": cfg.H, "K": cfg.K, "S": cfg.S, "M": cfg.M,
            "coords": cfg.coords, "fwd_us": 1e3 * fwd, "bwd_us": 1e3 * bwd, "knn_plan_us": 1e3 * knn,
            "tokens_per_s_fwd_bwd": tokens / ((fwd + bwd) * 1e-3), "algorithmic_bytes_per_token": fwd_b + bwd_b,
            "algorithmic_GBs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default="ft_s1_1024")
    ap.add_argument("--sets", type=int, default=4, help="rotating copies of all tensors")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-promise", action="store_true", help="do not pass near_clusters (gather kernels)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the other configurations, the relative-position, graph and point-decoder sections")
    ap.add_argument("--copy-probe", action="store_true", help="accepted for compatibility: the copy probe always runs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the path shards over images with no exchange "
              "(images of a batch are independent), and no multi-GPU figure is produced. Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2602_16249_amd as aff
    from workloads import CONFIGS, make_workload

    cfg = CONFIGS[args.config]
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = make_workload(cfg)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    tokens = cfg.B * cfg.N
    promise = not args.no_promise
    run = Runner(aff, torch, cfg, promise)
    scale = run.scale
    sets = [alloc_set(cfg, w, torch, dev, tdt) for _ in range(args.sets)]
    for s in sets:
        s["ws"] = torch.empty(run.ws_bytes, dtype=torch.uint8, device=dev)
        run.tables(s)  # every set holds its table before anything is measured, however short the warm-up
        run.fwd(s)     # ... and out / lse for the backward-only loops

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(s, rec=None):
        e = [ev() for _ in range(5)] if rec is not None else None
        if e: e[4].record()
        aff.affmae_cluster(s["coords"], cfg.S, run.frame, order=s["order"], cluster_id=s["cid"], workspace=s["ws"])
        if e: e[0].record()
        run.knn(s)
        if e: e[1].record()
        run.fwd(s)
        if e: e[2].record()
        run.bwd(s)
        if e:
            e[3].record()
            rec.append(e)

    def attn_only(s):
        run.fwd(s)
        run.bwd(s)

    for i in range(args.warmup):
        step(sets[i % len(sets)])
    torch.cuda.synchronize()
    # a plain 256 MiB device copy: the practical ceiling of this machine's HBM path (read + written bytes per
    # second), and the dispatch of known size that calibrates FETCH_SIZE / WRITE_SIZE under rocprofv3
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    copy_ms = []
    for _ in range(4):
        c0, c1 = ev(), ev()
        c0.record()
        dst.copy_(src)
        c1.record()
        torch.cuda.synchronize()
        copy_ms.append(c0.elapsed_time(c1))
    copy_gbs = 2 * src.numel() / (min(copy_ms[1:]) * 1e-3) / 1e9
    del src, dst

    # timed region: exactly `steps` steps, phase boundaries marked by events on the launch stream
    rec = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % len(sets)], rec)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    med = lambda xs: float(np.median(xs))
    cluster_ms = med([e[4].elapsed_time(e[0]) for e in rec])
    knn_ms = med([e[0].elapsed_time(e[1]) for e in rec])
    fwd_step_ms = med([e[1].elapsed_time(e[2]) for e in rec])
    bwd_step_ms = med([e[2].elapsed_time(e[3]) for e in rec])

    # the headline: forward and backward timed apart, every call on cold caches
    flush = torch.zeros(128 << 20, dtype=torch.int32, device=dev)  # 512 MiB
    cold_iters = max(args.steps, 20)
    fwd_ms = med(cold_times(torch, run.fwd, sets, cold_iters, flush))
    bwd_ms = med(cold_times(torch, run.bwd, sets, cold_iters, flush))
    attn_ms = fwd_ms + bwd_ms

    # per-kernel durations (HIP events around every launch, on the launch stream), same steps again
    aff.use_timed_library(True)   # the instrumented build of the same sources; the product library has no timing
    for i in range(max(2, min(args.warmup, len(sets)))):  # its code objects are loaded at their first launches
        step(sets[i % len(sets)])
    torch.cuda.synchronize()
    aff.timing_enable(True)
    aff.timing_reset()
    for i in range(args.steps):
        step(sets[i % len(sets)])
    torch.cuda.synchronize()
    kt = aff.timing_read()
    aff.timing_enable(False)
    aff.use_timed_library(False)
    kernels = {n: {"avg_us": 1e3 * ms / max(c, 1), "launches_per_step": c / args.steps} for n, (ms, c) in kt.items()}
    attn_kernels = {n: v for n, v in kernels.items() if n.startswith("pla_") and "plan" not in n}
    elt = 2 if cfg.dtype == "bf16" else 4
    fwd_b, bwd_b = algorithmic_bytes_per_token(cfg.C, cfg.H, cfg.K, elt)
    # Algorithmic bytes per token of each kernel: the tensors it is the first (and, by the method, only
    # necessary) reader or writer of.  The backward is split in two kernels: the key-stationary one owns
    # dk and dv; everything else of the backward belongs to the query-stationary one.
    own = {}
    for n in attn_kernels:
        if "fwd" in n:
            own[n] = fwd_b
        elif "bwd_key" in n:
            own[n] = 2 * cfg.C * elt
        elif "bwd_query" in n:
            own[n] = bwd_b - 2 * cfg.C * elt
        else:  # gather kernels: one kernel per direction
            own[n] = bwd_b
    dom = max(attn_kernels, key=lambda n: attn_kernels[n]["avg_us"] * attn_kernels[n]["launches_per_step"])
    dom_bytes = own[dom] * tokens
    dom_us = attn_kernels[dom]["avg_us"]
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9
    # HBM-side bytes per launch from the rocprofv3 counter runs kept under profiles/ (they cannot be taken inside
    # this process): used only when they were measured on the build that is running
    traffic_all, traffic_stale, traffic_build = {}, None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            tj = json.load(open(tpath))
            traffic_build = tj.get("build_id")
            traffic_stale = traffic_build != aff.build_id()
            if not traffic_stale:
                traffic_all = tj.get(args.config, {})
        except Exception:
            traffic_all = {}
    traffic = traffic_all.get(dom)
    rooflines = [{"kernel": n, "avg_us": attn_kernels[n]["avg_us"], "algorithmic_bytes_per_launch": own[n] * tokens,
                  "achieved": own[n] * tokens / (attn_kernels[n]["avg_us"] * 1e-6) / 1e9,
                  "frac": own[n] * tokens / (attn_kernels[n]["avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS,
                  "traffic": traffic_all.get(n)} for n in sorted(attn_kernels)]

    result = {
        "metric": "neighbourhood-attention fwd+bwd tokens/sec and achieved HBM GB/s (1 MI355X)",
        "value": tokens / (attn_ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * wall / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "N": cfg.N, "C": cfg.C, "H": cfg.H, "K": cfg.K, "S": cfg.S,
                   "M": cfg.M, "coords": cfg.coords, "cluster_promise": promise, "rotating_sets": len(sets),
                   "step": "affmae_cluster + affmae_knn + affmae_pla_plan + affmae_pla_fwd + affmae_pla_bwd; "
                           "value counts fwd+bwd only, each timed apart on cold caches (medians)"},
        "phases_ms": {"cluster": cluster_ms, "knn": knn_ms, "fwd": fwd_ms, "bwd": bwd_ms,
                      "fwd_in_step": fwd_step_ms, "bwd_in_step": bwd_step_ms},
        "cluster_tokens_per_s": tokens / (cluster_ms * 1e-3),
        "knn_tokens_per_s": tokens / (knn_ms * 1e-3),
        "step_tokens_per_s": tokens / (wall / args.steps),
        "algorithmic_bytes_per_token": {"fwd": fwd_b, "bwd": bwd_b},
        "attn_algorithmic_GBs": (fwd_b + bwd_b) * tokens / (attn_ms * 1e-3) / 1e9,
        "attn_frac_of_hbm_peak": (fwd_b + bwd_b) * tokens / (attn_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "copy_probe_GBs": copy_gbs,
        "build_id": aff.build_id(), "traffic_build_id": traffic_build, "traffic_stale": traffic_stale,
        "attn_counter_GBs": (sum(traffic_all[n] for n in attn_kernels) /
                             (sum(v["avg_us"] for v in attn_kernels.values()) * 1e-6) / 1e9
                             if attn_kernels and all(n in traffic_all for n in attn_kernels) else None),
        "kernels": kernels,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_us": dom_us},
        "rooflines_all_kernels": rooflines,
    }

    if not args.no_extras:
        result["relative_position_bias"] = bench_relpos(aff, torch, np, cfg, sets, scale, promise, flush)
        result["neighbourhood_merging"] = bench_merging(aff, torch, np, cfg, sets[0], flush)
        g = bench_graphs(torch, sets, step, attn_only, args.steps)
        result["hip_graph"] = {"step_ms": g["step_ms"], "attn_fwd_bwd_ms": g["attn_fwd_bwd_ms"],
                               "attn_tokens_per_s": tokens / (g["attn_fwd_bwd_ms"] * 1e-3),
                               "step_tokens_per_s": tokens / (g["step_ms"] * 1e-3)}
        result["virtual_tokens"] = bench_virtual_tokens(aff, torch, np, dev)
        del sets
        torch.cuda.empty_cache()
        # the other bf16 configurations of the workload list: same cold loops, fewer repetitions
        result["configs"] = [bench_config(aff, torch, np, CONFIGS[n], dev, flush, 20, promise)
                             for n in ("mae_pt_s1_1024", "merged_stage", "knn_scale") if n != cfg.name]

    if not args.no_cpu_baseline:
        import oracle
        nb = min(cfg.B, 8)
        sl = slice(0, nb)
        t = time.perf_counter()
        rnbr, _ = oracle.knn(w["coords"][sl], None, cfg.S, cfg.M, cfg.K)
        t_knn = time.perf_counter() - t
        reps, t_attn = 0, 0.0
        while t_attn < 1.5 and reps < 20:   # about 10-30 s of CPU work summed over the threads
            t = time.perf_counter()
            oracle.pla_fwd(w["q"][sl], w["k"][sl], w["v"][sl], w["bias"][sl], rnbr, scale)
            oracle.pla_bwd(w["q"][sl], w["k"][sl], w["v"][sl], w["bias"][sl], rnbr, w["dout"][sl], scale)
            t_attn += time.perf_counter() - t
            reps += 1
        result["cpu_baseline"] = {"value": reps * nb * cfg.N / t_attn, "unit": "tokens/s",
                                  "cores": min(oracle.num_threads(), nb), "kind": "oracle",
                                  "sample": f"first {nb} of {cfg.B} images of {cfg.name}, attention fwd+bwd x{reps}, "
                                            f"fp64, one OpenMP thread per image; knn separately",
                                  "knn_tokens_per_s": nb * cfg.N / t_knn, "seconds": t_attn}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
