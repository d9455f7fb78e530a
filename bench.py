#!/usr/bin/env python3
"""Benchmark of the sketched-AMSGrad step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic gradients that are already
resident in HBM: sketch_accumulate -> sketch_reduce -> unsketch_topk -> gather_topk ->
amsgrad_ef_update (which finishes the iteration and runs the dense moment update of the next one).
Prints ONE JSON line: coords/s (= d / t_step), the HBM roofline of the dominant kernel measured with
HIP events inside the timed region (the dominant kernel is found during the warm-up steps and is the only
one bracketed by events while the K steps are timed; the per-kernel table comes from a separate pass of
K steps afterwards), the whole-step roofline fraction, and the CPU oracle timed on a bounded sample of
the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--variant pa] [--overselect P] [--graph]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def step_algorithmic_bytes(d, n, r, c, k, pa=False):
    """Bytes the method itself must move per step: g read, m and e read+written (20nd); v read+written,
    vhat read (12d) -- with parameter averaging v and vhat are per worker, read and written (16nd instead);
    worker tables written once and read once, mean table written once and read once ((2n+2)rc*4); sparse
    second round and update (k(8n+24))."""
    dense = 36 * n * d if pa else 20 * n * d + 12 * d
    return dense + (2 * n + 2) * r * c * 4 + k * (8 * n + 24)


def kernel_algorithmic_bytes(name, d, n, r, c, k, pa=False):
    """Compulsory traffic of one launch of a kernel: its inputs read once plus its outputs written once."""
    rc4 = r * c * 4
    table = {
        "k_head": 20 * n * d + 12 * d,
        "k_sketch_atomic": 4 * n * d + n * rc4,
        "k_bin_scatter": 4 * n * d,             # reads u once; the staging it writes is not algorithmic
        "k_bin_accumulate": n * rc4,            # writes every table cell once; the staging it reads is not
        "k_sketch_lds": 4 * n * d + n * rc4,
        "k_head_sparse_v": k * (4 * n + 4 + 16),  # idx, g of every worker, v and vhat read and written
        "k_head_pa": 36 * n * d,                # g, m, e, v, vhat read; m, u, v, vhat written
        # the head's own traffic; the staging it also writes is not
        "k_head_scatter": 36 * n * d if pa else 20 * n * d + 12 * d,
        "k_bin_lookup": rc4,                    # reads the mean table once
        "k_bin_collect": None,                  # moves only scratch
        "k_est_median": 4 * d + 4 * d,          # vhat read, estimates written
        "k_reduce": (n + 1) * rc4,
        "k_estimate": rc4 + 4 * d + 4 * d,
        "k_sel_hist": 4 * d,
        "k_sel_count": 4 * d,
        "k_sel_write": 4 * d + 4 * k,
        "k_gather": k * (4 + 8 * n + 8),
        "k_tail_x": k * 16,
        "k_fill_u32": None,
    }
    return table.get(name)


def load_traffic(kernel, workload):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), if a summary for this
    workload has been recorded under profiles/ (rows: kernel, launches, fetched raw, fetched scaled, written,
    total scaled, in GB; a timing slot such as k_head_scatter covers the variants whose names start with it)."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"step_{workload}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                cols = line.strip().split(",")
                if line.startswith("#") or len(cols) < 6 or cols[0] == "kernel":
                    continue
                if cols[0].split("::")[-1].split("<")[0].startswith(kernel):
                    return round(float(cols[-1]) * 1e9)
    except (OSError, ValueError):
        pass
    return None


def cpu_baseline(w, sample_d):
    """The oracle as it stands (single thread), one full step on a scaled-down copy of the workload."""
    import numpy as np
    from oracle import Oracle
    from paper_2210_07454_amd import inputs
    ws = w.scaled(sample_d)
    gs = inputs.GradientStream(ws, device="cpu")
    hp = inputs.hash_params(ws.r, seed=ws.seed)
    o = Oracle("f32")
    st = o.init_state(gs.x1().numpy(), ws.n, ws.eps)
    o.step_c(gs.step(0).numpy(), st, hp, ws.c, ws.k, ws.beta1, ws.beta2, ws.lr)   # t = 1 (I_0 empty)
    g = gs.step(1).numpy()
    t0 = time.perf_counter()
    o.step_c(g, st, hp, ws.c, ws.k, ws.beta1, ws.beta2, ws.lr)
    dt = time.perf_counter() - t0
    return {"value": ws.d / dt, "unit": "coords/s", "cores": 1, "kind": "oracle",
            "sample": f"one full step (t=2) of {w.name} scaled to d={ws.d}, n={ws.n}, r={ws.r}, c={ws.c}, "
                      f"k={ws.k}; {dt:.2f} s on 1 thread"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--cpu-sample-d", type=int, default=30_000_000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pool", type=int, default=3, help="distinct gradient batches kept resident")
    ap.add_argument("--variant", choices=["ga", "pa"], default="ga",
                    help="ga: Alg. 2, gradient averaging (the headline); pa: Alg. 1, parameter averaging")
    ap.add_argument("--overselect", type=int, default=1,
                    help="P of the paper's second round: P*k candidates, then topk_refine (default 1: none)")
    ap.add_argument("--no-vram-precondition", action="store_true",
                    help="skip the allocate-and-free pass over the free device memory before the buffers are created")
    ap.add_argument("--graph", action="store_true",
                    help="time the K steps as one replay of a HIP graph captured from them (for small, launch-bound "
                         "workloads); the per-kernel figures then come from an eager pass of K steps run before it")
    ap.add_argument("--tune", default="fuse_head=2",
                    help="library tunables (sams_configure), e.g. fuse_head=1,tile_log2=14,win_log2=15")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the n workers are batched buffers on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2210_07454_amd import inputs, sams

    for item in filter(None, args.tune.split(",")):
        key, val = item.split("=")
        sams.sams_configure(key, int(val))
    w = inputs.WORKLOADS[args.workload]
    d, n, r, c, k = w.d, w.n, w.r, w.c, w.k
    P = max(1, args.overselect)
    kc = P * k                                   # candidates taken from the sketch
    torch.cuda.set_device(0)
    # a graph cannot be captured from the default stream: then everything runs on a stream of its own
    stream = torch.cuda.Stream() if args.graph else torch.cuda.current_stream()
    torch.cuda.set_stream(stream)
    if not args.no_vram_precondition:
        # nearly all free device memory allocated once in 1 GiB blocks and given back, before any buffer of the
        # run exists: afterwards the library's buffers are placed so that the same kernels run 3-14 % faster
        sams.sams_precondition_device_memory(0.995)
    gs = inputs.GradientStream(w, device="cuda")
    hp = inputs.hash_params(r, seed=w.seed)
    ctx = sams.Context(d, n, r, c, kc, hp)
    b = sams.Buffers(d, n, r, c, kc, w.eps, gs.x1())
    idx_f = torch.empty(k, device="cuda", dtype=torch.int32) if P > 1 else b.idx
    delta_f = torch.empty(k, device="cuda") if P > 1 else b.delta
    pool = [gs.step(t) for t in range(max(1, args.pool))]
    pa = args.variant == "pa"
    if pa:                                       # Alg. 1: every worker keeps its own second moments
        v_w = torch.full((n, d), w.eps, device="cuda")
        vhat_w = torch.full((n, d), w.eps, device="cuda")
    vh = None if pa else b.vhat
    torch.cuda.synchronize()

    def update(g, idx, delta, k_sel):
        if pa:
            ctx.amsgrad_ef_update_pa(g, b.m, b.e_u, v_w, vhat_w, b.x, idx, delta, k_sel, w.beta1, w.beta2, w.lr, 1.0)
        else:
            ctx.amsgrad_ef_update(g, b.m, b.e_u, b.v, b.vhat, b.x, idx, delta, k_sel, w.beta1, w.beta2, w.lr, 1.0)

    def one_step(t):
        ctx.sketch_accumulate(b.e_u, b.S_workers)
        ctx.sketch_reduce(b.S_workers, b.S_mean)
        ctx.unsketch_topk(b.S_mean, vh, b.idx, None)
        ctx.gather_topk(b.e_u, vh, b.idx, b.U_workers, b.delta)
        if P > 1:
            ctx.topk_refine(b.idx, b.delta, k, idx_f, delta_f)
        update(pool[(t + 1) % len(pool)], idx_f, delta_f, k)

    # head of the first iteration, then warm-up; the warm-up steps are timed kernel by kernel to find the
    # dominant kernel, which is then the only one bracketed by events inside the timed region (two event records
    # per launch of every kernel double the step time of the small workloads)
    update(pool[0], None, None, 0)
    t = 0
    for q in range(args.warmup):
        if q == min(1, args.warmup - 1):            # the first step carries one-time costs: not timed unless it is the only one
            ctx.sams_profile_enable(True)
        one_step(t)
        t += 1
    torch.cuda.synchronize()
    ctx.sams_profile_enable(False)
    warm = ctx.sams_profile_read()
    dom_name = max(warm.items(), key=lambda kv: kv[1][0])[0] if warm else None

    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed_eager(only):
        nonlocal t
        ctx.sams_profile_only(only)
        ctx.sams_profile_enable(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(args.steps):
            one_step(t)
            t += 1
        ev1.record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ctx.sams_profile_enable(False)
        ctx.sams_profile_only(None)
        return dt, ctx.sams_profile_read()

    wall, prof = timed_eager(dom_name)
    if args.graph:
        # the same K steps, captured once (capture executes nothing) and replayed: one untimed replay, one timed
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for q in range(args.steps):
                one_step(t + q)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        graph.replay()
        ev1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    ev_ms_per_step = ev0.elapsed_time(ev1) / args.steps

    # dominant kernel: largest total device time (over the warm-up steps); its launches inside the timed region
    dom = max(prof.items(), key=lambda kv: kv[1][0])
    dom_name, (dom_ms, dom_n) = dom
    # every kernel's share: a separate pass of K steps after the timed one, every launch bracketed
    _, breakdown = timed_eager(None)
    avg_ms = dom_ms / dom_n
    kbytes = kernel_algorithmic_bytes(dom_name, d, n, r, c, k, pa)
    achieved = (kbytes / (avg_ms * 1e-3)) / 1e9 if kbytes else None
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                "traffic": None if (pa or P > 1) else load_traffic(dom_name, args.workload),   # measured for the default variant
                "algorithmic_bytes_per_launch": kbytes, "avg_launch_ms": avg_ms,
                "launches_per_step": dom_n / args.steps}
    step_bytes = step_algorithmic_bytes(d, n, r, c, k, pa)
    step_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9

    out = {
        "metric": "sketched-AMSGrad step: coords/sec and achieved HBM GB/s vs peak, 1 GPU",
        "value": d / (ms_per_step * 1e-3),
        "unit": "coords/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: d={d}, n={n} simulated workers, sketch {r}x{c}, k={k}, "
                               f"{w.noise} gradients in {w.nseg} segments + {w.heavy} heavy coordinates",
                   "d": d, "n": n, "r": r, "c": c, "k": k, "tunables": args.tune, "overselect_P": P, "variant": args.variant,
                   "vram_preconditioned": not args.no_vram_precondition, "hip_graph": bool(args.graph)},
        "worker_coords_per_s": n * d / (ms_per_step * 1e-3),
        "device_ms_per_step": ev_ms_per_step,
        "step_algorithmic_bytes": step_bytes,
        "step_hbm_gbs": step_gbs,
        "step_roofline_frac": step_gbs / HBM_PEAK_GBS,
        "roofline": roofline,
        "kernels_ms_per_step": {kn: round(v[0] / args.steps, 4) for kn, v in sorted(breakdown.items())},
        "kernels_ms_per_step_from": f"a separate pass of {args.steps} steps after the timed region, every launch bracketed by events",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_d)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
