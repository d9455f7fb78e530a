#!/usr/bin/env python3
"""Benchmark of the sketched-AMSGrad step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic gradients that are already
resident in HBM: sketch_accumulate -> sketch_reduce -> unsketch_topk -> gather_topk ->
amsgrad_ef_update (which finishes the iteration and runs the dense moment update of the next one).
Prints ONE JSON line: coords/s (= d / t_step), the HBM roofline of the dominant kernel measured with
HIP events inside the timed region (the dominant kernel is found during the warm-up steps and is the only
one bracketed by events while the K steps are timed; the per-kernel table comes from a separate pass of
K steps afterwards), the whole-step roofline fraction (against the published 8 TB/s and against the rate a
plain copy reaches on this machine, measured in the run), the median of the per-step times from HIP events, and
the CPU oracle timed on a bounded sample of the same workload (one thread, and with its independent calls
spread over the host's threads).  The K steps are timed twice in one process: first with the device memory
as the process found it, then -- the headline -- after the allocate-and-free pass that
sams_precondition_device_memory describes ("fresh_memory_state" holds the first figure).

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
                    return round(float(cols[-1]) * 1e9), (f"profiles/step_{workload}_hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                                          "runs of this command recorded earlier, not counters of this run")
    except (OSError, ValueError):
        pass
    return None, None


def cpu_baseline(w, sample_d):
    """The oracle as it stands, one full step (t = 2) on a scaled-down copy of the workload: once through its single
    C entry point on one thread, and once stage by stage with the calls that are independent of each other (the n
    per-worker sketches; the estimates of disjoint coordinate ranges) issued from a pool of host threads.  The
    oracle's code is the same in both; every table is still filled by one thread in ascending coordinate order."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import Oracle
    from paper_2210_07454_amd import inputs
    ws = w.scaled(sample_d)
    gs = inputs.GradientStream(ws, device="cpu")
    hp = inputs.hash_params(ws.r, seed=ws.seed)
    o = Oracle("f32")
    g0, g1 = gs.step(0).numpy(), gs.step(1).numpy()
    st = o.init_state(gs.x1().numpy(), ws.n, ws.eps)
    o.step_c(g0, st, hp, ws.c, ws.k, ws.beta1, ws.beta2, ws.lr)   # t = 1 (I_0 empty)
    st2 = {key: val.copy() for key, val in st.items()}              # the same starting point for the threaded run
    t0 = time.perf_counter()
    ref = o.step_c(g1, st, hp, ws.c, ws.k, ws.beta1, ws.beta2, ws.lr)
    dt = time.perf_counter() - t0
    sample = (f"one full step (t=2) of {w.name} scaled to d={ws.d}, n={ws.n}, r={ws.r}, c={ws.c}, k={ws.k}")
    single = {"value": ws.d / dt, "unit": "coords/s", "cores": 1, "kind": "oracle",
              "sample": f"{sample}; {dt:.2f} s on 1 thread"}
    threads = max(1, min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), os.cpu_count() or 1))
    with ThreadPoolExecutor(threads) as pool:
        t0 = time.perf_counter()
        o.head(g1, st2["m"], st2["e"], st2["v"], st2["vhat"], st2["in_prev"], ws.beta1, ws.beta2)
        S_w = np.stack(list(pool.map(lambda i: o.sketch(st2["e"][i], hp, ws.c), range(ws.n))))
        S_mean = o.sketch_mean(S_w)
        cuts = np.linspace(0, ws.d, 4 * threads + 1).astype(np.int64)
        parts = pool.map(lambda q: o.unsketch(S_mean, st2["vhat"][cuts[q]:cuts[q + 1]], int(cuts[q + 1] - cuts[q]), hp,
                                              l0=int(cuts[q])), range(4 * threads))
        est = np.concatenate(list(parts))
        idx = o.topk(est, ws.k)
        _, delta = o.gather(st2["e"], st2["vhat"], idx)
        o.tail(st2["e"], st2["x"], idx, delta, ws.lr)
        dtp = time.perf_counter() - t0
    same = bool(np.array_equal(idx, ref["idx"]) and np.array_equal(st2["x"], st["x"]))
    par = {"value": ws.d / dtp, "unit": "coords/s", "cores": threads, "kind": "oracle", "host_cpu_count": os.cpu_count(),
           "same_result_as_single_thread": same,
           "sample": f"{sample}; {dtp:.2f} s with the per-worker sketches and the estimates of {4 * threads} coordinate "
                     f"ranges spread over {threads} host threads (head, top-k, second round and tail on one)"}
    return single, par


def stream_copy_gbs(torch, nbytes=2 << 30, reps=5):
    """What a plain device-to-device copy of nbytes reaches on this machine (read + written bytes per second, best of reps)."""
    a = torch.empty(nbytes // 4, device="cuda", dtype=torch.float32).fill_(1.0)
    b = torch.empty_like(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    best = float("inf")
    for _ in range(reps + 1):
        e0.record()
        b.copy_(a)
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1))
    del a, b
    return 2 * nbytes / (best * 1e-3) / 1e9


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
    ap.add_argument("--skip-fresh-state", action="store_true",
                    help="do not time the K steps a first time before the allocate-and-free pass (saves the second set-up)")
    ap.add_argument("--graph", action="store_true",
                    help="time the K steps as one replay of a HIP graph captured from them (for small, launch-bound "
                         "workloads); the per-kernel figures then come from an eager pass of K steps run before it")
    ap.add_argument("--tune", default="fuse_head=2,stage_spread=1",
                    help="library tunables (sams_configure), e.g. fuse_head=1,tile_log2=14,win_log2=15")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the n workers are batched buffers on it); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import gc
    import statistics

    import torch
    from paper_2210_07454_amd import inputs, sams

    for item in filter(None, args.tune.split(",")):
        key, val = item.split("=")
        sams.sams_configure(key, int(val))
    w = inputs.WORKLOADS[args.workload]
    d, n, r, c, k = w.d, w.n, w.r, w.c, w.k
    P = max(1, args.overselect)
    kc = P * k                                   # candidates taken from the sketch
    pa = args.variant == "pa"
    torch.cuda.set_device(0)
    # a graph cannot be captured from the default stream: then everything runs on a stream of its own
    stream = torch.cuda.Stream() if args.graph else torch.cuda.current_stream()
    torch.cuda.set_stream(stream)
    hp = inputs.hash_params(r, seed=w.seed)

    def measure(full):
        """Creates the context and the buffers, runs the warm-up and the K timed steps; with `full` also the
        per-kernel pass (and the graph replay).  Everything it allocated is released when it returns."""
        gs = inputs.GradientStream(w, device="cuda")
        ctx = sams.Context(d, n, r, c, kc, hp)
        b = sams.Buffers(d, n, r, c, kc, w.eps, gs.x1())
        idx_f = torch.empty(k, device="cuda", dtype=torch.int32) if P > 1 else b.idx
        delta_f = torch.empty(k, device="cuda") if P > 1 else b.delta
        pool = [gs.step(t) for t in range(max(1, args.pool))]
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
            if q == min(1, args.warmup - 1):        # the first step carries one-time costs: not timed unless it is the only one
                ctx.sams_profile_enable(True)
            one_step(t)
            t += 1
        torch.cuda.synchronize()
        ctx.sams_profile_enable(False)
        warm = ctx.sams_profile_read()
        dom_name = max(warm.items(), key=lambda kv: kv[1][0])[0] if warm else None

        evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]

        def timed_eager(only):
            nonlocal t
            ctx.sams_profile_only(only)
            ctx.sams_profile_enable(True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            evs[0].record()
            for q in range(args.steps):
                one_step(t)
                evs[q + 1].record()
                t += 1
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            ctx.sams_profile_enable(False)
            ctx.sams_profile_only(None)
            return dt, ctx.sams_profile_read()

        wall, prof = timed_eager(dom_name)
        step_ms = [evs[q].elapsed_time(evs[q + 1]) for q in range(args.steps)]
        res = {"wall": wall, "prof": prof, "step_ms": step_ms, "breakdown": None,
               "acc_variant": ctx.accumulate_variant, "scratch_bytes": ctx.scratch_bytes}
        if full and args.graph:
            # the same K steps, captured once (capture executes nothing) and replayed: one untimed replay, one timed
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for q in range(args.steps):
                    one_step(t + q)
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            evs[0].record()
            graph.replay()
            evs[1].record()
            torch.cuda.synchronize()
            res["wall"] = time.perf_counter() - t0
            res["step_ms"] = [evs[0].elapsed_time(evs[1]) / args.steps]
            del graph
        if full:
            # every kernel's share: a separate pass of K steps after the timed one, every launch bracketed
            _, res["breakdown"] = timed_eager(None)
        ctx.close()
        del b, pool, gs, ctx
        gc.collect()
        torch.cuda.empty_cache()
        return res

    # The placement of the library's buffers in device memory changes the step time by 10-14 % (cause not
    # established): on a fresh process the buffers are placed "as they come"; after one allocate-and-free pass over
    # nearly all free device memory (sams_precondition_device_memory) the same kernels run faster.  Both states are
    # timed in this one run, the fresh one first; the headline is the preconditioned one, which a long-running
    # training job would be in.
    fresh = None
    if not args.no_vram_precondition:
        if not args.skip_fresh_state:
            fresh = measure(full=False)
        sams.sams_precondition_device_memory(0.995)
    res = measure(full=True)
    copy_gbs = stream_copy_gbs(torch)

    wall, prof, breakdown = res["wall"], res["prof"], res["breakdown"]
    ms_per_step = wall * 1e3 / args.steps
    # dominant kernel: largest total device time (over the warm-up steps); its launches inside the timed region
    dom = max(prof.items(), key=lambda kv: kv[1][0])
    dom_name, (dom_ms, dom_n) = dom
    avg_ms = dom_ms / dom_n
    kbytes = kernel_algorithmic_bytes(dom_name, d, n, r, c, k, pa)
    achieved = (kbytes / (avg_ms * 1e-3)) / 1e9 if kbytes else None
    traffic, traffic_from = (None, None) if (pa or P > 1) else load_traffic(dom_name, args.workload)   # measured for the default variant
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": (achieved / HBM_PEAK_GBS) if achieved else None,
                "traffic": traffic, "traffic_from": traffic_from,
                "peak_measured_copy": copy_gbs, "frac_of_measured_copy": (achieved / copy_gbs) if achieved else None,
                "algorithmic_bytes_per_launch": kbytes, "avg_launch_ms": avg_ms,
                "launches_per_step": dom_n / args.steps}
    step_bytes = step_algorithmic_bytes(d, n, r, c, k, pa)
    step_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9
    med_ms = statistics.median(res["step_ms"])

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
                   "vram_preconditioned": not args.no_vram_precondition, "hip_graph": bool(args.graph),
                   "accumulate_variant": res["acc_variant"], "library_scratch_bytes": res["scratch_bytes"]},
        "worker_coords_per_s": n * d / (ms_per_step * 1e-3),
        "ms_per_step_median": med_ms,
        "ms_per_step_min_max": [min(res["step_ms"]), max(res["step_ms"])],
        "ms_per_step_from": "ms_per_step: wall clock around the K steps / K; median, min, max: HIP events recorded "
                            "after every step on the library's stream",
        "step_algorithmic_bytes": step_bytes,
        "step_hbm_gbs": step_gbs,
        "step_roofline_frac": step_gbs / HBM_PEAK_GBS,
        "step_frac_of_measured_copy": step_gbs / copy_gbs,
        "stream_copy_gbs": copy_gbs,
        "roofline": roofline,
        "kernels_ms_per_step": {kn: round(v[0] / args.steps, 4) for kn, v in sorted(breakdown.items())},
        "kernels_ms_per_step_from": f"a separate pass of {args.steps} steps after the timed region, every launch bracketed by events",
    }
    if fresh is not None:
        fms = fresh["wall"] * 1e3 / args.steps
        out["fresh_memory_state"] = {
            "ms_per_step": fms, "ms_per_step_median": statistics.median(fresh["step_ms"]), "value": d / (fms * 1e-3),
            "what": "the same K steps timed first in this process, before sams_precondition_device_memory was called "
                    "(context and buffers created, timed, released; then the pass; then everything again for the headline)"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["cpu_baseline_threads"] = cpu_baseline(w, args.cpu_sample_d)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
