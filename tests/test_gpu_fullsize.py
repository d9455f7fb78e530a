"""Parity at the full sizes of the workloads, in the launch configuration bench.py times (default tunables
plus the fused head with a workgroup per (tile, worker)).  Two iterations are run on the GPU; the second one is checked stage by stage:
the dense update on every element, the sketch tables of whole workers, every estimate, the gathered
values -- bit for bit against the oracle fed with the GPU's own inputs of that stage.  The index set is
compared with the oracle's full sort where that takes seconds, and otherwise through the properties that
define it uniquely (k coordinates, nothing outside beats anything inside, ties at the threshold go to the
smallest coordinates).
"""
import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2210_07454_amd import inputs

pytestmark = pytest.mark.gpu


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def check_topk_properties(est, idx, k):
    d = est.shape[0]
    assert idx.shape == (k,) and idx.min() >= 0 and idx.max() < d
    assert np.all(np.diff(idx.astype(np.int64)) > 0)                  # ascending, no repeats
    mag = np.abs(est)
    sel = np.zeros(d, bool)
    sel[idx] = True
    tau = mag[idx].min()
    assert mag[~sel].max() <= tau                                     # nothing outside beats anything inside
    eq = np.flatnonzero(mag == tau)                                   # ties at the threshold: smallest coordinates win
    taken = int(sel[eq].sum())
    assert taken >= 1 and sel[eq[:taken]].all() and not sel[eq[taken:]].any()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("wl,full_sort,sketch_workers", [("C2", True, None), ("C3", True, (0, 7, 15)),
                                                          ("C4", False, (7,)), ("P1", True, (0, 15))])
def test_full_size_second_iteration_matches_oracle(wl, full_sort, sketch_workers):
    from paper_2210_07454_amd import sams
    w = inputs.WORKLOADS[wl]
    d, n, r, c, k = w.d, w.n, w.r, w.c, w.k
    sams.sams_configure("fuse_head", 2)
    sams.sams_configure("stage_spread", 1)
    try:
        gs = inputs.GradientStream(w, device="cuda")
        hp = inputs.hash_params(r, seed=w.seed)
        o = Oracle("f32")
        with sams.Context(d, n, r, c, k, hp) as ctx:
            b = sams.Buffers(d, n, r, c, k, w.eps, gs.x1())
            g1, g2 = gs.step(0), gs.step(1)
            # iteration 1 on the GPU up to the gather
            ctx.amsgrad_ef_update(g1, b.m, b.e_u, b.v, b.vhat, b.x, None, None, 0, w.beta1, w.beta2, w.lr)
            ctx.sketch_accumulate(b.e_u, b.S_workers)
            ctx.sketch_reduce(b.S_workers, b.S_mean)
            ctx.unsketch_topk(b.S_mean, b.vhat, b.idx, None)
            ctx.gather_topk(b.e_u, b.vhat, b.idx, b.U_workers, b.delta)
            del g1
            st = dict(m=host(b.m).copy(), e=host(b.e_u).copy(), v=host(b.v).copy(), vhat=host(b.vhat).copy(),
                      x=host(b.x).copy())
            idx1, delta1 = host(b.idx).copy(), host(b.delta).copy()
            # tail of iteration 1 + head of iteration 2 (fused with the staging of u_2) on the GPU ...
            ctx.amsgrad_ef_update(g2, b.m, b.e_u, b.v, b.vhat, b.x, b.idx, b.delta, k, w.beta1, w.beta2, w.lr)
            # ... and in the oracle, on every element
            o.tail(st["e"], st["x"], idx1, delta1, w.lr)
            mask = np.zeros(d, np.uint8)
            mask[idx1] = 1
            o.head(host(g2), st["m"], st["e"], st["v"], st["vhat"], mask, w.beta1, w.beta2)
            del g2
            for key, t in (("m", b.m), ("e", b.e_u), ("v", b.v), ("vhat", b.vhat), ("x", b.x)):
                assert np.array_equal(host(t), st[key]), key
            u = st["e"]
            # stage 1: whole tables of some workers, bit for bit (the binned path adds in coordinate order)
            ctx.sketch_accumulate(b.e_u, b.S_workers)
            S_w = host(b.S_workers)
            for i in (range(n) if sketch_workers is None else sketch_workers):
                assert np.array_equal(S_w[i], o.sketch(u[i], hp, c)), ("sketch", i)
            # stage 2
            ctx.sketch_reduce(b.S_workers, b.S_mean)
            S_mean = host(b.S_mean)
            assert np.array_equal(S_mean, o.sketch_mean(S_w))
            del S_w
            # stage 3: every estimate, then the index set
            est_g = torch.empty(d, device="cuda")
            ctx.unsketch_estimates(b.S_mean, b.vhat, est_g)
            est = o.unsketch(S_mean, st["vhat"], d, hp)
            assert np.array_equal(host(est_g), est)
            del est_g
            ctx.unsketch_topk(b.S_mean, b.vhat, b.idx, None)
            idx = host(b.idx).copy()
            if full_sort:
                assert np.array_equal(idx, o.topk(est, k))
            check_topk_properties(est, idx, k)
            # stage 4
            ctx.gather_topk(b.e_u, b.vhat, b.idx, b.U_workers, b.delta)
            U_w, delta = o.gather(u, st["vhat"], idx)
            assert np.array_equal(host(b.U_workers), U_w) and np.array_equal(host(b.delta), delta)
            # stage 5, tail only
            ctx.amsgrad_ef_update(None, b.m, b.e_u, b.v, b.vhat, b.x, b.idx, b.delta, k, w.beta1, w.beta2, w.lr)
            o.tail(st["e"], st["x"], idx, delta, w.lr)
            assert np.array_equal(host(b.x), st["x"]) and np.array_equal(host(b.e_u), st["e"])
    finally:
        sams.sams_configure("fuse_head", 0)
        sams.sams_configure("stage_spread", 0)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("wl,P", [("C2", 4), ("P1", 8)])
def test_full_size_variants_parameter_averaging_and_second_round(wl, P):
    """The two variants bench.py can time (--variant pa, --overselect P), at a workload's full size and in
    bench.py's launch configuration: one iteration of Alg. 1 with P*k candidates and the exact second round,
    every output compared with the oracle fed with the GPU's inputs of that stage."""
    from paper_2210_07454_amd import sams
    w = inputs.WORKLOADS[wl]
    d, n, r, c, k = w.d, w.n, w.r, w.c, w.k
    kc = P * k
    sams.sams_configure("fuse_head", 2)
    sams.sams_configure("stage_spread", 1)
    try:
        gs = inputs.GradientStream(w, device="cuda")
        hp = inputs.hash_params(r, seed=w.seed)
        o = Oracle("f32")
        with sams.Context(d, n, r, c, kc, hp) as ctx:
            b = sams.Buffers(d, n, r, c, kc, w.eps, gs.x1())
            vw = torch.full((n, d), w.eps, device="cuda")
            vhw = torch.full((n, d), w.eps, device="cuda")
            idx_f = torch.empty(k, device="cuda", dtype=torch.int32)
            delta_f = torch.empty(k, device="cuda")
            st = dict(m=np.zeros((n, d), np.float32), e=np.zeros((n, d), np.float32),
                      vw=np.full((n, d), w.eps, np.float32), vhw=np.full((n, d), w.eps, np.float32), x=host(b.x).copy())
            g1, g2 = gs.step(0), gs.step(1)
            ctx.amsgrad_ef_update_pa(g1, b.m, b.e_u, vw, vhw, b.x, None, None, 0, w.beta1, w.beta2, w.lr)
            o.head_pa(host(g1), st["m"], st["e"], st["vw"], st["vhw"], w.beta1, w.beta2)
            for key, t in (("m", b.m), ("e", b.e_u), ("vw", vw), ("vhw", vhw)):
                assert np.array_equal(host(t), st[key]), key
            ctx.sketch_accumulate(b.e_u, b.S_workers)
            S_w = host(b.S_workers)
            for i in (0, n - 1):
                assert np.array_equal(S_w[i], o.sketch(st["e"][i], hp, c)), ("sketch", i)
            ctx.sketch_reduce(b.S_workers, b.S_mean)
            S_mean = host(b.S_mean)
            assert np.array_equal(S_mean, o.sketch_mean(S_w))
            del S_w
            ctx.unsketch_topk(b.S_mean, None, b.idx, None)            # Alg. 1: plain unsketch operator
            est = o.unsketch(S_mean, None, d, hp)
            cand = o.topk(est, kc)
            assert np.array_equal(host(b.idx), cand)
            ctx.gather_topk(b.e_u, None, b.idx, b.U_workers, b.delta)
            U_w, dcand = o.gather(st["e"], None, cand)
            assert np.array_equal(host(b.U_workers), U_w) and np.array_equal(host(b.delta), dcand)
            ctx.topk_refine(b.idx, b.delta, k, idx_f, delta_f)
            idx, delta = o.refine(cand, dcand, k)
            assert np.array_equal(host(idx_f), idx) and np.array_equal(host(delta_f), delta)
            # tail + the head of the next iteration, fused with the staging of its u
            ctx.amsgrad_ef_update_pa(g2, b.m, b.e_u, vw, vhw, b.x, idx_f, delta_f, k, w.beta1, w.beta2, w.lr)
            o.tail(st["e"], st["x"], idx, delta, w.lr)
            o.head_pa(host(g2), st["m"], st["e"], st["vw"], st["vhw"], w.beta1, w.beta2)
            for key, t in (("m", b.m), ("e", b.e_u), ("vw", vw), ("vhw", vhw), ("x", b.x)):
                assert np.array_equal(host(t), st[key]), ("second head", key)
            ctx.sketch_accumulate(b.e_u, b.S_workers)                 # from the staged copy
            assert np.array_equal(host(b.S_workers[0]), o.sketch(st["e"][0], hp, c))
    finally:
        sams.sams_configure("fuse_head", 0)
        sams.sams_configure("stage_spread", 0)


@pytest.mark.timeout(1500)
def test_stress_size_second_iteration_sampled(capfd):
    """C5 (d = 1.3 G): the binned path with two sketch rows staged at a time so that state, plan and staging fit
    in HBM together (the staging then also holds the looked-up values of all five rows, so the median stays fused).  Outputs the oracle can afford are checked in full (a whole (worker, row) table, the mean
    table, the gathered values), the rest on coordinate ranges at both ends of the vector, and the index set
    through the properties that define it."""
    from paper_2210_07454_amd import sams

    def say(msg):                                     # progress past pytest's capture: minutes of silence look hung
        with capfd.disabled():
            print(f"[fullsize] {msg}", flush=True)

    w = inputs.WORKLOADS["C5"]
    d, n, r, c, k = w.d, w.n, w.r, w.c, w.k
    free, total = torch.cuda.mem_get_info()
    if total < 250 * 2**30:
        pytest.skip("needs a 288 GB device")
    tun = dict(fuse_head=2, stage_rows=2, run_pad=16, stage_spread=1)
    for key, val in tun.items():
        sams.sams_configure(key, val)
    try:
        gs = inputs.GradientStream(w, device="cuda")
        hp = inputs.hash_params(r, seed=w.seed)
        o = Oracle("f32")
        edge = 8_000_000
        ranges = [(0, edge), (d - edge, d)]
        with sams.Context(d, n, r, c, k, hp) as ctx:
            say(f"context ready, scratch {ctx.scratch_bytes / 2**30:.1f} GiB")
            b = sams.Buffers(d, n, r, c, k, w.eps, gs.x1())
            g = gs.step(0)
            ctx.amsgrad_ef_update(g, b.m, b.e_u, b.v, b.vhat, b.x, None, None, 0, w.beta1, w.beta2, w.lr)
            ctx.sketch_accumulate(b.e_u, b.S_workers)
            ctx.sketch_reduce(b.S_workers, b.S_mean)
            ctx.unsketch_topk(b.S_mean, b.vhat, b.idx, None)
            ctx.gather_topk(b.e_u, b.vhat, b.idx, b.U_workers, b.delta)
            torch.cuda.synchronize()
            say("iteration 1 done")
            idx1, delta1 = host(b.idx).copy(), host(b.delta).copy()
            pre = [dict(m=host(b.m[:, a:z].contiguous()), e=host(b.e_u[:, a:z].contiguous()),
                        v=host(b.v[a:z].contiguous()), vhat=host(b.vhat[a:z].contiguous()),
                        x=host(b.x[a:z].contiguous())) for a, z in ranges]
            gs.step(1, out=g)
            ctx.amsgrad_ef_update(g, b.m, b.e_u, b.v, b.vhat, b.x, b.idx, b.delta, k, w.beta1, w.beta2, w.lr)
            # dense update on both ends of the vector, every worker
            for (a, z), st in zip(ranges, pre):
                sel = idx1[(idx1 >= a) & (idx1 < z)] - a
                dl = delta1[(idx1 >= a) & (idx1 < z)]
                o.tail(st["e"], st["x"], sel.astype(np.int32), dl, w.lr)
                mask = np.zeros(z - a, np.uint8)
                mask[sel] = 1
                o.head(host(g[:, a:z].contiguous()), st["m"], st["e"], st["v"], st["vhat"], mask, w.beta1, w.beta2)
                for key, t in (("m", b.m), ("e", b.e_u)):
                    assert np.array_equal(host(t[:, a:z].contiguous()), st[key]), (key, a)
                for key, t in (("v", b.v), ("vhat", b.vhat), ("x", b.x)):
                    assert np.array_equal(host(t[a:z].contiguous()), st[key]), (key, a)
            say("dense update checked on both ends")
            del g, pre
            # stage 1: one whole (worker, row) table, bit for bit (every coordinate of the worker's vector enters it)
            ctx.sketch_accumulate(b.e_u, b.S_workers)
            for i, j in ((n - 1, r - 1),):
                want = o.sketch(host(b.e_u[i]), hp[j:j + 1], c)[0]
                assert np.array_equal(host(b.S_workers[i, j]), want), ("sketch", i, j)
                say(f"table of worker {i}, row {j} checked")
            # stage 2
            ctx.sketch_reduce(b.S_workers, b.S_mean)
            S_mean = host(b.S_mean)
            assert np.array_equal(S_mean, o.sketch_mean(host(b.S_workers)))
            # stage 3: estimates on both ends, index set by its properties
            est_g = torch.empty(d, device="cuda")
            ctx.unsketch_estimates(b.S_mean, b.vhat, est_g)
            for a, z in ranges:
                want = o.unsketch(S_mean, host(b.vhat[a:z].contiguous()), z - a, hp, l0=a)
                assert np.array_equal(host(est_g[a:z].contiguous()), want), ("est", a)
            say("estimates checked on both ends")
            ctx.unsketch_topk(b.S_mean, b.vhat, b.idx, None)
            idx = host(b.idx).copy()
            est = host(est_g)
            del est_g
            check_topk_properties(est, idx, k)
            del est
            say("index set checked")
            # stage 4 on the compacted columns (same arithmetic, the oracle only ever reads u[:, idx])
            ctx.gather_topk(b.e_u, b.vhat, b.idx, b.U_workers, b.delta)
            il = torch.from_numpy(idx.astype(np.int64)).cuda()
            u_c = host(b.e_u[:, il].contiguous())
            vh_c = host(b.vhat[il].contiguous())
            U_w, delta = o.gather(u_c, vh_c, np.arange(k, dtype=np.int32))
            assert np.array_equal(host(b.U_workers), U_w) and np.array_equal(host(b.delta), delta)
            # stage 5, tail only, on the selected coordinates
            x_c = host(b.x[il].contiguous())
            ctx.amsgrad_ef_update(None, b.m, b.e_u, b.v, b.vhat, b.x, b.idx, b.delta, k, w.beta1, w.beta2, w.lr)
            o.tail(u_c, x_c, np.arange(k, dtype=np.int32), delta, w.lr)
            assert np.array_equal(host(b.x[il].contiguous()), x_c)
            assert not host(b.e_u[:, il].contiguous()).any()
            say("gather and tail checked")
    finally:
        for key, val in dict(fuse_head=0, stage_rows=0, run_pad=16, stage_spread=0).items():
            sams.sams_configure(key, val)
