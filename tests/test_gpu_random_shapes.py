"""Seeded sweep over shapes and launch configurations: for every sample one whole iteration (head, the four
sketch stages, tail + next head) runs on the GPU through the C ABI and is compared with the oracle stage by
stage, each stage fed with the GPU's own output of the stage before.  The shapes are small (the oracle takes
milliseconds) but deliberately awkward: d and c of any residue, d below one tile or one wavefront, c = 1,
r from 1 to 16, k from 1 to d, tiles and windows of every allowed size.
"""
import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2210_07454_amd import inputs

pytestmark = pytest.mark.gpu

TOL = 1e-5
DEFAULTS = dict(tile_log2=0, win_log2=0, chunk_log2=0, acc_threads=0, run_pad=16, scatter_threads=1024,
                sketch_path=0, estimate_path=0, fuse_head=0, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=2)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def sample(rng):
    """One shape and one launch configuration (all values inside the documented ranges)."""
    d = int(rng.choice([rng.integers(1, 70), rng.integers(70, 5000), rng.integers(5000, 120_000)]))
    if rng.random() < 0.3:
        d = max(4, d // 4 * 4)                       # the 16-byte paths need d to be a multiple of 4
    n = int(rng.integers(1, 7))
    r = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 13, 16]))
    c = int(rng.choice([1, rng.integers(2, 40), rng.integers(40, 3000), rng.integers(3000, 60_000)]))
    k = int(rng.choice([1, d, rng.integers(1, d + 1), max(1, d // 100)]))
    tun = dict(DEFAULTS)
    if rng.random() < 0.75:
        tun["tile_log2"] = int(rng.integers(6, 15))
        tun["win_log2"] = int(rng.integers(4, 16))
        chunk = int(rng.integers(6, 12))
        tun["chunk_log2"] = chunk
        tun["acc_threads"] = int(rng.choice([t for t in (256, 512, 1024) if t <= (1 << chunk)] or [0]))
        if tun["acc_threads"] == 0:
            tun["chunk_log2"] = 0
        tun["run_pad"] = int(rng.choice([4, 8, 16, 32]))
        tun["scatter_threads"] = int(rng.choice([256, 512, 1024]))
    tun["sketch_path"] = int(rng.choice([0, 0, 2, 2, 3, 1]))
    tun["estimate_path"] = int(rng.choice([0, 2, 2, 1]))
    tun["fuse_head"] = int(rng.integers(0, 3))
    tun["fuse_median"] = int(rng.choice([1, 1, 0]))
    tun["stage_rows"] = int(rng.choice([0, 0, 1, 2, 3]))
    tun["stage_interleave"] = int(rng.integers(0, 2))
    tun["acc_wide"] = int(rng.integers(0, 3))
    return (d, n, r, c, k), tun


def one_iteration(sams, shape, seed):
    d, n, r, c, k = shape
    rng = np.random.default_rng(seed)
    hp = inputs.hash_params(r, seed=seed)
    o = Oracle("f32")
    b1, b2, lr, eps, rho = 0.9, 0.99, 1e-2, 1e-6, 0.8
    scale = (10.0 ** rng.uniform(-3, 1, d)).astype(np.float32)
    g1 = (rng.standard_normal((n, d)) * scale).astype(np.float32)
    g2 = (rng.standard_normal((n, d)) * scale).astype(np.float32)
    x1 = rng.standard_normal(d).astype(np.float32)
    try:
        ctx = sams.Context(d, n, r, c, k, hp)
    except sams.SamsError as e:
        if e.code == sams.SAMS_EINVAL:
            return False                              # a combination of knobs the library refuses (documented)
        raise
    with ctx:
        b = sams.Buffers(d, n, r, c, k, eps, dev(x1))
        st = dict(m=np.zeros((n, d), np.float32), e=np.zeros((n, d), np.float32), v=np.full(d, eps, np.float32),
                  vhat=np.full(d, eps, np.float32), x=x1.copy())
        # head of the first iteration
        ctx.amsgrad_ef_update(dev(g1), b.m, b.e_u, b.v, b.vhat, b.x, None, None, 0, b1, b2, lr)
        o.head(g1, st["m"], st["e"], st["v"], st["vhat"], None, b1, b2)
        for key, t in (("m", b.m), ("e", b.e_u), ("v", b.v), ("vhat", b.vhat), ("x", b.x)):
            assert np.array_equal(host(t), st[key]), key
        u = st["e"]
        # stage 1
        ctx.sketch_accumulate(b.e_u, b.S_workers)
        S_w = host(b.S_workers)
        if ctx.sketch_mode == 2:                      # order-preserving path: the oracle's loop, bit for bit
            assert np.array_equal(S_w, np.stack([o.sketch(u[i], hp, c) for i in range(n)]))
        else:
            o64 = Oracle("f64")
            want = np.stack([o64.sketch(u[i].astype(np.float64), hp, c) for i in range(n)])
            mass = np.stack([o64.sketch(np.abs(u[i]).astype(np.float64), np.stack(
                [hp[:, 0], hp[:, 1], np.full(r, 2, np.uint32), np.zeros(r, np.uint32)], axis=1).astype(np.uint32), c)
                for i in range(n)])                  # sign hash 2*l + 0 is always even: all signs +1
            assert np.all(np.abs(S_w - want) <= TOL * mass + 1e-37)
        # stage 2
        ctx.sketch_reduce(b.S_workers, b.S_mean)
        S_mean = host(b.S_mean)
        assert np.array_equal(S_mean, o.sketch_mean(S_w))
        # stage 3
        est_g = torch.empty(d, device="cuda")
        ctx.unsketch_estimates(b.S_mean, b.vhat, est_g)
        est = o.unsketch(S_mean, st["vhat"], d, hp)
        assert np.array_equal(host(est_g), est)
        ctx.unsketch_topk(b.S_mean, b.vhat, b.idx, None)
        idx = o.topk(est, k)
        assert np.array_equal(host(b.idx), idx)
        # stage 4
        ctx.gather_topk(b.e_u, b.vhat, b.idx, b.U_workers, b.delta)
        U_w, delta = o.gather(u, st["vhat"], idx)
        assert np.array_equal(host(b.U_workers), U_w) and np.array_equal(host(b.delta), delta)
        # stage 5: tail, and the head of the next iteration with a step-size ratio
        ctx.amsgrad_ef_update(dev(g2), b.m, b.e_u, b.v, b.vhat, b.x, b.idx, b.delta, k, b1, b2, lr, ef_ratio=rho)
        o.tail(st["e"], st["x"], idx, delta, lr)
        mask = np.zeros(d, np.uint8)
        mask[idx] = 1
        o.head(g2, st["m"], st["e"], st["v"], st["vhat"], mask, b1, b2, rho=rho)
        for key, t in (("m", b.m), ("e", b.e_u), ("v", b.v), ("vhat", b.vhat), ("x", b.x)):
            assert np.array_equal(host(t), st[key]), ("second head", key)
        # a second sketch: with a fused head it comes from the staged copy
        ctx.sketch_accumulate(b.e_u, b.S_workers)
        if ctx.sketch_mode == 2:
            assert np.array_equal(host(b.S_workers), np.stack([o.sketch(st["e"][i], hp, c) for i in range(n)]))
    return True


@pytest.mark.parametrize("block", range(12))
def test_random_shapes_and_launch_configurations(block, capfd):
    from paper_2210_07454_amd import sams
    sams.load()
    rng = np.random.default_rng(1000 + block)
    ran = 0

    def say(msg):                                     # names the case before it runs, past pytest's capture
        with capfd.disabled():
            print(f"[random-shapes] {msg}", flush=True)

    try:
        for q in range(25):
            shape, tun = sample(rng)
            for key, val in tun.items():
                sams.sams_configure(key, val)
            say(f"sample {block}.{q}: d,n,r,c,k={shape} {tun}")
            ran += bool(one_iteration(sams, shape, seed=100 * block + q))
    finally:
        for key, val in DEFAULTS.items():
            sams.sams_configure(key, val)
    say(f"block {block}: {ran} of 25 samples ran")
    assert ran >= 12                                  # most samples are configurations the library accepts


LIMIT_SHAPES = {
    "most-workers-most-rows": (2048, 1024, 16, 300, 64),
    "most-workers-one-bucket": (4, 1024, 1, 1, 4),
    "one-coordinate": (1, 1, 1, 1, 1),
    "every-coordinate-selected-many-workers": (1000, 100, 5, 50, 1000),
    "one-worker-table-larger-than-the-vector": (3000, 1, 16, 70_000, 17),
}


@pytest.mark.parametrize("fuse_head", [0, 2], ids=["separate-head", "fused-head-per-worker"])
@pytest.mark.parametrize("name", list(LIMIT_SHAPES))
def test_shapes_at_the_documented_limits(name, fuse_head, capfd):
    """The largest worker and row counts sams_create accepts (n = 1024, r = 16), the smallest of everything, k = d,
    and a table with more buckets than the vector has coordinates: one iteration and the head of the next, bit for bit."""
    from paper_2210_07454_amd import sams
    sams.load()
    tun = dict(DEFAULTS, fuse_head=fuse_head, sketch_path=2 if fuse_head else 0)
    try:
        for key, val in tun.items():
            sams.sams_configure(key, val)
        with capfd.disabled():
            print(f"[limits] {name}: d,n,r,c,k={LIMIT_SHAPES[name]} fuse_head={fuse_head}", flush=True)
        assert one_iteration(sams, LIMIT_SHAPES[name], seed=len(name))
    finally:
        for key, val in DEFAULTS.items():
            sams.sams_configure(key, val)
