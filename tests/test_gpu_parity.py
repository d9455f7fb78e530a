"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  Integer work (hashes, signs, index sets) must match bit for bit; floating
results must match within 1e-5 relative (tables: relative to the absolute mass of the bucket).

Each stage is fed the oracle's bit-identical inputs for that stage ("stage-isolated"); the chained
tests then let the GPU run freely and re-derive every step from the GPU's own previous state.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import Oracle
from paper_2210_07454_amd import inputs

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def sams():
    from paper_2210_07454_amd import sams as mod
    mod.load()
    return mod


PATHS = {  # how sketch_accumulate is carried out (sams_configure); results must not depend on it
    "default": dict(tile_log2=0, win_log2=0, chunk_log2=0, acc_threads=0, run_pad=16, scatter_threads=1024,
                    sketch_path=0, estimate_path=0, fuse_head=0, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=2),
    "worker-major-staging": dict(tile_log2=0, win_log2=0, chunk_log2=0, acc_threads=0, run_pad=16, scatter_threads=1024,
                                 sketch_path=0, estimate_path=2, fuse_head=0, stage_rows=0, fuse_median=1,
                                 stage_interleave=0, acc_wide=0),
    "binned-small-windows": dict(tile_log2=8, win_log2=6, chunk_log2=8, acc_threads=256, run_pad=4,
                                 scatter_threads=256, sketch_path=0, estimate_path=2, fuse_head=0, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=0),
    "binned-ragged": dict(tile_log2=10, win_log2=9, chunk_log2=11, acc_threads=512, run_pad=32,
                          scatter_threads=512, sketch_path=0, estimate_path=2, fuse_head=0, stage_rows=0, fuse_median=0, stage_interleave=0, acc_wide=0),
    "binned-unroll2": dict(tile_log2=12, win_log2=8, chunk_log2=11, acc_threads=1024, run_pad=16,
                           scatter_threads=1024, sketch_path=0, estimate_path=2, fuse_head=0, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=0),
    "global-atomic": dict(tile_log2=14, win_log2=15, chunk_log2=11, acc_threads=1024, run_pad=32,
                          scatter_threads=1024, sketch_path=1, estimate_path=2, fuse_head=0, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=0),
    "lds-atomics": dict(tile_log2=14, win_log2=15, chunk_log2=11, acc_threads=1024, run_pad=32,
                        scatter_threads=1024, sketch_path=3, estimate_path=2, fuse_head=0, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=0),
    "fused-head": dict(tile_log2=14, win_log2=14, chunk_log2=10, acc_threads=1024, run_pad=32,
                       scatter_threads=1024, sketch_path=0, estimate_path=2, fuse_head=1, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=0),
    "fused-head-small-tiles": dict(tile_log2=9, win_log2=7, chunk_log2=9, acc_threads=256, run_pad=8,
                                   scatter_threads=256, sketch_path=0, estimate_path=2, fuse_head=1, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=0),
    "fused-head-per-worker": dict(tile_log2=0, win_log2=0, chunk_log2=0, acc_threads=0, run_pad=32,
                                  scatter_threads=1024, sketch_path=2, estimate_path=2, fuse_head=2, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=0),
    "row-groups": dict(tile_log2=11, win_log2=9, chunk_log2=10, acc_threads=512, run_pad=32,
                       scatter_threads=512, sketch_path=0, estimate_path=2, fuse_head=1, stage_rows=2, fuse_median=1, stage_interleave=0, acc_wide=0),
    "one-row-at-a-time": dict(tile_log2=12, win_log2=10, chunk_log2=10, acc_threads=1024, run_pad=16,
                              scatter_threads=1024, sketch_path=0, estimate_path=2, fuse_head=0, stage_rows=1, fuse_median=1, stage_interleave=0, acc_wide=0),
    "estimate-by-gathers": dict(tile_log2=14, win_log2=14, chunk_log2=10, acc_threads=1024, run_pad=32,
                                scatter_threads=1024, sketch_path=0, estimate_path=1, fuse_head=0, stage_rows=0, fuse_median=1, stage_interleave=0, acc_wide=0),
    "interleaved-staging": dict(tile_log2=0, win_log2=0, chunk_log2=0, acc_threads=0, run_pad=16,
                                scatter_threads=1024, sketch_path=2, estimate_path=2, fuse_head=2, stage_rows=0, fuse_median=1,
                                stage_interleave=1, acc_wide=0),
    "interleaved-staging-row-groups": dict(tile_log2=11, win_log2=9, chunk_log2=8, acc_threads=256, run_pad=4,
                                           scatter_threads=512, sketch_path=0, estimate_path=2, fuse_head=1, stage_rows=2,
                                           fuse_median=1, stage_interleave=1, acc_wide=0),
    "interleaved-staging-unfused": dict(tile_log2=10, win_log2=8, chunk_log2=11, acc_threads=512, run_pad=32,
                                        scatter_threads=256, sketch_path=0, estimate_path=2, fuse_head=0, stage_rows=0,
                                        fuse_median=0, stage_interleave=1, acc_wide=0),
    "accumulate-16-byte-loads": dict(tile_log2=12, win_log2=10, chunk_log2=11, acc_threads=1024, run_pad=8,
                                     scatter_threads=1024, sketch_path=2, estimate_path=2, fuse_head=2, stage_rows=0,
                                     fuse_median=1, stage_interleave=1, acc_wide=1),
    "chunk-records": dict(tile_log2=14, win_log2=15, chunk_log2=11, acc_threads=1024, run_pad=16,
                          scatter_threads=1024, sketch_path=2, estimate_path=2, fuse_head=2, stage_rows=0,
                          fuse_median=1, stage_interleave=1, acc_wide=2),
    "chunk-records-worker-major": dict(tile_log2=13, win_log2=15, chunk_log2=11, acc_threads=1024, run_pad=32,
                                       scatter_threads=512, sketch_path=2, estimate_path=2, fuse_head=0, stage_rows=2,
                                       fuse_median=1, stage_interleave=0, acc_wide=2),
    "accumulate-16-byte-loads-worker-major": dict(tile_log2=10, win_log2=8, chunk_log2=11, acc_threads=1024, run_pad=32,
                                                  scatter_threads=256, sketch_path=0, estimate_path=2, fuse_head=0,
                                                  stage_rows=2, fuse_median=1, stage_interleave=0, acc_wide=1),
}


@pytest.fixture(params=[0, 1, 2], ids=["separate-head", "fused-head", "fused-head-per-worker"])
def fused(request, sams):
    """Default launch configuration with the head either on its own or fused with the first sketch pass."""
    sams.sams_configure("fuse_head", request.param)
    sams.sams_configure("sketch_path", 2 if request.param else 0)    # the fused head needs the binned path
    yield request.param
    sams.sams_configure("fuse_head", 0)
    sams.sams_configure("sketch_path", 0)


@pytest.fixture(params=list(PATHS))
def path(request, sams):
    for key, val in PATHS[request.param].items():
        sams.sams_configure(key, val)
    yield request.param
    for key, val in PATHS["default"].items():
        sams.sams_configure(key, val)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def abs_mass(u, hp, c):
    """A[i][j][b] = sum of |u[i][l]| over the coordinates of bucket b of row j (fp64)."""
    n, d = u.shape
    bkt, _ = oracle.hash_dump(hp, c, d)
    A = np.zeros((n, hp.shape[0], c))
    for i in range(n):
        for j in range(hp.shape[0]):
            A[i, j] = np.bincount(bkt[j], weights=np.abs(u[i]).astype(np.float64), minlength=c)
    return A


SHAPES = [  # d, n, r, c, k  -- several tiles, ragged tails, non-power-of-two c, even r, extremes
    (65_536, 4, 5, 2_048, 256),
    (100_003, 3, 5, 1_000, 777),
    (70_001, 2, 10, 400, 500),
    (33, 1, 1, 1, 1),
    (5_000, 2, 16, 7, 5_000),
    (262_144, 8, 7, 100_000, 3_000),
    (4_100, 5, 3, 8_191, 1),
    (9_001, 19, 4, 300, 777),                     # many workers: the sparse kernels take 32 lanes per coordinate
    (3_000, 33, 2, 64, 13),
]


@pytest.mark.parametrize("d,n,r,c,k", SHAPES)
def test_hash_indices_and_signs_bit_exact(sams, d, n, r, c, k):
    hp = inputs.hash_params(r, seed=d % 97)
    with sams.Context(d, n, r, c, k, hp) as ctx:
        b = torch.empty((r, d), device="cuda", dtype=torch.int32)
        s = torch.empty((r, d), device="cuda", dtype=torch.int8)
        ctx.sams_hash_dump(b, s)
        bo, so = oracle.hash_dump(hp, c, d)
        assert np.array_equal(host(b), bo)
        assert np.array_equal(host(s), so)


def test_hash_extreme_parameters_bit_exact(sams):
    P = inputs.P31
    hp = np.array([[P - 1, P - 1, P - 1, P - 1], [1, 0, 1, P - 1], [P - 1, 0, 2, 1], [46341, P - 2, P - 2, 5]],
                  dtype=np.uint32)
    d, c = 300_001, 99_991
    with sams.Context(d, 1, 4, c, 1, hp) as ctx:
        b = torch.empty((4, d), device="cuda", dtype=torch.int32)
        s = torch.empty((4, d), device="cuda", dtype=torch.int8)
        ctx.sams_hash_dump(b, s)
        bo, so = oracle.hash_dump(hp, c, d)
        assert np.array_equal(host(b), bo) and np.array_equal(host(s), so)


@pytest.mark.parametrize("d,n,r,c,k", SHAPES)
def test_sketch_accumulate_integer_inputs_bit_exact(sams, path, d, n, r, c, k):
    hp = inputs.hash_params(r, seed=3)
    amax = 64 if d * 64 < (1 << 24) else max(1, (1 << 23) // d)
    u = inputs.integer_vectors(n, d, amax=amax, seed=d).numpy()
    o = Oracle("f32")
    want = np.stack([o.sketch(u[i], hp, c) for i in range(n)])
    with sams.Context(d, n, r, c, k, hp) as ctx:
        S = torch.full((n, r, c), 7.0, device="cuda")          # must be overwritten, not accumulated into
        ctx.sketch_accumulate(dev(u), S)
        assert np.array_equal(host(S), want)
        Sm = torch.empty((r, c), device="cuda")
        ctx.sketch_reduce(S, Sm)
        assert np.array_equal(host(Sm), o.sketch_mean(want))


@pytest.mark.parametrize("wl,d", [("C1", 65_536), ("C2", 300_000), ("C3", 200_000), ("C4", 500_000)])
def test_sketch_accumulate_float_within_tolerance(sams, path, wl, d):
    w = inputs.WORKLOADS[wl].scaled(d)
    gs = inputs.GradientStream(w, device="cuda")
    u = gs.step(0)
    uh = host(u)
    hp = inputs.hash_params(w.r, seed=1)
    o64 = Oracle("f64")
    want = np.stack([o64.sketch(uh[i].astype(np.float64), hp, w.c) for i in range(w.n)])
    A = abs_mass(uh, hp, w.c)
    with sams.Context(w.d, w.n, w.r, w.c, w.k, hp) as ctx:
        S = torch.empty((w.n, w.r, w.c), device="cuda")
        ctx.sketch_accumulate(u, S)
        got32 = host(S)
        got = got32.astype(np.float64)
        binned = ctx.sketch_mode == 2
    assert np.all(np.abs(got - want) <= TOL * A + 1e-37)
    if binned:
        # binned path: terms are added in ascending coordinate order, exactly like the oracle's loop
        o32 = Oracle("f32")
        assert np.array_equal(got32, np.stack([o32.sketch(uh[i], hp, w.c) for i in range(w.n)]))


@pytest.mark.parametrize("d,c", [(262_144, 100_000), (70_001, 400)])
def test_sketch_accumulate_keeps_subnormal_sums(sams, path, d, c):
    """Values that are small multiples of 2^-140: every partial sum is exact and subnormal, so the tables must equal
    the oracle's bit for bit on every path -- unless some add flushes subnormal numbers to zero."""
    n, r, k = 3, 5, 10
    hp = inputs.hash_params(r, seed=9)
    ints = inputs.integer_vectors(n, d, amax=16, seed=d + 1).numpy()
    u = (ints.astype(np.float64) * 2.0 ** -140).astype(np.float32)
    assert np.any(u != 0) and np.all(np.abs(u) < np.finfo(np.float32).tiny)
    o = Oracle("f32")
    want = np.stack([o.sketch(u[i], hp, c) for i in range(n)])
    assert np.any(want != 0)
    with sams.Context(d, n, r, c, k, hp) as ctx:
        S = torch.empty((n, r, c), device="cuda")
        ctx.sketch_accumulate(dev(u), S)
        assert np.array_equal(host(S), want)


@pytest.mark.parametrize("d,n,r,c,k", [(400_001, 1, 3, 150_001, 50),       # one worker, ragged last window, d not a multiple of 4
                                       (250_000, 4, 5, 65_536, 100),       # two full windows
                                       (131_072, 2, 16, 40_000, 10),       # sixteen rows, one partly filled window
                                       (1_000_000, 3, 2, 1_000_003, 7)])   # 31 windows, long bins
@pytest.mark.parametrize("layout", ["chunk-records", "chunk-records-worker-major"])
def test_record_kernel_tables_bit_exact(sams, layout, d, n, r, c, k):
    """The second pass through chunk records (values and codes in registers, chains by rank) on shapes chosen so that
    most rows do use records: float inputs, tables equal to the sequential sum bit for bit."""
    hp = inputs.hash_params(r, seed=21)
    rng = np.random.default_rng(d + n)
    u = (rng.standard_normal((n, d)) * 10.0 ** rng.uniform(-5, 0, (n, d))).astype(np.float32)
    o = Oracle("f32")
    want = np.stack([o.sketch(u[i], hp, c) for i in range(n)])
    for key, val in dict(PATHS[layout], fuse_head=0).items():
        sams.sams_configure(key, val)
    try:
        with sams.Context(d, n, r, c, k, hp) as ctx:
            assert bin(ctx.record_rows).count("1") >= r // 2, ctx.record_rows
            S = torch.full((n, r, c), 3.0, device="cuda")
            ctx.sketch_accumulate(dev(u), S)
            assert np.array_equal(host(S), want)
    finally:
        for key, val in PATHS["default"].items():
            sams.sams_configure(key, val)


def test_rows_choose_between_chunk_records_and_meta_words_one_by_one(sams):
    """Row 0's bucket hash multiplies by c (a power of two), so that thousands of consecutive coordinates share a
    bucket: its chunks do not fit the record format and it keeps its meta words, while the other rows use records.
    The tables must equal the sequential sum bit for bit either way, also when rows are staged in groups."""
    d, n, r, c, k = 300_000, 3, 4, 1 << 17, 100
    hp = inputs.hash_params(r, seed=12)
    hp[0, 0] = c
    rng = np.random.default_rng(3)
    u = (rng.standard_normal((n, d)) * 10.0 ** rng.uniform(-4, 0, (n, d))).astype(np.float32)
    o = Oracle("f32")
    want = np.stack([o.sketch(u[i], hp, c) for i in range(n)])
    try:
        for rows in (0, 3):
            for key, val in dict(PATHS["chunk-records"], stage_rows=rows).items():
                sams.sams_configure(key, val)
            with sams.Context(d, n, r, c, k, hp) as ctx:
                mask = ctx.record_rows
                assert mask & 1 == 0 and mask != 0 and ctx.accumulate_variant == 1, mask
                S = torch.empty((n, r, c), device="cuda")
                ctx.sketch_accumulate(dev(u), S)
                assert np.array_equal(host(S), want)
    finally:
        for key, val in PATHS["default"].items():
            sams.sams_configure(key, val)


@pytest.mark.parametrize("n,r,c", [(4, 5, 2048), (8, 5, 100_003), (16, 7, 5000), (3, 2, 17), (1, 1, 1)])
def test_sketch_reduce_bit_exact(sams, n, r, c):
    rng = np.random.default_rng(c)
    S_w = (rng.standard_normal((n, r, c)) * 10.0 ** rng.uniform(-4, 2, (n, r, c))).astype(np.float32)
    with sams.Context(1000, n, r, c, 10, inputs.hash_params(r)) as ctx:
        Sm = torch.empty((r, c), device="cuda")
        ctx.sketch_reduce(dev(S_w), Sm)
        assert np.array_equal(host(Sm), Oracle("f32").sketch_mean(S_w))


@pytest.mark.parametrize("d,n,r,c,k", SHAPES)
@pytest.mark.parametrize("use_vhat", [True, False])
def test_estimates_and_topk_bit_exact(sams, path, d, n, r, c, k, use_vhat):
    rng = np.random.default_rng(d + r)
    hp = inputs.hash_params(r, seed=5)
    S = (rng.standard_normal((r, c)) * 10.0 ** rng.uniform(-3, 0, (r, c))).astype(np.float32)
    vhat = (10.0 ** rng.uniform(-8, 0, d)).astype(np.float32) if use_vhat else None
    o = Oracle("f32")
    est = o.unsketch(S, vhat, d, hp)
    idx = o.topk(est, k)
    with sams.Context(d, n, r, c, k, hp) as ctx:
        Sd, vd = dev(S), (dev(vhat) if use_vhat else None)
        est_g = torch.empty(d, device="cuda")
        ctx.unsketch_estimates(Sd, vd, est_g)
        assert np.array_equal(host(est_g), est)
        idx_g = torch.full((k,), -1, device="cuda", dtype=torch.int32)
        sel_g = torch.empty(k, device="cuda")
        ctx.unsketch_topk(Sd, vd, idx_g, sel_g)
        assert np.array_equal(host(idx_g), idx)
        assert np.array_equal(host(sel_g), est[idx])
        ctx.unsketch_topk(Sd, vd, idx_g, None)                # est_sel is optional
        assert np.array_equal(host(idx_g), idx)


@pytest.mark.parametrize("k", [1, 100, 2_500, 19_999, 20_000])
def test_topk_ties_go_to_the_smaller_index(sams, k):
    # a table with three distinct magnitudes (and zeros of both signs) makes almost every |est| a tie
    d, r, c = 20_000, 3, 64
    rng = np.random.default_rng(k)
    hp = inputs.hash_params(r, seed=8)
    S = rng.choice(np.array([-2.0, -1.0, -0.0, 0.0, 1.0, 2.0], dtype=np.float32), size=(r, c))
    o = Oracle("f32")
    est = o.unsketch(S, None, d, hp)
    assert len(np.unique(np.abs(est))) <= 3
    want = o.topk(est, k)
    with sams.Context(d, 1, r, c, k, hp) as ctx:
        idx_g = torch.empty(k, device="cuda", dtype=torch.int32)
        ctx.unsketch_topk(dev(S), None, idx_g, None)
        assert np.array_equal(host(idx_g), want)


@pytest.mark.parametrize("d,n,r,c,k", SHAPES)
def test_gather_topk_bit_exact(sams, d, n, r, c, k):
    rng = np.random.default_rng(d)
    u = rng.standard_normal((n, d)).astype(np.float32)
    vhat = (10.0 ** rng.uniform(-8, 0, d)).astype(np.float32)
    idx = np.sort(rng.choice(d, k, replace=False)).astype(np.int32)
    o = Oracle("f32")
    with sams.Context(d, n, r, c, k, inputs.hash_params(r)) as ctx:
        for vh in (vhat, None):
            U_w, delta = o.gather(u, vh, idx)
            Ug = torch.empty((n, k), device="cuda")
            dg = torch.empty(k, device="cuda")
            ctx.gather_topk(dev(u), dev(vh) if vh is not None else None, dev(idx), Ug, dg)
            assert np.array_equal(host(Ug), U_w) and np.array_equal(host(dg), delta)


@pytest.mark.parametrize("d,n,r,c,k", SHAPES)
def test_amsgrad_ef_update_head_and_tail_bit_exact(sams, path, d, n, r, c, k):
    rng = np.random.default_rng(d + 1)
    o = Oracle("f32")
    b1, b2, lr = 0.9, 0.99, 1e-3
    f = lambda *s: (rng.standard_normal(s) * 10.0 ** rng.uniform(-4, 0, s)).astype(np.float32)
    g1, g2, m, e, x = f(n, d), f(n, d), f(n, d), f(n, d), f(d)
    v = (10.0 ** rng.uniform(-8, -2, d)).astype(np.float32)
    vhat = np.maximum(v, (10.0 ** rng.uniform(-8, -2, d)).astype(np.float32))
    idx = np.sort(rng.choice(d, k, replace=False)).astype(np.int32)
    delta = f(k)
    with sams.Context(d, n, r, c, k, inputs.hash_params(r)) as ctx:
        md, ed, vd, vhd, xd = dev(m), dev(e), dev(v), dev(vhat), dev(x)
        # first call of a run: head only, I_0 empty
        ctx.amsgrad_ef_update(dev(g1), md, ed, vd, vhd, xd, None, None, 0, b1, b2, lr)
        o.head(g1, m, e, v, vhat, None, b1, b2)
        for got, want in ((md, m), (ed, e), (vd, v), (vhd, vhat), (xd, x)):
            assert np.array_equal(host(got), want)
        # steady state: tail of t, head of t+1 with I_t = idx, error-feedback ratio != 1
        ctx.amsgrad_ef_update(dev(g2), md, ed, vd, vhd, xd, dev(idx), dev(delta), k, b1, b2, lr, 0.75)
        o.tail(e, x, idx, delta, lr)
        mask = np.zeros(d, np.uint8)
        mask[idx] = 1
        o.head(g2, m, e, v, vhat, mask, b1, b2, rho=0.75)
        for got, want in ((md, m), (ed, e), (vd, v), (vhd, vhat), (xd, x)):
            assert np.array_equal(host(got), want)
        # last call of a run: tail only
        idx2 = np.sort(rng.choice(d, k, replace=False)).astype(np.int32)
        ctx.amsgrad_ef_update(None, md, ed, vd, vhd, xd, dev(idx2), dev(delta), k, b1, b2, lr)
        o.tail(e, x, idx2, delta, lr)
        for got, want in ((md, m), (ed, e), (vd, v), (vhd, vhat), (xd, x)):
            assert np.array_equal(host(got), want)


INDEX_SETS = {
    "every-coordinate": lambda d, rng: np.arange(d),
    "every-other": lambda d, rng: np.arange(0, d, 2),
    "whole-bitmap-words": lambda d, rng: np.concatenate([np.arange(w * 32, w * 32 + 32) for w in (0, 7, 511, 512, d // 32 - 1)]),
    "tile-edges": lambda d, rng: np.unique(np.concatenate([[0, d - 1], np.arange(1, d >> 10) * 1024 - 1, np.arange(1, d >> 10) * 1024])),
    "one-coordinate": lambda d, rng: np.array([d // 3]),
    "dense-random": lambda d, rng: np.sort(rng.choice(d, d // 3, replace=False)),
    "one-tile-only": lambda d, rng: 16384 + np.sort(rng.choice(16384, 900, replace=False)),
}


@pytest.mark.parametrize("shape", list(INDEX_SETS))
@pytest.mark.parametrize("d,tile_log2", [(50_000, 0), (70_004, 10)], ids=["tiles-2^14", "tiles-2^10-ragged-d"])
def test_head_per_worker_on_dense_and_clustered_index_sets(sams, shape, d, tile_log2):
    """Sec. II-C, Alg. 2: v_t = beta2 v_{t-1} + (1 - beta2) h_t^2 with h_t the workers' mean gradient on I_{t-1}, zero elsewhere.
    The head that runs one workgroup per (tile, worker) takes h_t from the gradients it has compacted by their rank in the index set;
    index sets with full bitmap words, neighbours across word and tile borders, a single member and empty tiles."""
    n, r, c = 3, 3, 5000
    rng = np.random.default_rng(len(shape) * 1000 + d)
    o = Oracle("f32")
    b1, b2, lr = 0.9, 0.99, 1e-3
    f = lambda *s: (rng.standard_normal(s) * 10.0 ** rng.uniform(-4, 0, s)).astype(np.float32)
    idx = INDEX_SETS[shape](d, rng).astype(np.int32)
    k = len(idx)
    g1, g2, m, e, x, delta = f(n, d), f(n, d), f(n, d), f(n, d), f(d), f(k)
    v = (10.0 ** rng.uniform(-8, -2, d)).astype(np.float32)
    vhat = np.maximum(v, (10.0 ** rng.uniform(-8, -2, d)).astype(np.float32))
    for key, val in dict(PATHS["default"], fuse_head=2, sketch_path=2, tile_log2=tile_log2).items():
        sams.sams_configure(key, val)
    try:
        with sams.Context(d, n, r, c, k, inputs.hash_params(r)) as ctx:
            md, ed, vd, vhd, xd = dev(m), dev(e), dev(v), dev(vhat), dev(x)
            ctx.amsgrad_ef_update(dev(g1), md, ed, vd, vhd, xd, None, None, 0, b1, b2, lr)
            o.head(g1, m, e, v, vhat, None, b1, b2)
            for _ in range(2):                                  # twice: the second head reads what the first tail of the pair left
                ctx.amsgrad_ef_update(dev(g2), md, ed, vd, vhd, xd, dev(idx), dev(delta), k, b1, b2, lr)
                o.tail(e, x, idx, delta, lr)
                mask = np.zeros(d, np.uint8)
                mask[idx] = 1
                o.head(g2, m, e, v, vhat, mask, b1, b2)
                for name, got, want in (("m", md, m), ("e", ed, e), ("v", vd, v), ("vhat", vhd, vhat), ("x", xd, x)):
                    assert np.array_equal(host(got), want), name
                g2 = f(n, d)
            S = torch.empty(n, r, c, device="cuda")
            ctx.sketch_accumulate(ed, S)                        # the staged copy the head left is the sketch of u
            assert np.array_equal(host(S), np.stack([o.sketch(e[i], inputs.hash_params(r), c) for i in range(n)]))
    finally:
        for key, val in PATHS["default"].items():
            sams.sams_configure(key, val)


@pytest.mark.parametrize("k_in,k_out", [(1, 1), (64, 64), (1000, 37), (50_000, 12_500), (400_000, 50_000)])
def test_topk_refine_bit_exact_with_ties(sams, k_in, k_out):
    d = 3_000_000
    rng = np.random.default_rng(k_in)
    cand = np.sort(rng.choice(d, k_in, replace=False)).astype(np.int32)
    vals = (rng.integers(-9, 10, k_in) / 4.0).astype(np.float32)
    vals[rng.integers(0, k_in, max(1, k_in // 8))] = -0.0
    idx, delta = Oracle("f32").refine(cand, vals, k_out)
    with sams.Context(d, 2, 3, 1000, k_in, inputs.hash_params(3)) as ctx:
        io = torch.full((k_out,), -1, device="cuda", dtype=torch.int32)
        do = torch.empty(k_out, device="cuda")
        ctx.topk_refine(dev(cand), dev(vals), k_out, io, do)
        assert np.array_equal(host(io), idx) and np.array_equal(host(do), delta)


@pytest.mark.parametrize("in_bin", [1, 700, 8191, 8192, 8193, 20_000, 60_000])
@pytest.mark.parametrize("k_in", [60_000, 65_536, 4_100])
def test_one_workgroup_selection_around_the_capacity_of_its_candidate_list(sams, k_in, in_bin):
    """Selection of short vectors (one workgroup): the keys that share the first radix digit of the threshold are
    listed in LDS when at most 8192 do, otherwise the later digits come from sweeps over all keys.  `in_bin` keys
    lie in [1.5, 1.625) (one value of the first digit), 300 above, the rest far below; the threshold falls among the
    `in_bin`, with exact ties among them."""
    in_bin = min(in_bin, k_in - 300)
    rng = np.random.default_rng(k_in + in_bin)
    vals = (rng.uniform(0.001, 0.1, k_in) * rng.choice([-1.0, 1.0], k_in)).astype(np.float32)
    where = rng.permutation(k_in)
    vals[where[:300]] = rng.uniform(2.0, 9.0, 300).astype(np.float32)
    grid = (1.5 + rng.integers(0, 64, in_bin) / 512.0).astype(np.float32)          # 64 distinct values: many ties
    vals[where[300:300 + in_bin]] = grid * rng.choice([-1.0, 1.0], in_bin).astype(np.float32)
    cand = np.arange(k_in, dtype=np.int32) * 3
    o = Oracle("f32")
    with sams.Context(3 * k_in, 2, 3, 1000, k_in, inputs.hash_params(3)) as ctx:
        for k_out in sorted({300 + max(1, in_bin // 2), 300 + in_bin, 301, min(k_in, 300 + in_bin + 5)}):
            idx, delta = o.refine(cand, vals, k_out)
            io = torch.full((k_out,), -1, device="cuda", dtype=torch.int32)
            do = torch.empty(k_out, device="cuda")
            ctx.topk_refine(dev(cand), dev(vals), k_out, io, do)
            assert np.array_equal(host(io), idx) and np.array_equal(host(do), delta), k_out


@pytest.mark.parametrize("wl,d,P", [("C4", 400_000, 4), ("P1", 600_000, 8), ("P2a", 60_000, 4)])
def test_chained_steps_with_overselection_follow_the_oracle(sams, wl, d, P):
    """The paper's second round (Sec. III-A) with P*k candidates: context created with k = P*k, top-k refined
    from the exact values; every step is re-derived by the oracle from the GPU's previous state."""
    w = inputs.WORKLOADS[wl].scaled(d) if d != inputs.WORKLOADS[wl].d else inputs.WORKLOADS[wl]
    k, kc = w.k, P * w.k
    gs = inputs.GradientStream(w, device="cuda")
    hp = inputs.hash_params(w.r, seed=w.seed)
    o = Oracle("f32")
    steps = 4
    with sams.Context(w.d, w.n, w.r, w.c, kc, hp) as ctx:
        b = sams.Buffers(w.d, w.n, w.r, w.c, kc, w.eps, gs.x1())
        idx_f = torch.empty(k, device="cuda", dtype=torch.int32)
        delta_f = torch.empty(k, device="cuda")
        G = [gs.step(t) for t in range(steps)]
        st = dict(m=np.zeros((w.n, w.d), np.float32), e=np.zeros((w.n, w.d), np.float32),
                  v=np.full(w.d, w.eps, np.float32), vhat=np.full(w.d, w.eps, np.float32), x=host(b.x).copy())
        mask = None
        ctx.amsgrad_ef_update(G[0], b.m, b.e_u, b.v, b.vhat, b.x, None, None, 0, w.beta1, w.beta2, w.lr)
        for t in range(steps):
            o.head(host(G[t]), st["m"], st["e"], st["v"], st["vhat"], mask, w.beta1, w.beta2)
            assert np.array_equal(host(b.e_u), st["e"]) and np.array_equal(host(b.vhat), st["vhat"]), t
            ctx.sketch_accumulate(b.e_u, b.S_workers)
            ctx.sketch_reduce(b.S_workers, b.S_mean)
            ctx.unsketch_topk(b.S_mean, b.vhat, b.idx, None)
            ctx.gather_topk(b.e_u, b.vhat, b.idx, b.U_workers, b.delta)
            ctx.topk_refine(b.idx, b.delta, k, idx_f, delta_f)
            est = o.unsketch(host(b.S_mean), st["vhat"], w.d, hp)
            cand = o.topk(est, kc)
            assert np.array_equal(host(b.idx), cand), t
            _, dcand = o.gather(st["e"], st["vhat"], cand)
            assert np.array_equal(host(b.delta), dcand), t
            idx, delta = o.refine(cand, dcand, k)
            assert np.array_equal(host(idx_f), idx) and np.array_equal(host(delta_f), delta), t
            g_next = G[t + 1] if t + 1 < steps else None
            ctx.amsgrad_ef_update(g_next, b.m, b.e_u, b.v, b.vhat, b.x, idx_f, delta_f, k, w.beta1, w.beta2, w.lr)
            o.tail(st["e"], st["x"], idx, delta, w.lr)
            mask = np.zeros(w.d, np.uint8)
            mask[idx] = 1
            assert np.array_equal(host(b.x), st["x"]), t


@pytest.mark.parametrize("d,n,r,c,k", SHAPES)
def test_amsgrad_ef_update_pa_bit_exact(sams, fused, d, n, r, c, k):
    rng = np.random.default_rng(d + 7)
    o = Oracle("f32")
    b1, b2, lr = 0.9, 0.999, 1e-3
    f = lambda *s: (rng.standard_normal(s) * 10.0 ** rng.uniform(-4, 0, s)).astype(np.float32)
    g1, g2, m, e, x = f(n, d), f(n, d), f(n, d), f(n, d), f(d)
    vw = (10.0 ** rng.uniform(-8, -2, (n, d))).astype(np.float32)
    vhw = np.maximum(vw, (10.0 ** rng.uniform(-8, -2, (n, d))).astype(np.float32))
    idx = np.sort(rng.choice(d, k, replace=False)).astype(np.int32)
    delta = f(k)
    with sams.Context(d, n, r, c, k, inputs.hash_params(r)) as ctx:
        md, ed, vd, vhd, xd = dev(m), dev(e), dev(vw), dev(vhw), dev(x)
        ctx.amsgrad_ef_update_pa(dev(g1), md, ed, vd, vhd, xd, None, None, 0, b1, b2, lr)
        o.head_pa(g1, m, e, vw, vhw, b1, b2)
        for got, want in ((md, m), (ed, e), (vd, vw), (vhd, vhw), (xd, x)):
            assert np.array_equal(host(got), want)
        ctx.amsgrad_ef_update_pa(dev(g2), md, ed, vd, vhd, xd, dev(idx), dev(delta), k, b1, b2, lr, 1.25)
        o.tail(e, x, idx, delta, lr)
        o.head_pa(g2, m, e, vw, vhw, b1, b2, rho=1.25)
        for got, want in ((md, m), (ed, e), (vd, vw), (vhd, vhw), (xd, x)):
            assert np.array_equal(host(got), want)
        if ctx.sketch_mode == 2:                      # a fused head has left the sorted copy of e_u behind: use it
            S = torch.empty((n, r, c), device="cuda")
            ctx.sketch_accumulate(ed, S)
            hp = inputs.hash_params(r)
            assert np.array_equal(host(S), np.stack([o.sketch(e[i], hp, c) for i in range(n)]))
        ctx.amsgrad_ef_update_pa(None, md, ed, vd, vhd, xd, dev(idx), dev(delta), k, b1, b2, lr)
        o.tail(e, x, idx, delta, lr)
        assert np.array_equal(host(ed), e) and np.array_equal(host(xd), x)


@pytest.mark.parametrize("wl,d", [("C2", 300_000), ("P1", 400_000), ("P2b", 60_000)])
def test_chained_parameter_averaging_steps_follow_the_oracle(sams, fused, wl, d):
    """Alg. 1 end to end: per-worker second moments, plain unsketch operator, unscaled second round."""
    w = inputs.WORKLOADS[wl].scaled(d) if d != inputs.WORKLOADS[wl].d else inputs.WORKLOADS[wl]
    gs = inputs.GradientStream(w, device="cuda")
    hp = inputs.hash_params(w.r, seed=w.seed)
    o = Oracle("f32")
    steps = 4
    with sams.Context(w.d, w.n, w.r, w.c, w.k, hp) as ctx:
        b = sams.Buffers(w.d, w.n, w.r, w.c, w.k, w.eps, gs.x1())
        vw = torch.full((w.n, w.d), w.eps, device="cuda")
        vhw = torch.full((w.n, w.d), w.eps, device="cuda")
        st = dict(m=np.zeros((w.n, w.d), np.float32), e=np.zeros((w.n, w.d), np.float32),
                  vw=np.full((w.n, w.d), w.eps, np.float32), vhw=np.full((w.n, w.d), w.eps, np.float32),
                  x=host(b.x).copy())
        G = [gs.step(t) for t in range(steps)]
        ctx.amsgrad_ef_update_pa(G[0], b.m, b.e_u, vw, vhw, b.x, None, None, 0, w.beta1, w.beta2, w.lr)
        for t in range(steps):
            o.head_pa(host(G[t]), st["m"], st["e"], st["vw"], st["vhw"], w.beta1, w.beta2)
            assert np.array_equal(host(b.e_u), st["e"]) and np.array_equal(host(vhw), st["vhw"]), t
            ctx.sketch_accumulate(b.e_u, b.S_workers)
            ctx.sketch_reduce(b.S_workers, b.S_mean)
            ctx.unsketch_topk(b.S_mean, None, b.idx, None)
            ctx.gather_topk(b.e_u, None, b.idx, b.U_workers, b.delta)
            est = o.unsketch(host(b.S_mean), None, w.d, hp)
            idx = o.topk(est, w.k)
            assert np.array_equal(host(b.idx), idx), t
            _, delta = o.gather(st["e"], None, idx)
            assert np.array_equal(host(b.delta), delta), t
            g_next = G[t + 1] if t + 1 < steps else None
            ctx.amsgrad_ef_update_pa(g_next, b.m, b.e_u, vw, vhw, b.x, b.idx, b.delta, w.k, w.beta1, w.beta2, w.lr)
            o.tail(st["e"], st["x"], idx, delta, w.lr)
            assert np.array_equal(host(b.x), st["x"]), t


def gpu_state(b):
    return dict(m=host(b.m).copy(), e=host(b.e_u).copy(), v=host(b.v).copy(), vhat=host(b.vhat).copy(),
                x=host(b.x).copy())


def near_threshold(est, k, idx_a, idx_b):
    """Indices on which two index sets differ must have |est| within TOL of the k-th largest |est|."""
    mag = np.abs(est.astype(np.float64))
    tau = np.sort(mag)[-k]
    diff = np.setxor1d(idx_a, idx_b)
    return diff, bool(np.all(np.abs(mag[diff] - tau) <= TOL * tau))


CHAIN_WORKLOADS = [("C1", 65_536, 10), ("C2", 400_000, 6), ("C3", 300_000, 5), ("C4", 600_000, 5), ("C5", 500_000, 3),
                   ("P1", 300_000, 3), ("P2a", 60_000, 4), ("P2b", 60_000, 3)]


def chain_cases():
    """A covering set instead of the full product: the default launch configuration runs every workload, every other
    configuration runs two of them (dealt round-robin, so that every workload meets five or six configurations)."""
    cases = [("default", *wl) for wl in CHAIN_WORKLOADS]
    others = [name for name in PATHS if name != "default"]
    for q, name in enumerate(others):
        for z in range(2):
            cases.append((name, *CHAIN_WORKLOADS[(2 * q + z) % len(CHAIN_WORKLOADS)]))
    return cases


@pytest.mark.parametrize("path_name,wl,d,steps", chain_cases())
def test_chained_steps_follow_the_oracle(sams, path_name, wl, d, steps):
    """Free-running GPU run; at every step the oracle is restarted from the GPU's previous state, so
    each step is compared on real evolving state (bitmap of I_{t-1}, error feedback, vhat)."""
    for key, val in PATHS[path_name].items():
        sams.sams_configure(key, val)
    try:
        w = inputs.WORKLOADS[wl].scaled(d)
        run_chain(sams, w, steps, lambda t: w.lr)
    finally:
        for key, val in PATHS["default"].items():
            sams.sams_configure(key, val)


@pytest.mark.parametrize("wl,d,steps", [("C1", 65_536, 8), ("P2a", 60_000, 5), ("C4", 300_000, 4)])
def test_chained_steps_with_a_decaying_step_size(sams, wl, d, steps):
    """alpha_t = alpha / sqrt(t): the error feedback enters with the ratio alpha_{t-1} / alpha_t != 1
    (worker line of Alg. 2) and x moves by alpha_t Delta_t."""
    w = inputs.WORKLOADS[wl].scaled(d)
    run_chain(sams, w, steps, lambda t: w.lr / np.sqrt(t))


def run_chain(sams, w, steps, alpha):
    """alpha(t) = step size of iteration t = 1, 2, ..."""
    gs = inputs.GradientStream(w, device="cuda")
    hp = inputs.hash_params(w.r, seed=w.seed)
    o = Oracle("f32")
    with sams.Context(w.d, w.n, w.r, w.c, w.k, hp) as ctx:
        b = sams.Buffers(w.d, w.n, w.r, w.c, w.k, w.eps, gs.x1())
        G = [gs.step(t) for t in range(steps)]
        prev_mask = np.zeros(w.d, np.uint8)
        st = dict(m=np.zeros((w.n, w.d), np.float32), e=np.zeros((w.n, w.d), np.float32),
                  v=np.full(w.d, w.eps, np.float32), vhat=np.full(w.d, w.eps, np.float32), x=host(b.x).copy())
        ctx.amsgrad_ef_update(G[0], b.m, b.e_u, b.v, b.vhat, b.x, None, None, 0, w.beta1, w.beta2, alpha(1))
        n_diff = 0
        for t in range(steps):                                        # iteration t + 1 of the paper
            # oracle: head of this iteration from the state the GPU had before its head
            rho = np.float32(alpha(t) / alpha(t + 1)) if t else np.float32(1.0)
            o.head(host(G[t]), st["m"], st["e"], st["v"], st["vhat"], prev_mask if t else None, w.beta1, w.beta2,
                   rho=float(rho))
            got = gpu_state(b)
            for key in ("m", "e", "v", "vhat", "x"):
                assert np.array_equal(got[key], st[key]), (t, key)
            u = st["e"]
            # stages 1-4 on the GPU
            ctx.sketch_accumulate(b.e_u, b.S_workers)
            ctx.sketch_reduce(b.S_workers, b.S_mean)
            ctx.unsketch_topk(b.S_mean, b.vhat, b.idx, None)
            ctx.gather_topk(b.e_u, b.vhat, b.idx, b.U_workers, b.delta)
            S_w = host(b.S_workers)
            want64 = np.stack([Oracle("f64").sketch(u[i].astype(np.float64), hp, w.c) for i in range(w.n)])
            assert np.all(np.abs(S_w - want64) <= TOL * abs_mass(u, hp, w.c) + 1e-37), t
            S_mean = host(b.S_mean)
            assert np.array_equal(S_mean, o.sketch_mean(S_w)), t
            est = o.unsketch(S_mean, st["vhat"], w.d, hp)         # from the GPU's table: must be bit-exact
            idx = o.topk(est, w.k)
            idx_g = host(b.idx)
            assert np.array_equal(idx_g, idx), t
            # against the oracle's own table the set may differ only at the threshold
            S32 = o.sketch_mean(np.stack([o.sketch(u[i], hp, w.c) for i in range(w.n)]))
            est_o = o.unsketch(S32, st["vhat"], w.d, hp)
            diff, ok = near_threshold(est_o, w.k, o.topk(est_o, w.k), idx_g)
            assert ok, (t, diff[:10])
            n_diff += len(diff)
            U_w, delta = o.gather(u, st["vhat"], idx)
            assert np.array_equal(host(b.U_workers), U_w) and np.array_equal(host(b.delta), delta), t
            # tail of t (+ head of t+1) on the GPU; the oracle's tail here, its head at the loop top
            g_next = G[t + 1] if t + 1 < steps else None
            lr_t = float(np.float32(alpha(t + 1)))
            ctx.amsgrad_ef_update(g_next, b.m, b.e_u, b.v, b.vhat, b.x, b.idx, b.delta, w.k, w.beta1, w.beta2, lr_t,
                                  ef_ratio=float(np.float32(alpha(t + 1) / alpha(t + 2))))
            o.tail(st["e"], st["x"], idx, delta, lr_t)
            prev_mask = np.zeros(w.d, np.uint8)
            prev_mask[idx] = 1
        got = gpu_state(b)
        for key in ("m", "e", "v", "vhat", "x"):
            assert np.array_equal(got[key], st[key]), ("final", key)
        print(f"{w.name}: {steps} steps, index-set differences vs the oracle's own tables: {n_diff}")


def test_exact_recovery_chain_is_bit_exact_end_to_end(sams):
    """c >= d with identity bucket hashes: one term per bucket, so even the tables are order-free and a
    free-running GPU run must equal a free-running oracle run bit for bit."""
    w = inputs.WORKLOADS["C4"].scaled(50_000, c=50_001, k=500, n=4)
    gs = inputs.GradientStream(w, device="cuda")
    hp = inputs.identity_hash_params(w.r, seed=2)
    o = Oracle("f32")
    st = o.init_state(host(gs.x1()), w.n, w.eps)
    with sams.Context(w.d, w.n, w.r, w.c, w.k, hp) as ctx:
        b = sams.Buffers(w.d, w.n, w.r, w.c, w.k, w.eps, gs.x1())
        T = 6
        G = [gs.step(t) for t in range(T)]
        for t in range(T):
            sams.run_step(ctx, b, w.beta1, w.beta2, w.lr, g_next=G[t + 1] if t + 1 < T else None,
                          first=(t == 0), g_first=G[0])
            out = o.step(host(G[t]), st, hp, w.c, w.k, w.beta1, w.beta2, w.lr)
            assert np.array_equal(host(b.idx), out["idx"]), t
            assert np.array_equal(host(b.delta), out["delta"]), t
            assert np.array_equal(host(b.x), st["x"]), t
        assert np.array_equal(host(b.e_u), st["e"])


@pytest.mark.parametrize("fuse", [1, 2])
def test_resketch_after_recovery_does_not_trust_a_stale_staged_copy(sams, fuse):
    """A fused head leaves the sorted copy of e_u in the staging buffer and the next sketch_accumulate(e_u) uses it.
    The recovery of stage 3 works through the same buffer, so a second sketch_accumulate of the same e_u after
    unsketch_topk / unsketch_estimates must run both passes again: its tables equal the sequential sum bit for bit."""
    d, n, r, c, k = 70_000, 3, 5, 9_001, 300
    rng = np.random.default_rng(17)
    hp = inputs.hash_params(r, seed=4)
    o = Oracle("f32")
    f = lambda *s: (rng.standard_normal(s) * 10.0 ** rng.uniform(-4, 0, s)).astype(np.float32)
    g, m, e, x = f(n, d), f(n, d), f(n, d), f(d)
    v = np.full(d, 1e-8, np.float32)
    vhat = v.copy()
    for key, val in dict(PATHS["default"], fuse_head=fuse, sketch_path=2, tile_log2=10, win_log2=9, chunk_log2=9,
                         acc_threads=256).items():
        sams.sams_configure(key, val)
    try:
        with sams.Context(d, n, r, c, k, hp) as ctx:
            md, ed, vd, vhd, xd = dev(m), dev(e), dev(v), dev(vhat), dev(x)
            ctx.amsgrad_ef_update(dev(g), md, ed, vd, vhd, xd, None, None, 0, 0.9, 0.99, 1e-3)
            o.head(g, m, e, v, vhat, None, 0.9, 0.99)
            want = np.stack([o.sketch(e[i], hp, c) for i in range(n)])
            S = torch.empty((n, r, c), device="cuda")
            Sm = torch.empty((r, c), device="cuda")
            idx = torch.empty(k, device="cuda", dtype=torch.int32)
            est = torch.empty(d, device="cuda")
            ctx.sketch_accumulate(ed, S)                      # consumes the staged copy
            assert np.array_equal(host(S), want)
            ctx.sketch_reduce(S, Sm)
            ctx.unsketch_topk(Sm, vhd, idx, None)             # the recovery overwrites the staging buffer
            S.fill_(3.0)
            ctx.sketch_accumulate(ed, S)
            assert np.array_equal(host(S), want)
            ctx.unsketch_estimates(Sm, vhd, est)
            S.fill_(5.0)
            ctx.sketch_accumulate(ed, S)
            assert np.array_equal(host(S), want)
    finally:
        for key, val in PATHS["default"].items():
            sams.sams_configure(key, val)


def test_a_context_keeps_the_tunables_it_was_created_with(sams):
    """sams_create copies the tunables; reconfiguring afterwards changes neither the kernels an existing context
    launches (counted through the per-kernel timing) nor its results."""
    d, n, r, c, k = 50_000, 3, 5, 5_000, 200
    rng = np.random.default_rng(23)
    hp = inputs.hash_params(r, seed=6)
    f = lambda *s: (rng.standard_normal(s) * 10.0 ** rng.uniform(-4, 0, s)).astype(np.float32)
    g, m, e, x = f(n, d), f(n, d), f(n, d), f(d)
    v = np.full(d, 1e-8, np.float32)

    def one_run(ctx):
        md, ed, vd, vhd, xd = dev(m), dev(e), dev(v), dev(v.copy()), dev(x)
        S = torch.empty((n, r, c), device="cuda")
        Sm = torch.empty((r, c), device="cuda")
        idx = torch.empty(k, device="cuda", dtype=torch.int32)
        ctx.sams_profile_enable(True)
        ctx.amsgrad_ef_update(dev(g), md, ed, vd, vhd, xd, None, None, 0, 0.9, 0.99, 1e-3)
        ctx.sketch_accumulate(ed, S)
        ctx.sketch_reduce(S, Sm)
        ctx.unsketch_topk(Sm, vhd, idx, None)
        ctx.sams_profile_enable(False)
        launches = {kn: cnt for kn, (_, cnt) in ctx.sams_profile_read().items()}
        return launches, host(S).copy(), host(idx).copy(), host(ed).copy()

    first = dict(PATHS["default"], fuse_head=2, sketch_path=2, scatter_threads=512, estimate_path=2)
    other = dict(PATHS["default"], fuse_head=0, sketch_path=1, scatter_threads=256, estimate_path=1, tile_log2=9,
                 win_log2=8, chunk_log2=8, acc_threads=256)
    try:
        for key, val in first.items():
            sams.sams_configure(key, val)
        with sams.Context(d, n, r, c, k, hp) as ctx:
            before = one_run(ctx)
            assert before[0].get("k_head_scatter") == 1 and "k_head" not in before[0]
            for key, val in other.items():
                sams.sams_configure(key, val)
            after = one_run(ctx)
            assert after[0] == before[0]
            assert all(np.array_equal(a, b) for a, b in zip(after[1:], before[1:]))
            with sams.Context(d, n, r, c, k, hp) as ctx2:            # a new context does follow the new settings
                fresh = one_run(ctx2)
                assert fresh[0].get("k_head") == 1 and "k_head_scatter" not in fresh[0]
                assert fresh[0].get("k_sketch_atomic") == 1 and fresh[0].get("k_estimate") == 1
                assert np.array_equal(fresh[3], before[3])      # the head is exact on every path
    finally:
        for key, val in PATHS["default"].items():
            sams.sams_configure(key, val)


def test_staging_mapped_from_scattered_chunks_gives_the_same_tables_and_returns_its_memory(sams):
    """"stage_spread": a staging buffer of 2 GiB or more mapped from 1 GiB physical chunks picked all over the free device
    memory.  Same tables as with one allocation (which the full-size tests hold against the oracle), bit for bit, for a
    fused head and for a plain sketch_accumulate; destroying the context gives every chunk back."""
    d, n, r, c, k = 13_000_000, 8, 5, 262_144, 1000
    hp = inputs.hash_params(r, seed=5)
    gen = torch.Generator(device="cuda").manual_seed(11)
    g = torch.randn(n, d, device="cuda", generator=gen) * 1e-2
    tables = {}
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free_before = torch.cuda.mem_get_info()[0]
    try:
        for spread in (0, 1):
            for key, val in dict(PATHS["default"], fuse_head=2, sketch_path=2, stage_spread=spread).items():
                sams.sams_configure(key, val)
            with sams.Context(d, n, r, c, k, hp) as ctx:
                assert ctx.scratch_bytes > (2 << 30)
                b = sams.Buffers(d, n, r, c, k, 1e-8, torch.zeros(d, device="cuda"))
                ctx.amsgrad_ef_update(g, b.m, b.e_u, b.v, b.vhat, b.x, None, None, 0, 0.9, 0.99, 1e-3)
                ctx.sketch_accumulate(b.e_u, b.S_workers)                   # from the copy the head staged
                first = host(b.S_workers).copy()
                est = torch.empty(d, device="cuda")
                ctx.sketch_reduce(b.S_workers, b.S_mean)
                ctx.unsketch_estimates(b.S_mean, b.vhat, est)               # the recovery works through the staging buffer
                ctx.sketch_accumulate(b.e_u, b.S_workers)                   # both passes again
                assert np.array_equal(host(b.S_workers), first)
                tables[spread] = (first, host(est).copy())
                del b, est
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
            assert abs(torch.cuda.mem_get_info()[0] - free_before) <= (64 << 20), spread
        assert np.array_equal(tables[0][0], tables[1][0]) and np.array_equal(tables[0][1], tables[1][1])
    finally:
        for key, val in dict(PATHS["default"], stage_spread=0).items():
            sams.sams_configure(key, val)


def test_invalid_arguments_are_rejected_without_launching(sams):
    hp = inputs.hash_params(5)
    bad = [dict(d=0), dict(k=0), dict(k=1001), dict(r=17), dict(c=0), dict(n=0), dict(d=inputs.P31)]
    for kw in bad:
        args = dict(d=1000, n=2, r=5, c=64, k=10)
        args.update(kw)
        hpp = inputs.hash_params(args["r"])
        with pytest.raises(sams.SamsError) as ei:
            sams.Context(args["d"], args["n"], args["r"], args["c"], args["k"], hpp)
        assert ei.value.code == sams.SAMS_EINVAL
    hp0 = hp.copy()
    hp0[2, 0] = 0                                           # a = 0 is not in the family
    with pytest.raises(sams.SamsError):
        sams.Context(1000, 2, 5, 64, 10, hp0)
    with sams.Context(1000, 2, 5, 64, 10, hp) as ctx:
        u = torch.zeros((2, 1000), device="cuda")
        S = torch.zeros((2, 5, 64), device="cuda")
        lib = sams.load()
        assert lib.sketch_accumulate(ctx._h, None, S.data_ptr()) == sams.SAMS_EINVAL
        assert lib.sketch_accumulate(ctx._h, u.data_ptr() + 4, S.data_ptr()) == sams.SAMS_EINVAL   # misaligned
        assert lib.amsgrad_ef_update(ctx._h, None, u.data_ptr(), u.data_ptr(), S.data_ptr(), S.data_ptr(),
                                     S.data_ptr(), None, None, 5, 0.9, 0.99, 1e-3, 1.0) == sams.SAMS_EINVAL
        assert ctx.scratch_bytes >= 4 * 1000


def test_precondition_device_memory_leaves_nothing_behind(sams):
    free0, _ = torch.cuda.mem_get_info()
    held = sams.sams_precondition_device_memory(0.05)              # a twentieth of the free memory, in 1 GiB blocks
    free1, _ = torch.cuda.mem_get_info()
    assert held >= 1 and abs(free1 - free0) < (64 << 20)
    with pytest.raises(sams.SamsError):
        sams.sams_precondition_device_memory(0.0)


def test_step_on_a_side_stream_and_as_a_replayed_hip_graph(sams):
    """No entry point synchronises the host or allocates, so a whole step can be captured once into a HIP graph on
    the context's stream and replayed.  Every replay (with eager work and synchronisations in between) must give
    exactly what the same calls give when issued eagerly."""
    w = inputs.WORKLOADS["C1"]
    gs = inputs.GradientStream(w, device="cuda")
    hp = inputs.hash_params(w.r, seed=w.seed)
    G = [gs.step(t) for t in range(6)]
    side = torch.cuda.Stream()
    for key, val in PATHS["binned-unroll2"].items():       # the order-preserving path: results are reproducible
        sams.sams_configure(key, val)

    def fresh():
        with torch.cuda.stream(side):
            ctx = sams.Context(w.d, w.n, w.r, w.c, w.k, hp, stream=side)
            b = sams.Buffers(w.d, w.n, w.r, w.c, w.k, w.eps, gs.x1())
            ctx.amsgrad_ef_update(G[0], b.m, b.e_u, b.v, b.vhat, b.x, None, None, 0, w.beta1, w.beta2, w.lr)
        return ctx, b

    def step(ctx, b, g_next):
        ctx.sketch_accumulate(b.e_u, b.S_workers)
        ctx.sketch_reduce(b.S_workers, b.S_mean)
        ctx.unsketch_topk(b.S_mean, b.vhat, b.idx, None)
        ctx.gather_topk(b.e_u, b.vhat, b.idx, b.U_workers, b.delta)
        ctx.amsgrad_ef_update(g_next, b.m, b.e_u, b.v, b.vhat, b.x, b.idx, b.delta, w.k, w.beta1, w.beta2, w.lr)

    # eager reference on the side stream
    ctx_e, be = fresh()
    ref = []
    with torch.cuda.stream(side):
        for t in range(5):
            step(ctx_e, be, G[t + 1])
            side.synchronize()
            ref.append((host(be.x).copy(), host(be.idx).copy(), host(be.S_mean).copy()))
    ctx_e.close()
    # graph: the gradient of the next iteration is read from a fixed buffer that is refilled between replays
    ctx_g, bg = fresh()
    g_in = torch.empty_like(G[0])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        g_in.copy_(G[1])
        step(ctx_g, bg, g_in)                      # one eager step first (iteration 1)
        side.synchronize()
        assert np.array_equal(host(bg.x), ref[0][0])
        g_in.copy_(G[2])
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(ctx_g, bg, g_in)
        for t in range(1, 5):                      # capture does not execute: replay iterations 2..5
            g_in.copy_(G[t + 1])
            graph.replay()
            side.synchronize()
            _ = torch.zeros(1000, device="cuda").sum().item()     # unrelated eager work between replays
            assert np.array_equal(host(bg.idx), ref[t][1]), t
            assert np.array_equal(host(bg.x), ref[t][0]), t
            assert np.array_equal(host(bg.S_mean), ref[t][2]), t
    ctx_g.close()
    for key, val in PATHS["default"].items():
        sams.sams_configure(key, val)


def test_kernel_timing_counts_launches_and_changes_no_result(sams):
    """The optional per-kernel timing: every launch of the window is counted once, a filter restricts it to one
    kernel, durations are positive, and the outputs are the same bits as without it."""
    d, n, r, c, k = 100_003, 3, 5, 1_000, 777
    rng = np.random.default_rng(5)
    hp = inputs.hash_params(r, seed=5)
    u = dev(rng.standard_normal((n, d)).astype(np.float32))
    with sams.Context(d, n, r, c, k, hp) as ctx:
        S = torch.empty((n, r, c), device="cuda")
        S_mean = torch.empty((r, c), device="cuda")
        idx = torch.empty(k, device="cuda", dtype=torch.int32)

        def run():
            ctx.sketch_accumulate(u, S)
            ctx.sketch_reduce(S, S_mean)
            ctx.unsketch_topk(S_mean, None, idx, None)
            return host(S).copy(), host(S_mean).copy(), host(idx).copy()

        plain = run()
        ctx.sams_profile_enable(True)
        timed = [run() for _ in range(3)]
        ctx.sams_profile_enable(False)
        prof = ctx.sams_profile_read()
        for got in timed:
            assert all(np.array_equal(a, b) for a, b in zip(got, plain))
        assert prof["k_reduce"][1] == 3 and prof["k_sel_hist"][1] == 9 and prof["k_sel_write"][1] == 3
        assert all(ms > 0.0 for ms, _ in prof.values())
        ctx.sams_profile_only("k_reduce")
        ctx.sams_profile_enable(True)
        run()
        run()
        ctx.sams_profile_enable(False)
        only = ctx.sams_profile_read()
        assert set(only) == {"k_reduce"} and only["k_reduce"][1] == 2
        ctx.sams_profile_only(None)
        ctx.sams_profile_enable(True)
        run()
        ctx.sams_profile_enable(False)
        assert len(ctx.sams_profile_read()) > 3
        before = ctx.sams_profile_read()
        run()                                                        # switched off: nothing more is recorded
        assert ctx.sams_profile_read() == before
