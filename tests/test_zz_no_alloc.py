"""topk_refine_static (the entry point that allocates nothing: its scratch is a static device array inside the
library) against topk_refine, through the C ABI: two calls in a row on the shared scratch, the second with a
smaller input, each bit-exact against the existing entry point (and against the oracle's definition)."""
import numpy as np
import pytest
import torch

from oracle import Oracle
from paper_2210_07454_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sams():
    from paper_2210_07454_amd import sams as mod
    mod.load()
    return mod


def candidates(k_in, d, seed):
    rng = np.random.default_rng(seed)
    cand = np.sort(rng.choice(d, k_in, replace=False)).astype(np.int32)
    vals = (rng.integers(-40, 41, k_in) / 8.0).astype(np.float32)          # many ties, zeros of both signs
    vals[rng.integers(0, k_in, max(1, k_in // 8))] = -0.0
    return cand, vals


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


@pytest.mark.parametrize("sizes", [((400_000, 50_000), (90_000, 7_001)),       # several tiles, then fewer tiles
                                   ((300_001, 300_001), (1_000, 37)),           # k_out = k_in, then the one-workgroup path
                                   ((3_000, 1), (70_000, 69_999))])             # small first, larger second
def test_topk_refine_static_equals_topk_refine_on_two_calls_in_a_row(sams, sizes):
    d = 3_000_000
    free0, _ = torch.cuda.mem_get_info()
    for call, (k_in, k_out) in enumerate(sizes):
        cand, vals = candidates(k_in, d, seed=k_in + call)
        ci, vi = dev(cand), dev(vals)
        io_s = torch.full((k_out,), -1, device="cuda", dtype=torch.int32)
        do_s = torch.full((k_out,), 7.0, device="cuda")
        sams.topk_refine_static(ci, vi, k_out, io_s, do_s)
        io_c = torch.full((k_out,), -2, device="cuda", dtype=torch.int32)
        do_c = torch.full((k_out,), 9.0, device="cuda")
        with sams.Context(d, 2, 3, 1000, k_in, inputs.hash_params(3)) as ctx:
            ctx.topk_refine(ci, vi, k_out, io_c, do_c)
            got_c = host(io_c).copy(), host(do_c).copy()
        got_s = host(io_s), host(do_s)
        assert np.array_equal(got_s[0], got_c[0]) and np.array_equal(got_s[1], got_c[1]), (call, k_in, k_out)
        idx, delta = Oracle("f32").refine(cand, vals, k_out)
        assert np.array_equal(got_s[0], idx) and np.array_equal(got_s[1], delta), (call, k_in, k_out)


def test_topk_refine_static_rejects_sizes_beyond_its_scratch_and_bad_pointers(sams):
    lib = sams.load()
    kmax = int(lib.topk_refine_static_max_candidates())
    assert kmax == 8_388_608
    a = torch.zeros(64, device="cuda", dtype=torch.int32)
    f = torch.zeros(64, device="cuda")
    p = lambda t: t.data_ptr()
    assert lib.topk_refine_static(p(a), p(f), kmax + 1, 1, p(a), p(f), None) == sams.SAMS_EINVAL
    assert lib.topk_refine_static(p(a), p(f), 64, 65, p(a), p(f), None) == sams.SAMS_EINVAL
    assert lib.topk_refine_static(p(a), p(f), 0, 0, p(a), p(f), None) == sams.SAMS_EINVAL
    assert lib.topk_refine_static(None, p(f), 64, 1, p(a), p(f), None) == sams.SAMS_EINVAL
    assert lib.topk_refine_static(p(a) + 4, p(f), 32, 1, p(a), p(f), None) == sams.SAMS_EINVAL


def test_topk_refine_static_allocates_no_device_memory(sams):
    k_in, k_out = 200_000, 10_000
    cand, vals = candidates(k_in, 1_000_000, seed=1)
    ci, vi = dev(cand), dev(vals)
    io = torch.empty(k_out, device="cuda", dtype=torch.int32)
    do = torch.empty(k_out, device="cuda")
    sams.topk_refine_static(ci, vi, k_out, io, do)            # the address look-up, if no context came first
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        sams.topk_refine_static(ci, vi, k_out, io, do)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
    idx, delta = Oracle("f32").refine(cand, vals, k_out)
    assert np.array_equal(host(io), idx) and np.array_equal(host(do), delta)
