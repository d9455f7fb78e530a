"""The C-ABI library loads and exports every symbol include/sams.h declares (no GPU work here)."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch  # noqa: F401  (loads the HIP runtime the library binds to)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sams.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"^\s*(?:int|int64_t|const char \*)\s*(\w+)\s*\(", text, flags=re.M)


def test_header_declares_the_five_stage_calls():
    names = declared_functions()
    for want in ("sketch_accumulate", "sketch_reduce", "unsketch_topk", "gather_topk", "amsgrad_ef_update",
                 "sams_create", "sams_destroy"):
        assert want in names


def test_library_exports_every_declared_symbol():
    from paper_2210_07454_amd import sams
    lib = sams.load()
    names = declared_functions()
    assert sorted(names) == sorted(sams.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name


def test_argument_validation_needs_no_gpu():
    from paper_2210_07454_amd import sams
    lib = sams.load()
    h = ctypes.c_void_p()
    hp = np.ones((5, 4), dtype=np.uint32)
    hpp = hp.ctypes.data_as(ctypes.c_void_p)
    assert lib.sams_create(ctypes.byref(h), 0, 1, 5, 8, 1, hpp, None) == sams.SAMS_EINVAL        # d < 1
    assert lib.sams_create(ctypes.byref(h), 100, 1, 17, 8, 1, hpp, None) == sams.SAMS_EINVAL     # r too large
    assert lib.sams_create(ctypes.byref(h), 100, 1, 5, 8, 101, hpp, None) == sams.SAMS_EINVAL    # k > d
    assert lib.sams_create(ctypes.byref(h), 100, 1, 5, 8, 1, None, None) == sams.SAMS_EINVAL     # no hashes
    assert lib.sams_create(ctypes.byref(h), 2**31 - 1, 1, 5, 8, 1, hpp, None) == sams.SAMS_EINVAL
    hp[3, 0] = 0
    assert lib.sams_create(ctypes.byref(h), 100, 1, 5, 8, 1, hpp, None) == sams.SAMS_EINVAL      # a = 0
    assert h.value is None
    assert lib.sams_destroy(None) == sams.SAMS_OK
    assert lib.sketch_accumulate(None, None, None) == sams.SAMS_EINVAL


def test_binding_refuses_to_run_without_a_gpu():
    from paper_2210_07454_amd import sams
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        sams.Context(100, 1, 5, 8, 1, np.ones((5, 4), dtype=np.uint32))


def test_configure_rejects_unknown_keys_and_bad_values_without_a_gpu():
    from paper_2210_07454_amd import sams
    lib = sams.load()
    ok = [(b"tile_log2", 14), (b"tile_log2", 0), (b"win_log2", 15), (b"win_log2", 0), (b"chunk_log2", 0), (b"acc_threads", 0),
          (b"run_pad", 32), (b"run_pad", 16), (b"scatter_threads", 1024), (b"sketch_path", 0), (b"estimate_path", 2), (b"estimate_path", 0),
          (b"fuse_head", 0), (b"fuse_median", 1), (b"stage_rows", 0), (b"stage_spread", 1), (b"stage_spread", 0)]
    bad = [(b"tile_log2", 15), (b"tile_log2", 5), (b"win_log2", 16), (b"win_log2", 3), (b"chunk_log2", 12),
           (b"acc_threads", 384), (b"run_pad", 5), (b"scatter_threads", 100), (b"sketch_path", 4),
           (b"estimate_path", -1), (b"estimate_path", 3), (b"stage_spread", 2), (b"fuse_head", 3), (b"stage_rows", 17), (b"no_such_key", 1)]
    for key, val in bad:
        assert lib.sams_configure(key, val) == sams.SAMS_EINVAL, (key, val)
    assert lib.sams_configure(None, 0) == sams.SAMS_EINVAL
    for key, val in ok:                      # leaves the defaults in place
        assert lib.sams_configure(key, val) == sams.SAMS_OK, (key, val)
    assert lib.sams_sketch_mode(None) == -1
    assert lib.sams_precondition_device_memory(0.0) == sams.SAMS_EINVAL       # refused before any device call
    assert lib.sams_precondition_device_memory(1.5) == sams.SAMS_EINVAL
    assert lib.sams_profile_kernels() > 10
    names = {lib.sams_profile_name(q).decode() for q in range(lib.sams_profile_kernels())}
    assert {"k_head_scatter", "k_bin_accumulate", "k_sel_hist"} <= names


def test_bench_refuses_more_than_one_gpu():
    """Every box of this build has one GPU: bench.py says so instead of starting ranks."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], cwd=root, capture_output=True,
                       text=True, timeout=120)
    assert p.returncode != 0 and "ONE GPU" in p.stderr
