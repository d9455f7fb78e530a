"""Thin ctypes binding over the C ABI of ``include/sams.h`` (argument marshalling only).

Every function has the name and argument order of its C entry point and takes torch
CUDA tensors (device memory and streams are all PyTorch is used for).  There is no
fallback: if the HIP library has not been built, or no GPU is present, the calls raise.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsams.so")

SAMS_OK, SAMS_EINVAL, SAMS_ENOMEM, SAMS_EHIP = 0, -1, -2, -3
_ERR = {SAMS_EINVAL: "SAMS_EINVAL (bad argument)", SAMS_ENOMEM: "SAMS_ENOMEM (scratch allocation failed)",
        SAMS_EHIP: "SAMS_EHIP (HIP runtime error)"}

# every symbol include/sams.h declares
EXPORTS = ["sams_create", "sams_destroy", "sams_scratch_bytes", "sams_precondition_device_memory", "sams_last_hip_error", "sams_hash_dump",
           "sams_configure", "sams_sketch_mode", "sams_accumulate_variant", "sams_record_rows", "sams_profile_kernels", "sams_profile_name", "sams_profile_enable", "sams_profile_only", "sams_profile_read",
           "sketch_accumulate", "sketch_reduce", "unsketch_topk", "unsketch_estimates", "gather_topk", "topk_refine",
           "amsgrad_ef_update", "amsgrad_ef_update_pa", "topk_refine_static", "topk_refine_static_max_candidates"]

_lib = None


class SamsError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        extra = ""
        if code == SAMS_EHIP and _lib is not None:
            extra = f" hipError={_lib.sams_last_hip_error()}"
        super().__init__(f"{where}: {_ERR.get(code, code)}{extra}")


def load() -> ctypes.CDLL:
    """Load libsams.so (built by ``paper_2210_07454_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2210_07454_amd.build`")
    # torch has already loaded its HIP runtime (soname libamdhip64.so.7); the library binds to that one
    lib = ctypes.CDLL(LIB_PATH, mode=ctypes.RTLD_GLOBAL)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.sams_create.argtypes = [ctypes.POINTER(vp), i64, i32, i32, i64, i64, vp, vp]
    lib.sams_destroy.argtypes = [vp]
    lib.sams_scratch_bytes.argtypes = [vp]
    lib.sams_scratch_bytes.restype = i64
    lib.sams_precondition_device_memory.argtypes = [ctypes.c_double]
    lib.sams_precondition_device_memory.restype = i64
    lib.sams_last_hip_error.argtypes = []
    lib.sams_hash_dump.argtypes = [vp, vp, vp]
    lib.sams_configure.argtypes = [ctypes.c_char_p, ctypes.c_int]
    lib.sams_sketch_mode.argtypes = [vp]
    lib.sams_accumulate_variant.argtypes = [vp]
    lib.sams_record_rows.argtypes = [vp]
    lib.sams_record_rows.restype = i64
    lib.sams_profile_kernels.argtypes = []
    lib.sams_profile_name.argtypes = [ctypes.c_int]
    lib.sams_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.sams_profile_only.argtypes = [vp, ctypes.c_int]
    lib.sams_profile_read.argtypes = [vp, vp, vp]
    lib.sketch_accumulate.argtypes = [vp, vp, vp]
    lib.sketch_reduce.argtypes = [vp, vp, vp]
    lib.unsketch_topk.argtypes = [vp, vp, vp, vp, vp]
    lib.unsketch_estimates.argtypes = [vp, vp, vp, vp]
    lib.gather_topk.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.topk_refine.argtypes = [vp, vp, vp, i64, vp, vp]
    lib.amsgrad_ef_update.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, f32, f32, f32, f32]
    lib.amsgrad_ef_update_pa.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, f32, f32, f32, f32]
    lib.topk_refine_static.argtypes = [vp, vp, i64, i64, vp, vp, vp]
    lib.topk_refine_static_max_candidates.argtypes = []
    lib.topk_refine_static_max_candidates.restype = i64
    for name in EXPORTS:
        if name not in ("sams_scratch_bytes", "sams_profile_name", "sams_precondition_device_memory",
                        "topk_refine_static_max_candidates", "sams_record_rows"):
            getattr(lib, name).restype = ctypes.c_int
    lib.sams_profile_name.restype = ctypes.c_char_p
    _lib = lib
    return lib


def sams_configure(key: str, value: int):
    _check(load().sams_configure(key.encode(), int(value)), f"sams_configure({key}={value})")


def sams_precondition_device_memory(fraction: float = 0.995) -> int:
    """Allocate-and-free pass over the free memory of the current device (see sams.h); returns the GiB held."""
    if not torch.cuda.is_available():
        raise RuntimeError("paper_2210_07454_amd needs a GPU: no CPU fallback exists")
    got = int(load().sams_precondition_device_memory(float(fraction)))
    if got < 0:
        raise SamsError(got, "sams_precondition_device_memory")
    return got


def _ptr(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _check(code, where):
    if code != SAMS_OK:
        raise SamsError(code, where)


def topk_refine_static(idx_in, delta_in, k_out, idx_out, delta_out, stream=None):
    """Context-free topk_refine on the library's static scratch (allocates nothing); see sams.h."""
    if not torch.cuda.is_available():
        raise RuntimeError("paper_2210_07454_amd needs a GPU: no CPU fallback exists")
    k_in = idx_in.numel()
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(load().topk_refine_static(
        _ptr(idx_in, torch.int32, (k_in,), "idx_in"), _ptr(delta_in, torch.float32, (k_in,), "delta_in"), int(k_in),
        int(k_out), _ptr(idx_out, torch.int32, (k_out,), "idx_out"), _ptr(delta_out, torch.float32, (k_out,), "delta_out"),
        ctypes.c_void_p(st.cuda_stream)), "topk_refine_static")


class Context:
    """Owns one ``sams_ctx``.  Work is enqueued on the torch stream that is current at creation."""

    def __init__(self, d: int, n: int, r: int, c: int, k: int, hash_params, stream=None):
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2210_07454_amd needs a GPU: no CPU fallback exists")
        lib = load()
        hp = np.ascontiguousarray(hash_params, dtype=np.uint32)
        if hp.shape != (r, 4):
            raise ValueError(f"hash_params: expected shape ({r}, 4)")
        self.d, self.n, self.r, self.c, self.k = d, n, r, c, k
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = ctypes.c_void_p()
        self._lib = lib
        code = lib.sams_create(ctypes.byref(self._h), d, n, r, c, k, hp.ctypes.data_as(ctypes.c_void_p),
                               ctypes.c_void_p(self.stream.cuda_stream))
        _check(code, "sams_create")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.sams_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    @property
    def scratch_bytes(self) -> int:
        return int(self._lib.sams_scratch_bytes(self._h))

    @property
    def sketch_mode(self) -> int:
        return int(self._lib.sams_sketch_mode(self._h))

    @property
    def accumulate_variant(self) -> int:
        return int(self._lib.sams_accumulate_variant(self._h))

    @property
    def record_rows(self) -> int:
        """Bit mask of the rows whose second pass reads chunk records (see sams.h)."""
        return int(self._lib.sams_record_rows(self._h))

    def sams_profile_enable(self, on: bool):
        _check(self._lib.sams_profile_enable(self._h, 1 if on else 0), "sams_profile_enable")

    def sams_profile_only(self, name=None):
        """Restrict the timing to the kernel called ``name`` (None: every kernel)."""
        nk = self._lib.sams_profile_kernels()
        names = [self._lib.sams_profile_name(q).decode() for q in range(nk)]
        _check(self._lib.sams_profile_only(self._h, -1 if name is None else names.index(name)), "sams_profile_only")

    def sams_profile_read(self):
        """{kernel name: (total milliseconds, launches)} since profiling was enabled."""
        nk = self._lib.sams_profile_kernels()
        ms = (ctypes.c_double * nk)()
        cnt = (ctypes.c_int64 * nk)()
        _check(self._lib.sams_profile_read(self._h, ms, cnt), "sams_profile_read")
        return {self._lib.sams_profile_name(q).decode(): (ms[q], cnt[q]) for q in range(nk) if cnt[q]}

    # ---- entry points, same names and argument order as the C ABI ----
    def sams_hash_dump(self, bucket, sign):
        _check(self._lib.sams_hash_dump(self._h, _ptr(bucket, torch.int32, (self.r, self.d), "bucket"),
                                        _ptr(sign, torch.int8, (self.r, self.d), "sign")), "sams_hash_dump")

    def sketch_accumulate(self, u, S_workers):
        _check(self._lib.sketch_accumulate(
            self._h, _ptr(u, torch.float32, (self.n, self.d), "u"),
            _ptr(S_workers, torch.float32, (self.n, self.r, self.c), "S_workers")), "sketch_accumulate")

    def sketch_reduce(self, S_workers, S_mean):
        _check(self._lib.sketch_reduce(
            self._h, _ptr(S_workers, torch.float32, (self.n, self.r, self.c), "S_workers"),
            _ptr(S_mean, torch.float32, (self.r, self.c), "S_mean")), "sketch_reduce")

    def unsketch_topk(self, S_mean, vhat, idx, est_sel=None):
        _check(self._lib.unsketch_topk(
            self._h, _ptr(S_mean, torch.float32, (self.r, self.c), "S_mean"),
            _ptr(vhat, torch.float32, (self.d,), "vhat"), _ptr(idx, torch.int32, (self.k,), "idx"),
            _ptr(est_sel, torch.float32, (self.k,), "est_sel")), "unsketch_topk")

    def unsketch_estimates(self, S_mean, vhat, est):
        _check(self._lib.unsketch_estimates(
            self._h, _ptr(S_mean, torch.float32, (self.r, self.c), "S_mean"),
            _ptr(vhat, torch.float32, (self.d,), "vhat"), _ptr(est, torch.float32, (self.d,), "est")),
            "unsketch_estimates")

    def gather_topk(self, u, vhat, idx, U_workers, delta):
        _check(self._lib.gather_topk(
            self._h, _ptr(u, torch.float32, (self.n, self.d), "u"), _ptr(vhat, torch.float32, (self.d,), "vhat"),
            _ptr(idx, torch.int32, (self.k,), "idx"), _ptr(U_workers, torch.float32, (self.n, self.k), "U_workers"),
            _ptr(delta, torch.float32, (self.k,), "delta")), "gather_topk")

    def topk_refine(self, idx_in, delta_in, k_out, idx_out, delta_out):
        _check(self._lib.topk_refine(
            self._h, _ptr(idx_in, torch.int32, (self.k,), "idx_in"), _ptr(delta_in, torch.float32, (self.k,), "delta_in"),
            int(k_out), _ptr(idx_out, torch.int32, (k_out,), "idx_out"),
            _ptr(delta_out, torch.float32, (k_out,), "delta_out")), "topk_refine")

    def amsgrad_ef_update(self, g_next, m, e_u, v, vhat, x, idx, delta, k_sel, beta1, beta2, lr, ef_ratio=1.0):
        nd = (self.n, self.d)
        if k_sel:
            if idx is None or delta is None or idx.numel() < k_sel or delta.numel() < k_sel:
                raise ValueError("idx/delta shorter than k_sel")
        _check(self._lib.amsgrad_ef_update(
            self._h, _ptr(g_next, torch.float32, nd, "g_next"), _ptr(m, torch.float32, nd, "m"),
            _ptr(e_u, torch.float32, nd, "e_u"), _ptr(v, torch.float32, (self.d,), "v"),
            _ptr(vhat, torch.float32, (self.d,), "vhat"), _ptr(x, torch.float32, (self.d,), "x"),
            _ptr(idx, torch.int32, None, "idx"), _ptr(delta, torch.float32, None, "delta"), int(k_sel),
            float(beta1), float(beta2), float(lr), float(ef_ratio)), "amsgrad_ef_update")


    def _update_pa(self, g_next, m, e_u, v_w, vhat_w, x, idx, delta, k_sel, beta1, beta2, lr, ef_ratio):
        nd = (self.n, self.d)
        _check(self._lib.amsgrad_ef_update_pa(
            self._h, _ptr(g_next, torch.float32, nd, "g_next"), _ptr(m, torch.float32, nd, "m"),
            _ptr(e_u, torch.float32, nd, "e_u"), _ptr(v_w, torch.float32, nd, "v_workers"),
            _ptr(vhat_w, torch.float32, nd, "vhat_workers"), _ptr(x, torch.float32, (self.d,), "x"),
            _ptr(idx, torch.int32, None, "idx"), _ptr(delta, torch.float32, None, "delta"), int(k_sel),
            float(beta1), float(beta2), float(lr), float(ef_ratio)), "amsgrad_ef_update_pa")

    def amsgrad_ef_update_pa(self, g_next, m, e_u, v_workers, vhat_workers, x, idx, delta, k_sel, beta1, beta2, lr,
                             ef_ratio=1.0):
        if k_sel and (idx is None or delta is None or idx.numel() < k_sel or delta.numel() < k_sel):
            raise ValueError("idx/delta shorter than k_sel")
        self._update_pa(g_next, m, e_u, v_workers, vhat_workers, x, idx, delta, k_sel, beta1, beta2, lr, ef_ratio)


class Buffers:
    """Caller-owned device buffers for a run (the library itself allocates none of these)."""

    def __init__(self, d, n, r, c, k, eps, x1, device="cuda"):
        f = dict(device=device, dtype=torch.float32)
        self.m = torch.zeros((n, d), **f)
        self.e_u = torch.zeros((n, d), **f)
        self.v = torch.full((d,), eps, **f)
        self.vhat = torch.full((d,), eps, **f)
        self.x = x1.to(device=device, dtype=torch.float32).clone()
        self.S_workers = torch.empty((n, r, c), **f)
        self.S_mean = torch.empty((r, c), **f)
        self.idx = torch.empty((k,), device=device, dtype=torch.int32)
        self.U_workers = torch.empty((n, k), **f)
        self.delta = torch.empty((k,), **f)


def run_step(ctx: Context, b: Buffers, beta1, beta2, lr, g_next=None, first=False, g_first=None,
             use_vhat=True):
    """The calling sequence of one iteration, in the order sams.h documents.

    ``first``: enqueue the head-only call for ``g_first`` before the five stages.
    After the stages, ``amsgrad_ef_update`` finishes the iteration and, if ``g_next`` is
    given, starts the next one.
    """
    if first:
        ctx.amsgrad_ef_update(g_first, b.m, b.e_u, b.v, b.vhat, b.x, None, None, 0, beta1, beta2, lr)
    vh = b.vhat if use_vhat else None
    ctx.sketch_accumulate(b.e_u, b.S_workers)
    ctx.sketch_reduce(b.S_workers, b.S_mean)
    ctx.unsketch_topk(b.S_mean, vh, b.idx, None)
    ctx.gather_topk(b.e_u, vh, b.idx, b.U_workers, b.delta)
    ctx.amsgrad_ef_update(g_next, b.m, b.e_u, b.v, b.vhat, b.x, b.idx, b.delta, ctx.k, beta1, beta2, lr)
