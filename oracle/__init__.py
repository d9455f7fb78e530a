"""ctypes front end of the CPU oracle (``sams_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package.  It imports nothing from the HIP library or its binding, and holds no
arithmetic of its own: every function marshals numpy arrays into the C routine of
the same name.  ``Oracle("f32")`` computes in float (the kernels' precision; use it
where a floating value decides an integer), ``Oracle("f64")`` in double.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "sams_oracle.c"), os.path.join(_HERE, "sams_oracle_impl.h")]
_SO = os.path.join(_HERE, "libsams_oracle.so")
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no contraction, no fast-math). Returns the .so path."""
    stale = force or not os.path.exists(_SO) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRC)
    if stale:
        subprocess.check_call(["gcc", *CFLAGS, _SRC[0], "-o", _SO, "-lm"])
    return _SO


def _declare(l: ctypes.CDLL) -> ctypes.CDLL:
    l.orc_hash_y.restype = ctypes.c_uint32
    l.orc_hash_y.argtypes = [ctypes.c_uint32] * 3
    l.orc_bucket.restype = ctypes.c_int64
    l.orc_bucket.argtypes = [ctypes.c_uint32] * 3 + [ctypes.c_int64]
    l.orc_sign.restype = ctypes.c_int
    l.orc_sign.argtypes = [ctypes.c_uint32] * 3
    return l


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = _declare(ctypes.CDLL(build()))
    return _lib


def use_library(path: str | None) -> None:
    """Tests only: route every later call to another build of the oracle (a deliberately broken copy,
    to show that the pins notice); ``None`` goes back to the real one."""
    global _lib
    _lib = None if path is None else _declare(ctypes.CDLL(path))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def hash_y(a: int, b: int, l: int) -> int:
    return int(lib().orc_hash_y(a, b, l))


def bucket(a: int, b: int, l: int, c: int) -> int:
    return int(lib().orc_bucket(a, b, l, c))


def sign(a: int, b: int, l: int) -> int:
    return int(lib().orc_sign(a, b, l))


def hash_dump(hash_params: np.ndarray, c: int, d: int):
    """bucket[r][d] (int32) and sign[r][d] (int8) for every row and coordinate."""
    hp = np.ascontiguousarray(hash_params, dtype=np.uint32)
    r = hp.shape[0]
    b = np.empty((r, d), dtype=np.int32)
    s = np.empty((r, d), dtype=np.int8)
    lib().orc_hash_dump(_p(hp), ctypes.c_int32(r), ctypes.c_int64(c), ctypes.c_int64(d), _p(b), _p(s))
    return b, s


class Oracle:
    """The oracle in one precision. Arrays must be C-contiguous numpy arrays of ``self.dtype``."""

    def __init__(self, precision: str = "f32"):
        assert precision in ("f32", "f64")
        self.suffix = "_" + precision
        self.dtype = np.float32 if precision == "f32" else np.float64
        self.creal = ctypes.c_float if precision == "f32" else ctypes.c_double
        self._l = lib()

    def _fn(self, name):
        return getattr(self._l, name + self.suffix)

    def _chk(self, *arrs):
        for a in arrs:
            if a is not None:
                assert a.dtype == self.dtype and a.flags.c_contiguous, (a.dtype, a.flags)

    def one_minus(self, beta: float):
        """1 - beta rounded in this precision (both operands already in this precision)."""
        return self.dtype(1) - self.dtype(beta)

    def sketch(self, u, hash_params, c):
        hp = np.ascontiguousarray(hash_params, dtype=np.uint32)
        r = hp.shape[0]
        self._chk(u)
        S = np.empty((r, c), dtype=self.dtype)
        self._fn("orc_sketch")(_p(u), ctypes.c_int64(u.shape[0]), ctypes.c_int32(r),
                               ctypes.c_int64(c), _p(hp), _p(S))
        return S

    def sketch_mean(self, S_w):
        self._chk(S_w)
        n, r, c = S_w.shape
        out = np.empty((r, c), dtype=self.dtype)
        self._fn("orc_sketch_mean")(_p(S_w), ctypes.c_int32(n), ctypes.c_int32(r), ctypes.c_int64(c), _p(out))
        return out

    def unsketch(self, S, vhat, d, hash_params, l0=0):
        """Estimates of the d coordinates l0 .. l0+d-1 (vhat, if given, holds those d entries)."""
        hp = np.ascontiguousarray(hash_params, dtype=np.uint32)
        self._chk(S, vhat)
        r, c = S.shape
        assert hp.shape[0] == r
        est = np.empty(d, dtype=self.dtype)
        self._fn("orc_unsketch")(_p(S), _p(vhat), ctypes.c_int64(d), ctypes.c_int32(r),
                                 ctypes.c_int64(c), _p(hp), _p(est), ctypes.c_int64(l0))
        return est

    def topk(self, est, k):
        self._chk(est)
        idx = np.empty(k, dtype=np.int32)
        fn = self._fn("orc_topk")
        fn.restype = ctypes.c_int
        rc = fn(_p(est), ctypes.c_int64(est.shape[0]), ctypes.c_int64(k), _p(idx))
        if rc != 0:
            raise MemoryError("orc_topk")
        return idx

    def gather(self, u, vhat, idx):
        self._chk(u, vhat)
        n, d = u.shape
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        k = idx.shape[0]
        U_w = np.empty((n, k), dtype=self.dtype)
        delta = np.empty(k, dtype=self.dtype)
        self._fn("orc_gather")(_p(u), _p(vhat), _p(idx), ctypes.c_int64(k), ctypes.c_int32(n),
                               ctypes.c_int64(d), _p(U_w), _p(delta))
        return U_w, delta

    def refine(self, idx_in, delta_in, k_out):
        self._chk(delta_in)
        idx_in = np.ascontiguousarray(idx_in, dtype=np.int32)
        idx_out = np.empty(k_out, dtype=np.int32)
        delta_out = np.empty(k_out, dtype=self.dtype)
        fn = self._fn("orc_refine")
        fn.restype = ctypes.c_int
        rc = fn(_p(idx_in), _p(delta_in), ctypes.c_int64(idx_in.shape[0]), ctypes.c_int64(k_out), _p(idx_out),
                _p(delta_out))
        if rc != 0:
            raise MemoryError("orc_refine")
        return idx_out, delta_out

    def head(self, g, m, e_u, v, vhat, in_prev, beta1, beta2, rho=1.0):
        """In place on m, e_u (receives u), v, vhat."""
        self._chk(g, m, e_u, v, vhat)
        n, d = g.shape
        if in_prev is not None:
            assert in_prev.dtype == np.uint8 and in_prev.shape == (d,)
        R = self.creal
        self._fn("orc_head")(_p(g), _p(m), _p(e_u), _p(v), _p(vhat), _p(in_prev), ctypes.c_int32(n),
                             ctypes.c_int64(d), R(self.dtype(beta1)), R(self.one_minus(beta1)),
                             R(self.dtype(beta2)), R(self.one_minus(beta2)), R(self.dtype(rho)))

    def head_pa(self, g, m, e_u, v_w, vhat_w, beta1, beta2, rho=1.0):
        """Alg. 1 worker lines, in place on m, e_u (receives u), v_w, vhat_w (all [n][d])."""
        self._chk(g, m, e_u, v_w, vhat_w)
        n, d = g.shape
        R = self.creal
        self._fn("orc_head_pa")(_p(g), _p(m), _p(e_u), _p(v_w), _p(vhat_w), ctypes.c_int32(n), ctypes.c_int64(d),
                                R(self.dtype(beta1)), R(self.one_minus(beta1)), R(self.dtype(beta2)),
                                R(self.one_minus(beta2)), R(self.dtype(rho)))

    def tail(self, e_u, x, idx, delta, lr):
        """In place on e_u (u in, e out) and x."""
        self._chk(e_u, x, delta)
        n, d = e_u.shape
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        self._fn("orc_tail")(_p(e_u), _p(x), _p(idx), _p(delta), ctypes.c_int64(idx.shape[0]),
                             ctypes.c_int32(n), ctypes.c_int64(d), self.creal(self.dtype(lr)))

    def step(self, g, state, hash_params, c, k, beta1, beta2, lr, rho=1.0, use_vhat=True):
        """One iteration of Alg. 2 on ``state`` (dict with m, e, v, vhat, x, in_prev), in place.

        Returns the intermediates: S_w, S_mean, est, idx, U_w, delta, and u (a copy of the
        sketched vector, taken before the tail turns it into e).
        """
        hp = np.ascontiguousarray(hash_params, dtype=np.uint32)
        r = hp.shape[0]
        n, d = g.shape
        m, e, v, vhat, x, in_prev = (state[q] for q in ("m", "e", "v", "vhat", "x", "in_prev"))
        self._chk(g, m, e, v, vhat, x)
        assert in_prev.dtype == np.uint8
        S_w = np.empty((n, r, c), dtype=self.dtype)
        S_mean = np.empty((r, c), dtype=self.dtype)
        est = np.empty(d, dtype=self.dtype)
        idx = np.empty(k, dtype=np.int32)
        U_w = np.empty((n, k), dtype=self.dtype)
        delta = np.empty(k, dtype=self.dtype)
        # the composite C routine runs head..tail in one go; to hand back u we run the same
        # routines one by one here (identical calls, identical order)
        self.head(g, m, e, v, vhat, in_prev, beta1, beta2, rho)
        u = e.copy()
        for i in range(n):
            S_w[i] = self.sketch(e[i], hp, c)
        S_mean[...] = self.sketch_mean(S_w)
        est[...] = self.unsketch(S_mean, vhat if use_vhat else None, d, hp)
        idx[...] = self.topk(est, k)
        U_w_, delta_ = self.gather(e, vhat if use_vhat else None, idx)
        U_w[...] = U_w_
        delta[...] = delta_
        self.tail(e, x, idx, delta, lr)
        in_prev[...] = 0
        in_prev[idx] = 1
        return dict(S_w=S_w, S_mean=S_mean, est=est, idx=idx, U_w=U_w, delta=delta, u=u)

    def step_c(self, g, state, hash_params, c, k, beta1, beta2, lr, rho=1.0, use_vhat=True):
        """Same iteration through the single C entry point ``orc_step`` (used for timing)."""
        hp = np.ascontiguousarray(hash_params, dtype=np.uint32)
        r = hp.shape[0]
        n, d = g.shape
        m, e, v, vhat, x, in_prev = (state[q] for q in ("m", "e", "v", "vhat", "x", "in_prev"))
        self._chk(g, m, e, v, vhat, x)
        S_w = np.empty((n, r, c), dtype=self.dtype)
        S_mean = np.empty((r, c), dtype=self.dtype)
        est = np.empty(d, dtype=self.dtype)
        idx = np.empty(k, dtype=np.int32)
        U_w = np.empty((n, k), dtype=self.dtype)
        delta = np.empty(k, dtype=self.dtype)
        R = self.creal
        fn = self._fn("orc_step")
        fn.restype = ctypes.c_int
        rc = fn(_p(g), _p(m), _p(e), _p(v), _p(vhat), _p(x), _p(in_prev), ctypes.c_int32(n),
                ctypes.c_int64(d), ctypes.c_int32(r), ctypes.c_int64(c), ctypes.c_int64(k), _p(hp),
                R(self.dtype(beta1)), R(self.one_minus(beta1)), R(self.dtype(beta2)),
                R(self.one_minus(beta2)), R(self.dtype(rho)), R(self.dtype(lr)),
                ctypes.c_int(1 if use_vhat else 0), _p(S_w), _p(S_mean), _p(est), _p(idx), _p(U_w), _p(delta))
        if rc != 0:
            raise MemoryError("orc_step")
        return dict(S_w=S_w, S_mean=S_mean, est=est, idx=idx, U_w=U_w, delta=delta)

    def init_state(self, x1, n, eps):
        """Alg. 2 'Set' line: m_0 = e_0 = 0, v_0 = vhat_0 = eps, I_0 empty."""
        d = x1.shape[0]
        return dict(m=np.zeros((n, d), self.dtype), e=np.zeros((n, d), self.dtype),
                    v=np.full(d, eps, self.dtype), vhat=np.full(d, eps, self.dtype),
                    x=np.array(x1, dtype=self.dtype), in_prev=np.zeros(d, np.uint8))
