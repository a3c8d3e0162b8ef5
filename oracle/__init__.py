"""CPU oracle for the DC-ASGD parameter server (test infrastructure only).

The arithmetic lives in ``dcasgd_oracle.cpp`` (plain sequential C++); this
module compiles it with g++ and exposes it through ctypes.  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import it.  It imports nothing from the GPU package.

Paper passages followed: Algorithm 2 (server state, push and pull branches),
Eq. 4.1 (update rule), Eq. 18 and the text below it (adaptive lambda).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "dcasgd_oracle.cpp")
LIB = os.path.join(_HERE, "libdcasgd_oracle.so")

# One rounding per operation: no contraction, no fast-math.
CXXFLAGS = ["-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math",
            "-fPIC", "-shared", "-pthread"]

MODE_C = 0
MODE_A = 1


def build(force: bool = False) -> str:
    """Compile the oracle (g++) if the library is missing or older than its source."""
    stale = (not os.path.exists(LIB)) or os.path.getmtime(LIB) < os.path.getmtime(SRC)
    if force or stale:
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", *CXXFLAGS, SRC, "-o", tmp])
        os.replace(tmp, LIB)
    return LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, u32p, f32p, u64p, i32p = (C.c_void_p, C.POINTER(C.c_uint32),
                                      C.POINTER(C.c_float), C.POINTER(C.c_uint64),
                                      C.POINTER(C.c_int))
        L.oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_normal_pair.argtypes = [C.c_uint32, C.c_uint32, f32p]
        L.oracle_normal_pair.restype = None
        L.oracle_philox4x32_10_many.argtypes = [u32p, u32p, u32p, C.c_size_t]
        L.oracle_philox4x32_10_many.restype = None
        L.oracle_normal_pairs.argtypes = [u32p, u32p, f32p, C.c_size_t]
        L.oracle_normal_pairs.restype = None
        L.oracle_run_checked.argtypes = [vp, i32p, C.c_size_t, f32p, f32p, C.c_float, C.c_uint64,
                                         u64p, C.c_int, C.c_int, C.POINTER(C.c_longlong)]
        L.oracle_run_checked.restype = C.c_int
        L.oracle_normal_quad.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, f32p]
        L.oracle_normal_quad.restype = None
        L.oracle_bf16_rne.argtypes = [f32p, C.POINTER(C.c_uint16), C.c_size_t]
        L.oracle_bf16_rne.restype = None
        L.oracle_create.argtypes = [C.c_size_t, C.c_int, C.c_float, C.c_float, C.c_int,
                                    C.c_float, C.c_float, f32p]
        L.oracle_create.restype = vp
        L.oracle_destroy.argtypes = [vp]
        L.oracle_destroy.restype = None
        L.oracle_step.argtypes = [vp]
        L.oracle_step.restype = C.c_uint64
        L.oracle_set_momentum.argtypes = [vp, C.c_float]
        L.oracle_set_momentum.restype = None
        L.oracle_get_vel.argtypes = [vp, f32p]
        L.oracle_get_vel.restype = None
        L.oracle_set_backup_bf16.argtypes = [vp, C.c_int]
        L.oracle_set_backup_bf16.restype = None
        L.oracle_set_eta.argtypes = [vp, C.c_float]
        L.oracle_set_eta.restype = None
        L.oracle_set_lambda.argtypes = [vp, C.c_float]
        L.oracle_set_lambda.restype = None
        L.oracle_push.argtypes = [vp, C.c_int, f32p]
        L.oracle_push.restype = C.c_int
        L.oracle_pull.argtypes = [vp, C.c_int]
        L.oracle_pull.restype = C.c_int
        L.oracle_get_w.argtypes = [vp, f32p]
        L.oracle_get_w.restype = None
        L.oracle_get_ms.argtypes = [vp, f32p]
        L.oracle_get_ms.restype = None
        L.oracle_set_ms.argtypes = [vp, f32p]
        L.oracle_set_ms.restype = None
        L.oracle_get_bak.argtypes = [vp, C.c_int, f32p]
        L.oracle_get_bak.restype = C.c_int
        L.oracle_grad_sqnorms.argtypes = [f32p, C.c_int, C.c_size_t, C.POINTER(C.c_double)]
        L.oracle_grad_sqnorms.restype = None
        L.oracle_sync_fold_part.argtypes = [vp, f32p, C.c_int, C.c_int, C.c_float, f32p]
        L.oracle_sync_fold_part.restype = C.c_int
        L.oracle_sync_fold.argtypes = [vp, f32p, C.c_int, C.c_float]
        L.oracle_sync_fold.restype = C.c_int
        L.oracle_synth_grad.argtypes = [f32p, f32p, f32p, C.c_float, C.c_uint64, C.c_uint32,
                                        u64p, C.c_int, f32p, C.c_size_t]
        L.oracle_synth_grad.restype = None
        L.oracle_run.argtypes = [vp, i32p, C.c_size_t, f32p, f32p, C.c_float, C.c_uint64,
                                 u64p, C.c_int, C.c_int]
        L.oracle_run.restype = C.c_int
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _fp(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    u32p = C.POINTER(C.c_uint32)
    lib().oracle_philox4x32_10(c.ctypes.data_as(u32p), k.ctypes.data_as(u32p),
                               out.ctypes.data_as(u32p))
    return out


def philox4x32_10_many(ctr, key) -> np.ndarray:
    """Philox4x32-10 of n counters (n x 4 words) under n keys (n x 2 words): n x 4 words."""
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.ndim == 2 and c.shape[1] == 4 and k.shape == (c.shape[0], 2)
    out = np.zeros_like(c)
    u32p = C.POINTER(C.c_uint32)
    lib().oracle_philox4x32_10_many(c.ctypes.data_as(u32p), k.ctypes.data_as(u32p),
                                    out.ctypes.data_as(u32p), c.shape[0])
    return out


def normal_pairs(xa, xb) -> np.ndarray:
    """normal_pair over arrays of words: n x 2 float32."""
    a = np.ascontiguousarray(xa, dtype=np.uint32)
    b = np.ascontiguousarray(xb, dtype=np.uint32)
    assert a.ndim == 1 and a.shape == b.shape
    z = np.zeros((a.size, 2), dtype=np.float32)
    u32p = C.POINTER(C.c_uint32)
    lib().oracle_normal_pairs(a.ctypes.data_as(u32p), b.ctypes.data_as(u32p), _fp(z), a.size)
    return z


def normal_pair(xa: int, xb: int) -> np.ndarray:
    z = np.zeros(2, dtype=np.float32)
    lib().oracle_normal_pair(int(xa), int(xb), _fp(z))
    return z


def normal_quad(seed: int, t: int, q: int, tag: int = 0) -> np.ndarray:
    z = np.zeros(4, dtype=np.float32)
    lib().oracle_normal_quad(int(seed), int(t), int(q), int(tag), _fp(z))
    return z


def bf16_rne(x) -> np.ndarray:
    x = _f32(x).ravel()
    out = np.zeros(x.size, dtype=np.uint16)
    lib().oracle_bf16_rne(_fp(x), out.ctypes.data_as(C.POINTER(C.c_uint16)), x.size)
    return out


def grad_sqnorms(grads) -> np.ndarray:
    """Squared norms of the rows of ``grads`` (J x n float32), accumulated in double."""
    g = np.ascontiguousarray(grads, dtype=np.float32)
    assert g.ndim == 2
    out = np.zeros(g.shape[0], dtype=np.float64)
    lib().oracle_grad_sqnorms(_fp(g), int(g.shape[0]), int(g.shape[1]),
                              out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def synth_grad(snap, hdiag, wstar, sigma, seed, push_idx, gidx=None, as_bf16=False) -> np.ndarray:
    snap, hdiag, wstar = _f32(snap), _f32(hdiag), _f32(wstar)
    n = snap.size
    assert hdiag.size == n and wstar.size == n
    g = np.zeros(n, dtype=np.float32)
    gp = None
    if gidx is not None:
        gidx = np.ascontiguousarray(gidx, dtype=np.uint64)
        assert gidx.size == n
        gp = gidx.ctypes.data_as(C.POINTER(C.c_uint64))
    lib().oracle_synth_grad(_fp(snap), _fp(hdiag), _fp(wstar), float(sigma), int(seed),
                            int(push_idx), gp, int(bool(as_bf16)), _fp(g), n)
    return g


class Server:
    """Algorithm 2's parameter server, on the host, one element at a time."""

    def __init__(self, w0, M, eta, lambda0, mode, ema_m=0.0, eps=0.0):
        w0 = _f32(w0).ravel()
        self.n, self.M = int(w0.size), int(M)
        self._h = lib().oracle_create(self.n, self.M, float(eta), float(lambda0), int(mode),
                                      float(ema_m), float(eps), _fp(w0))
        if not self._h:
            raise ValueError("oracle_create rejected its arguments")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().oracle_destroy(self._h)
            self._h = None

    @property
    def t(self) -> int:
        return int(lib().oracle_step(self._h))

    def set_eta(self, eta: float) -> None:
        lib().oracle_set_eta(self._h, float(eta))

    def set_lambda(self, lambda0: float) -> None:
        """lambda_t of Algorithm 2 for all later pushes (lambda_0 in the adaptive variant)."""
        lib().oracle_set_lambda(self._h, float(lambda0))

    def set_backup_bf16(self, on: bool = True) -> None:
        """Snapshots travel and are kept as bfloat16 (round to nearest even of w)."""
        lib().oracle_set_backup_bf16(self._h, int(bool(on)))

    def set_momentum(self, mu: float) -> None:
        """Heavy-ball momentum on the compensated gradient; the velocity restarts at zero."""
        lib().oracle_set_momentum(self._h, float(mu))
        self._mu = float(mu)

    def vel(self) -> np.ndarray:
        out = np.zeros(self.n, dtype=np.float32)
        lib().oracle_get_vel(self._h, _fp(out))
        return out

    def push(self, worker: int, g) -> None:
        g = _f32(g).ravel()
        assert g.size == self.n
        if lib().oracle_push(self._h, int(worker), _fp(g)) != 0:
            raise ValueError("bad worker id")

    def pull(self, worker: int) -> np.ndarray:
        if lib().oracle_pull(self._h, int(worker)) != 0:
            raise ValueError("bad worker id")
        return self.bak(worker)

    def sync_fold(self, grads, eta_hat: float) -> None:
        """Supplement's synchronous variant: fold the rows of ``grads`` (J x n, all taken
        at the current model) into the model with step eta_hat/J, in row order."""
        g = np.ascontiguousarray(grads, dtype=np.float32)
        assert g.ndim == 2 and g.shape[1] == self.n
        if lib().oracle_sync_fold(self._h, _fp(g), int(g.shape[0]), float(eta_hat)) != 0:
            raise ValueError("sync_fold needs at least one gradient")

    def sync_fold_part(self, grads, J_total: int, eta_hat: float, anchor) -> None:
        """Some of the J_total gradients of one fold (rows of ``grads``), compensated against
        ``anchor``, the model the fold started from."""
        g = np.ascontiguousarray(grads, dtype=np.float32)
        a = _f32(anchor).ravel()
        assert g.ndim == 2 and g.shape[1] == self.n and a.size == self.n
        if lib().oracle_sync_fold_part(self._h, _fp(g), int(g.shape[0]), int(J_total),
                                       float(eta_hat), _fp(a)) != 0:
            raise ValueError("bad part of a fold")

    def w(self) -> np.ndarray:
        out = np.zeros(self.n, dtype=np.float32)
        lib().oracle_get_w(self._h, _fp(out))
        return out

    def ms(self) -> np.ndarray:
        out = np.zeros(self.n, dtype=np.float32)
        lib().oracle_get_ms(self._h, _fp(out))
        return out

    def set_ms(self, ms) -> None:
        ms = _f32(ms).ravel()
        assert ms.size == self.n
        lib().oracle_set_ms(self._h, _fp(ms))

    def bak(self, worker: int) -> np.ndarray:
        out = np.zeros(self.n, dtype=np.float32)
        if lib().oracle_get_bak(self._h, int(worker), _fp(out)) != 0:
            raise ValueError("bad worker id")
        return out

    def run(self, order, hdiag, wstar, sigma, seed, gidx=None, as_bf16=False, nthreads=1,
            check_finite=False):
        """T arrivals: gradient at the worker's backup, push, pull (Algorithm 1's cycle).
        With check_finite the state is inspected after every push and the index of the
        first arrival that left an inf or NaN in w, MeanSquare or the velocity is returned
        (None if there was none)."""
        order = np.ascontiguousarray(order, dtype=np.int32)
        hdiag, wstar = _f32(hdiag), _f32(wstar)
        assert hdiag.size == self.n and wstar.size == self.n
        gp = None
        if gidx is not None:
            gidx = np.ascontiguousarray(gidx, dtype=np.uint64)
            assert gidx.size == self.n
            gp = gidx.ctypes.data_as(C.POINTER(C.c_uint64))
        if check_finite:
            bad = C.c_longlong(-1)
            rc = lib().oracle_run_checked(self._h, order.ctypes.data_as(C.POINTER(C.c_int)),
                                          order.size, _fp(hdiag), _fp(wstar), float(sigma),
                                          int(seed), gp, int(bool(as_bf16)), int(nthreads),
                                          C.byref(bad))
            if rc != 0:
                raise ValueError("order holds a worker id outside [0, M)")
            return None if bad.value < 0 else int(bad.value)
        rc = lib().oracle_run(self._h, order.ctypes.data_as(C.POINTER(C.c_int)), order.size,
                              _fp(hdiag), _fp(wstar), float(sigma), int(seed), gp,
                              int(bool(as_bf16)), int(nthreads))
        if rc != 0:
            raise ValueError("order holds a worker id outside [0, M)")
        return None
