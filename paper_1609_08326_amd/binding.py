"""ctypes binding over ``libdcasgd.so`` (the C ABI of ``include/dcasgd.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory (``torch.empty(device="cuda")``) and
the stream handle; nothing here computes on tensors.  There is no fallback:
if the library is missing or a call is rejected, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdcasgd.so")

MODE_C = 0
MODE_A = 1
GRAD_BF16 = 1 << 4
PULL_ON_PUSH = 1 << 5
BAK_BF16 = 1 << 6
MAX_K = 16
FOLD_WS_BYTES = 262656

OK, EINVAL, EALIGN, ESTATE, EHIP = 0, -1, -2, -3, -4

# name -> (restype, argtypes); mirrors include/dcasgd.h one to one
_PROTOTYPES = {
    "dcasgd_create": (C.c_void_p, [C.c_size_t, C.c_int, C.c_float, C.c_float, C.c_int,
                                   C.c_float, C.c_float]),
    "dcasgd_destroy": (C.c_int, [C.c_void_p]),
    "dcasgd_bind": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "dcasgd_init": (C.c_int, [C.c_void_p, C.c_void_p]),
    "dcasgd_push": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]),
    "dcasgd_push_batch": (C.c_int, [C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_void_p),
                                    C.c_int, C.c_void_p]),
    "dcasgd_sync_fold": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int, C.c_float,
                                   C.c_void_p]),
    "dcasgd_grad_sqnorms": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int, C.c_void_p,
                                      C.c_void_p]),
    "dcasgd_sync_fold_part": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int, C.c_int,
                                        C.c_float, C.c_void_p, C.c_void_p]),
    "dcasgd_sync_fold_ordered": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int, C.c_float,
                                           C.c_void_p, C.c_void_p]),
    "dcasgd_sync_fold_ordered_static": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int,
                                                  C.c_float, C.c_void_p]),
    "dcasgd_push_synth": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_float,
                                    C.c_uint64, C.c_void_p]),
    "dcasgd_run_synth": (C.c_int, [C.c_void_p, C.POINTER(C.c_int), C.c_size_t, C.c_void_p,
                                   C.c_void_p, C.c_float, C.c_uint64, C.c_void_p]),
    "dcasgd_pull": (C.c_void_p, [C.c_void_p, C.c_int]),
    "dcasgd_step": (C.c_uint64, [C.c_void_p]),
    "dcasgd_last_error": (C.c_int, [C.c_void_p]),
    "dcasgd_strerror": (C.c_char_p, [C.c_int]),
    "dcasgd_set_momentum": (C.c_int, [C.c_void_p, C.c_float, C.c_void_p, C.c_void_p]),
    "dcasgd_bind_counter": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "dcasgd_set_step": (C.c_int, [C.c_void_p, C.c_uint64]),
    "dcasgd_worker_grad": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_float,
                                     C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p]),
    "dcasgd_timing": (C.c_int, [C.c_void_p, C.c_int]),
    "dcasgd_timing_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]),
    "dcasgd_timing_read_each": (C.c_int, [C.c_void_p, C.POINTER(C.c_float), C.c_size_t,
                                          C.POINTER(C.c_uint64)]),
    "dcasgd_set_eta": (C.c_int, [C.c_void_p, C.c_float]),
    "dcasgd_set_lambda": (C.c_int, [C.c_void_p, C.c_float]),
    "dcasgd_set_launch": (C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int]),
    "dcasgd_synth_grad": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_uint64,
                                    C.c_uint32, C.c_void_p, C.c_int, C.c_size_t, C.c_void_p,
                                    C.c_int, C.c_int]),
}

_lib = None


class DcasgdError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, strerror(code), code))


def load() -> C.CDLL:
    """Open the built library.  torch is imported first so that the HIP runtime
    the library resolves against is the one that owns torch's allocations."""
    global _lib
    if _lib is None:
        import torch  # noqa: F401  (loads libamdhip64 before our library asks for it)
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s is not built; run `python -m paper_1609_08326_amd.build`" % LIB_PATH)
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def strerror(code: int) -> str:
    return load().dcasgd_strerror(int(code)).decode()


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise DcasgdError(rc, where)


def _stream_ptr(stream=None) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def synth_grad(snap, hdiag, wstar, sigma: float, seed: int, push_idx: int, out, stream=None,
               threads: int = 0, items: int = 0, uncached: bool = False) -> None:
    """Launch the synthetic worker kernel: out <- h*(snap-wstar) + sigma*z(seed, push_idx, i).
    ``out`` and ``snap`` are float32 or bfloat16 CUDA tensors of the same length.
    ``uncached``: snapshot read and gradient write non-temporal (nothing is left in the
    last-level cache for the push that follows)."""
    import torch
    d = snap.numel()
    assert hdiag.numel() == d and wstar.numel() == d and out.numel() == d
    assert hdiag.dtype == wstar.dtype == torch.float32
    assert snap.dtype in (torch.float32, torch.bfloat16)
    assert out.dtype in (torch.float32, torch.bfloat16)
    formats = int(out.dtype == torch.bfloat16) | (int(snap.dtype == torch.bfloat16) << 1) \
        | (int(bool(uncached)) << 2)
    rc = load().dcasgd_synth_grad(snap.data_ptr(), hdiag.data_ptr(), wstar.data_ptr(),
                                  float(sigma), int(seed), int(push_idx), out.data_ptr(),
                                  formats, d, _stream_ptr(stream),
                                  int(threads), int(items))
    _check(rc, "dcasgd_synth_grad")


class Server:
    """One DC-ASGD parameter server (Algorithm 2) whose state lives in torch-owned HBM.

    ``w0`` is a float32 CUDA tensor holding the initial model; it becomes the
    live model ``self.w``.  ``self.bak`` is the M x stride backup matrix (row m
    is the snapshot worker m last pulled; bfloat16 with ``bak_bf16``), ``self.ms``
    the MeanSquare vector.
    """

    def __init__(self, w0, M: int, eta: float, lambda0: float, mode: int,
                 ema_m: float = 0.0, eps: float = 0.0, grad_bf16: bool = False,
                 pull_on_push: bool = False, stream=None, bak_bf16: bool = False):
        import torch
        lib = load()
        assert w0.is_cuda and w0.dtype == torch.float32 and w0.dim() == 1 and w0.is_contiguous()
        self.d, self.M = int(w0.numel()), int(M)
        self.mode = int(mode)
        self.grad_dtype = torch.bfloat16 if grad_bf16 else torch.float32
        flags = self.mode | (GRAD_BF16 if grad_bf16 else 0) | (PULL_ON_PUSH if pull_on_push else 0) \
            | (BAK_BF16 if bak_bf16 else 0)
        self.bak_dtype = torch.bfloat16 if bak_bf16 else torch.float32
        self._h = lib.dcasgd_create(self.d, self.M, float(eta), float(lambda0), flags,
                                    float(ema_m), float(eps))
        if not self._h:
            raise DcasgdError(EINVAL, "dcasgd_create")
        self._rows = None                               # cached views of the backup rows
        self.vel = None                                 # velocity, once momentum is on
        self.counter = None                             # device copy of t, once bound
        self.stride = (self.d + 63) // 64 * 64          # rows start 256-byte aligned
        self.w = w0
        self.bak = torch.empty((self.M, self.stride), dtype=self.bak_dtype, device=w0.device)
        self.ms = torch.empty(self.d, dtype=torch.float32, device=w0.device) \
            if self.mode == MODE_A else None
        _check(lib.dcasgd_bind(self._h, self.w.data_ptr(), self.bak.data_ptr(), self.stride,
                               self.ms.data_ptr() if self.ms is not None else None),
               "dcasgd_bind")
        self._update_stream = _stream_ptr(stream)       # where dcasgd_pull will enqueue its copy
        _check(lib.dcasgd_init(self._h, self._update_stream), "dcasgd_init")

    def close(self) -> None:
        if getattr(self, "_h", None):
            load().dcasgd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def t(self) -> int:
        return int(load().dcasgd_step(self._h))

    def set_momentum(self, mu: float, stream=None) -> None:
        """Heavy-ball momentum on the compensated gradient for all later pushes; the
        velocity (``self.vel``, torch-owned) restarts at zero.  mu = 0 switches it off."""
        import torch
        if mu == 0.0:
            self.vel = None
            _check(load().dcasgd_set_momentum(self._h, 0.0, None, _stream_ptr(stream)),
                   "dcasgd_set_momentum")
            return
        self.vel = torch.empty(self.d, dtype=torch.float32, device=self.w.device)
        _check(load().dcasgd_set_momentum(self._h, float(mu), self.vel.data_ptr(),
                                          _stream_ptr(stream)), "dcasgd_set_momentum")

    def bind_counter(self, stream=None) -> None:
        """Keep the push counter in device memory too (``self.counter``, one int32 owned by
        torch) so that launch sequences can be captured into a HIP graph and replayed."""
        import torch
        self.counter = torch.zeros(1, dtype=torch.int32, device=self.w.device)
        _check(load().dcasgd_bind_counter(self._h, self.counter.data_ptr(), _stream_ptr(stream)),
               "dcasgd_bind_counter")

    def set_step(self, t: int) -> None:
        """Tell the handle how many pushes have been applied (after graph replays)."""
        _check(load().dcasgd_set_step(self._h, int(t)), "dcasgd_set_step")

    def worker_grad(self, worker: int, hdiag, wstar, sigma: float, seed: int, out,
                    offset: int = 0, stream=None) -> None:
        """Synthetic gradient of worker's current backup, noise keyed by t + offset."""
        assert out.is_cuda and out.dtype == self.grad_dtype and out.numel() == self.d
        _check(load().dcasgd_worker_grad(self._h, int(worker), hdiag.data_ptr(), wstar.data_ptr(),
                                         float(sigma), int(seed), int(offset), out.data_ptr(),
                                         _stream_ptr(stream)), "dcasgd_worker_grad")

    def timing(self, enable: bool) -> None:
        """Attach start/stop HIP events to every server-update launch from now on."""
        _check(load().dcasgd_timing(self._h, int(bool(enable))), "dcasgd_timing")

    def timing_read(self):
        """(summed kernel milliseconds, launches) since the last read; waits for them."""
        ms, n = C.c_double(0.0), C.c_uint64(0)
        _check(load().dcasgd_timing_read(self._h, C.byref(ms), C.byref(n)), "dcasgd_timing_read")
        return float(ms.value), int(n.value)

    def timing_read_each(self, capacity: int = 65536):
        """Durations in milliseconds of the timed launches since the last read, in
        launch order (numpy float32 array); waits for them."""
        import numpy as np
        buf = np.zeros(int(capacity), dtype=np.float32)
        n = C.c_uint64(0)
        _check(load().dcasgd_timing_read_each(self._h, buf.ctypes.data_as(C.POINTER(C.c_float)),
                                              buf.size, C.byref(n)), "dcasgd_timing_read_each")
        return buf[: min(int(n.value), buf.size)].copy()

    def set_eta(self, eta: float) -> None:
        """Learning rate of all later pushes (step schedules)."""
        _check(load().dcasgd_set_eta(self._h, float(eta)), "dcasgd_set_eta")

    def set_lambda(self, lambda0: float) -> None:
        """lambda_t of Algorithm 2 for all later pushes (lambda_0 in the adaptive variant)."""
        _check(load().dcasgd_set_lambda(self._h, float(lambda0)), "dcasgd_set_lambda")

    def set_launch(self, threads: int = 0, items: int = 0, max_blocks: int = 0,
                   streaming: int = 2) -> None:
        _check(load().dcasgd_set_launch(self._h, int(threads), int(items), int(max_blocks),
                                        int(streaming)), "dcasgd_set_launch")

    def push(self, worker: int, grad, stream=None) -> None:
        assert grad.is_cuda and grad.dtype == self.grad_dtype and grad.numel() == self.d
        self._update_stream = _stream_ptr(stream)
        _check(load().dcasgd_push(self._h, int(worker), grad.data_ptr(), self._update_stream),
               "dcasgd_push")

    def push_batch(self, workers: Sequence[int], grads: Sequence, stream=None) -> None:
        K = len(workers)
        assert K == len(grads)
        for g in grads:
            assert g.is_cuda and g.dtype == self.grad_dtype and g.numel() == self.d
        wa = (C.c_int * K)(*[int(m) for m in workers])
        ga = (C.c_void_p * K)(*[g.data_ptr() for g in grads])
        self._update_stream = _stream_ptr(stream)
        _check(load().dcasgd_push_batch(self._h, wa, ga, K, self._update_stream),
               "dcasgd_push_batch")

    def push_synth(self, worker: int, hdiag, wstar, sigma: float, seed: int, stream=None) -> None:
        """Synthetic worker fused into the push: the gradient of worker's snapshot is
        formed in registers (noise keyed by the server's push counter) and applied."""
        assert hdiag.is_cuda and wstar.is_cuda and hdiag.numel() == wstar.numel() == self.d
        self._update_stream = _stream_ptr(stream)
        _check(load().dcasgd_push_synth(self._h, int(worker), hdiag.data_ptr(), wstar.data_ptr(),
                                        float(sigma), int(seed), self._update_stream),
               "dcasgd_push_synth")

    def run_synth(self, workers, hdiag, wstar, sigma: float, seed: int, stream=None) -> None:
        """push_synth for every entry of ``workers`` in order, looped in native code."""
        assert hdiag.is_cuda and wstar.is_cuda and hdiag.numel() == wstar.numel() == self.d
        ws = [int(m) for m in workers]
        arr = (C.c_int * len(ws))(*ws)
        self._update_stream = _stream_ptr(stream)
        _check(load().dcasgd_run_synth(self._h, arr, len(ws), hdiag.data_ptr(), wstar.data_ptr(),
                                       float(sigma), int(seed), self._update_stream),
               "dcasgd_run_synth")

    def sync_fold(self, grads: Sequence, eta_hat: float, stream=None, workspace=None) -> None:
        """Fold J same-snapshot gradients into w (the supplement's synchronous variant).
        With a workspace (see fold_workspace) the gradients are ranked by norm on the
        device first and folded smallest first; otherwise in the order given."""
        J = len(grads)
        for g in grads:
            assert g.is_cuda and g.dtype == self.grad_dtype and g.numel() == self.d
        ga = (C.c_void_p * J)(*[g.data_ptr() for g in grads])
        self._update_stream = _stream_ptr(stream)
        if workspace is None:
            _check(load().dcasgd_sync_fold(self._h, ga, J, float(eta_hat), self._update_stream),
                   "dcasgd_sync_fold")
            return
        assert workspace.is_cuda and workspace.is_contiguous()
        assert workspace.numel() * workspace.element_size() >= FOLD_WS_BYTES
        _check(load().dcasgd_sync_fold_ordered(self._h, ga, J, float(eta_hat),
                                               workspace.data_ptr(), self._update_stream),
               "dcasgd_sync_fold_ordered")

    def sync_fold_ordered_static(self, grads: Sequence, eta_hat: float, stream=None) -> None:
        """The ordered fold with the library's own static workspace: nothing is allocated
        by the call (for callers that cannot allocate); calls on one GPU must not overlap."""
        J = len(grads)
        for g in grads:
            assert g.is_cuda and g.dtype == self.grad_dtype and g.numel() == self.d
        ga = (C.c_void_p * J)(*[g.data_ptr() for g in grads])
        self._update_stream = _stream_ptr(stream)
        _check(load().dcasgd_sync_fold_ordered_static(self._h, ga, J, float(eta_hat),
                                                      self._update_stream),
               "dcasgd_sync_fold_ordered_static")

    def grad_sqnorms(self, grads: Sequence, workspace, stream=None) -> None:
        """Squared norms and ranking of up to 16 gradients into ``workspace`` (read them
        with fold_order after synchronising); the model is not touched."""
        J = len(grads)
        for g in grads:
            assert g.is_cuda and g.dtype == self.grad_dtype and g.numel() == self.d
        assert workspace.is_cuda and workspace.numel() * workspace.element_size() >= FOLD_WS_BYTES
        ga = (C.c_void_p * J)(*[g.data_ptr() for g in grads])
        _check(load().dcasgd_grad_sqnorms(self._h, ga, J, workspace.data_ptr(),
                                          _stream_ptr(stream)), "dcasgd_grad_sqnorms")

    def sync_fold_part(self, grads: Sequence, J_total: int, eta_hat: float, kept_w,
                       stream=None) -> None:
        """Some of the J_total gradients of one fold, compensated against ``kept_w``, the
        caller's copy of the model the fold started from (a float32 backup row will do)."""
        J = len(grads)
        for g in grads:
            assert g.is_cuda and g.dtype == self.grad_dtype and g.numel() == self.d
        import torch
        assert kept_w.is_cuda and kept_w.dtype == torch.float32 and kept_w.numel() == self.d
        ga = (C.c_void_p * J)(*[g.data_ptr() for g in grads])
        self._update_stream = _stream_ptr(stream)
        _check(load().dcasgd_sync_fold_part(self._h, ga, J, int(J_total), float(eta_hat),
                                            kept_w.data_ptr(), self._update_stream),
               "dcasgd_sync_fold_part")

    @staticmethod
    def fold_workspace(device="cuda"):
        """Device buffer of the size dcasgd_sync_fold_ordered asks for."""
        import torch
        return torch.empty(FOLD_WS_BYTES // 8, dtype=torch.float64, device=device)

    @staticmethod
    def fold_order(workspace, J: int):
        """(squared norms, permutation) the last ordered fold left in its workspace;
        the caller synchronises first."""
        import torch
        sq = workspace[:J].cpu().numpy().copy()
        perm = workspace.view(torch.int32)[32:32 + J].cpu().numpy().copy()
        return sq, perm

    def pull(self, worker: int, stream=None):
        """Refresh worker's backup from w and return it (a view of row `worker`).
        dcasgd_pull takes no stream: the library enqueues the copy on the stream of the
        last call that changed w.  ``stream`` (default: torch's current stream) states
        where the caller expects it; if that is another stream the copy would not be
        ordered with the caller's work, and this raises instead of racing."""
        if _stream_ptr(stream) != self._update_stream:
            raise ValueError("pull: the library refreshes the backup on the stream of the last "
                             "update (init/push/fold); pass that stream, or make it current")
        ptr = load().dcasgd_pull(self._h, int(worker))
        if not ptr:
            raise DcasgdError(load().dcasgd_last_error(self._h), "dcasgd_pull")
        row = self.snapshot(worker)
        assert row.data_ptr() == ptr
        return row

    def snapshot(self, worker: int):
        """The backup row of `worker` as it stands (no refresh).  The views are made once:
        slicing a tensor costs microseconds, which matters for 1 MB models."""
        if self._rows is None:
            self._rows = [self.bak[m, : self.d] for m in range(self.M)]
        return self._rows[int(worker)]
