"""Helpers for the GPU parity tests: drive the HIP library and the CPU oracle
through the same seeded arrival sequence and compare bits."""
from __future__ import annotations

import numpy as np

import oracle
from paper_1609_08326_amd import workloads as W


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def assert_same_bits(got: np.ndarray, ref: np.ndarray, what: str) -> None:
    gb, rb = bits(got), bits(ref)
    assert gb.shape == rb.shape, (what, gb.shape, rb.shape)
    bad = np.flatnonzero(gb != rb)
    if bad.size:
        i = int(bad[0])
        raise AssertionError("%s: %d of %d elements differ; first at %d: gpu %r (0x%08x) oracle %r (0x%08x)"
                             % (what, bad.size, gb.size, i, float(got[i]), int(gb[i]),
                                float(ref[i]), int(rb[i])))


class DeviceRun:
    """State after running a workload through the HIP library."""

    def __init__(self, wl: W.Workload, *, fused: bool = True, batched: bool = False,
                 launch: dict | None = None, synth_launch: tuple = (0, 0), momentum: float = 0.0,
                 hdiag=None, wstar=None, arrivals=None, bak_bf16: bool = False):
        import torch
        from paper_1609_08326_amd import binding as B
        dev = torch.device("cuda:0")
        self.wl = wl
        self.hdiag_host = wl.hdiag() if hdiag is None else hdiag
        self.wstar_host = wl.wstar() if wstar is None else wstar
        self.arrivals = wl.arrivals() if arrivals is None else np.asarray(arrivals, dtype=np.int32)
        h = torch.from_numpy(self.hdiag_host).to(dev)
        ws = torch.from_numpy(self.wstar_host).to(dev)
        w = torch.from_numpy(wl.w0()).to(dev)
        sv = B.Server(w, wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps,
                      grad_bf16=wl.grad_bf16, pull_on_push=fused and not batched,
                      bak_bf16=bak_bf16)
        if launch:
            sv.set_launch(**launch)
        if momentum:
            sv.set_momentum(momentum)
        gdt = torch.bfloat16 if wl.grad_bf16 else torch.float32
        K = wl.K if batched else 1
        gbuf = [torch.empty(wl.d, dtype=gdt, device=dev) for _ in range(K)]
        T = len(self.arrivals)
        t = 0
        while t < T:
            k = min(K, T - t)
            ms_ = [int(m) for m in self.arrivals[t:t + k]]
            if batched:
                # a worker that shows up twice in one queue pushes its second
                # gradient from the backup refreshed inside the queue, which
                # only exists once the first part has run: feed such queues
                # in pieces that hold distinct workers
                start = 0
                while start < k:
                    end = start + 1
                    while end < k and ms_[end] not in ms_[start:end]:
                        end += 1
                    for j in range(start, end):
                        B.synth_grad(sv.snapshot(ms_[j]), h, ws, wl.sigma, wl.seed, t + j,
                                     gbuf[j], threads=synth_launch[0], items=synth_launch[1])
                    sv.push_batch(ms_[start:end], gbuf[start:end])
                    start = end
            else:
                m = ms_[0]
                B.synth_grad(sv.snapshot(m), h, ws, wl.sigma, wl.seed, t, gbuf[0],
                             threads=synth_launch[0], items=synth_launch[1])
                sv.push(m, gbuf[0])
                if not fused:
                    sv.pull(m)
            t += k
        torch.cuda.synchronize()
        assert sv.t == T
        self.server = sv
        self.w = sv.w.cpu().numpy()
        self.ms = sv.ms.cpu().numpy() if sv.ms is not None else None
        self.bak = sv.bak[:, : wl.d].float().cpu().numpy()
        self.vel = sv.vel.cpu().numpy() if getattr(sv, "vel", None) is not None else None


def oracle_run(wl: W.Workload, hdiag, wstar, arrivals, idx=None, nthreads: int = 8,
               momentum: float = 0.0, bak_bf16: bool = False):
    """The oracle on the same inputs; idx selects a subset of elements."""
    w0 = wl.w0()
    if idx is not None:
        hdiag, wstar, w0 = hdiag[idx], wstar[idx], w0[idx]
    sv = oracle.Server(w0, wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    if momentum:
        sv.set_momentum(momentum)
    if bak_bf16:
        sv.set_backup_bf16()
    bad = sv.run(arrivals, hdiag, wstar, wl.sigma, wl.seed, gidx=idx, as_bf16=wl.grad_bf16,
                 nthreads=nthreads, check_finite=True)
    assert bad is None, "%s: oracle state not finite after push %d" % (wl.name, bad)
    return sv


def compare(run: DeviceRun, ref: "oracle.Server", idx=None, tag: str = "") -> None:
    sel = (lambda a: a) if idx is None else (lambda a: a[idx.astype(np.int64)])
    w_ref = ref.w()
    assert np.all(np.isfinite(w_ref)), tag + " oracle produced non-finite w"
    assert_same_bits(sel(run.w), w_ref, tag + " w")
    if run.ms is not None:
        assert_same_bits(sel(run.ms), ref.ms(), tag + " ms")
    for m in range(run.wl.M):
        assert_same_bits(sel(run.bak[m]), ref.bak(m), tag + " bak[%d]" % m)
    if run.vel is not None:
        assert_same_bits(sel(run.vel), ref.vel(), tag + " velocity")
