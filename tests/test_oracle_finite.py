"""Section 5 warns that a large lambda adds variance; the compensated step
contracts towards the backup only while eta * lambda_t * g^2 < 2, and the
adaptive variant starts with a small MeanSquare, so the first pushes of
configuration 1 can overshoot.  Parity on NaNs would be meaningless, so the
oracle looks at its state after EVERY push: configurations 0 and 1 (run in
full) must never leave an inf or NaN behind, and a run that does blow up must
be reported at the push where it happens."""
import numpy as np
import pytest

import oracle
from paper_1609_08326_amd import workloads as W


@pytest.mark.parametrize("cfg", [0, 1])
def test_small_configurations_stay_finite_after_every_push(cfg):
    wl = W.CONFIGS[cfg]
    sv = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    bad = sv.run(wl.arrivals(), wl.hdiag(), wl.wstar(), wl.sigma, wl.seed, nthreads=8,
                 check_finite=True)
    assert bad is None, "state not finite after push %s of %s" % (bad, wl.name)
    assert sv.t == wl.T
    assert np.all(np.isfinite(sv.w())) and np.all(np.isfinite(sv.ms()))
    for m in range(wl.M):
        assert np.all(np.isfinite(sv.bak(m)))


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_large_configurations_stay_finite_on_a_sample(cfg):
    """Every push of the large configurations, on a seeded sample of elements
    (elements never interact, so each sampled history is complete)."""
    wl = W.CONFIGS[cfg]
    idx = wl.sample_indices(60_000, edge=512)
    sel = idx.astype(np.int64)
    sv = oracle.Server(wl.w0()[sel], wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    bad = sv.run(wl.arrivals(), wl.hdiag()[sel], wl.wstar()[sel], wl.sigma, wl.seed, gidx=idx,
                 as_bf16=wl.grad_bf16, nthreads=8, check_finite=True)
    assert bad is None, "state not finite after push %s of %s" % (bad, wl.name)


def test_a_run_that_blows_up_is_reported_at_the_push_where_it_happens():
    """The checker itself: a step far beyond the stability bound makes w grow
    without bound; the index it reports is the one a push-by-push replay with
    numpy's isfinite finds, and the checked run leaves the same state as the
    plain one."""
    wl = W.CONFIGS[0].replace(name="unstable", d=4099, T=400, eta=3.0e4, lambda0=50.0)
    hd, ws, order = wl.hdiag(), wl.wstar(), wl.arrivals()
    sv = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    bad = sv.run(order, hd, ws, wl.sigma, wl.seed, nthreads=3, check_finite=True)
    assert bad is not None and 0 < bad < wl.T
    step = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    first = None
    for t, m in enumerate(order):
        g = oracle.synth_grad(step.bak(int(m)), hd, ws, wl.sigma, wl.seed, t)
        step.push(int(m), g)
        if first is None and not np.all(np.isfinite(step.w())):
            first = t
        step.pull(int(m))
    assert first == bad
    plain = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    plain.run(order, hd, ws, wl.sigma, wl.seed)
    assert sv.w().tobytes() == plain.w().tobytes() == step.w().tobytes()
