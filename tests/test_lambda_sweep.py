"""Behaviour of the compensation strength on the synthetic quadratic, mirroring
the supplement's experiment on the influence of lambda: a small lambda
degrades to ASGD, a moderate one improves on it (and tolerates a step size at
which plain ASGD diverges under the same delay), a too-large one destroys the
run.  This is a sanity check of the method's behaviour, not a parity pin; the
GPU variant checks that the library reproduces the oracle's table exactly."""
import math

import numpy as np
import pytest

import oracle
from paper_1609_08326_amd import workloads as W

N, M, T, SEED = 4096, 8, 1200, 7


def _problem():
    rng = np.random.default_rng(0)
    h = np.exp(rng.uniform(math.log(1e-2), 0, N)).astype(np.float32)
    ws = rng.standard_normal(N).astype(np.float32)
    return h, ws, (np.arange(T) % M).astype(np.int32)


def _loss(w, h, ws):
    dw = w.astype(np.float64) - ws
    with np.errstate(all="ignore"):
        return 0.5 * float(np.sum(h * dw * dw))


def _oracle_loss(mode, eta, lam, sigma):
    h, ws, order = _problem()
    sv = oracle.Server(np.zeros(N, dtype=np.float32), M, eta, lam, mode, 0.95, 1e-7)
    sv.run(order, h, ws, sigma, SEED, nthreads=4)
    return _loss(sv.w(), h, ws), sv.w()


def test_oracle_lambda_regimes():
    # constant lambda, stable step size: more compensation helps until it blows up
    l0, _ = _oracle_loss(oracle.MODE_C, 0.2, 0.0, 0.05)
    l_small, _ = _oracle_loss(oracle.MODE_C, 0.2, 1e-4, 0.05)
    l_mid, _ = _oracle_loss(oracle.MODE_C, 0.2, 0.2, 0.05)
    l_good, _ = _oracle_loss(oracle.MODE_C, 0.2, 1.0, 0.05)
    l_huge, _ = _oracle_loss(oracle.MODE_C, 0.2, 5.0, 0.05)
    assert abs(l_small - l0) < 1e-3 * l0            # tiny lambda: ASGD again
    assert l_good < l_mid < l0                      # moderate lambda: better than ASGD
    assert not math.isfinite(l_huge) or l_huge > 100 * l0    # too large: destroyed
    # adaptive lambda shows the same three regimes
    a0, _ = _oracle_loss(oracle.MODE_A, 0.2, 0.0, 0.05)
    a_mid, _ = _oracle_loss(oracle.MODE_A, 0.2, 0.5, 0.05)
    a_huge, _ = _oracle_loss(oracle.MODE_A, 0.2, 8.0, 0.05)
    assert a0 == l0 and a_mid < a0
    assert not math.isfinite(a_huge) or a_huge > 100 * a0
    # delay tolerance: at eta = 0.4 the delayed plain update diverges, the compensated one does not
    d0, _ = _oracle_loss(oracle.MODE_C, 0.4, 0.0, 0.05)
    d_dc, _ = _oracle_loss(oracle.MODE_C, 0.4, 0.2, 0.05)
    assert not math.isfinite(d0) and math.isfinite(d_dc)


@pytest.mark.gpu
def test_gpu_reproduces_the_oracle_table():
    from gpu_harness import DeviceRun, assert_same_bits
    h, ws, order = _problem()
    for mode, eta, lam in ((W.MODE_C, 0.2, 0.0), (W.MODE_C, 0.2, 1.0), (W.MODE_A, 0.2, 0.5),
                           (W.MODE_C, 0.4, 0.2), (W.MODE_C, 0.4, 0.0), (W.MODE_A, 0.2, 8.0)):
        wl = W.Workload("sweep", d=N, M=M, T=T, mode=mode, eta=eta, lambda0=lam, ema_m=0.95,
                        eps=1e-7, h_lo=1e-2, h_hi=1.0, wstar_sigma=1.0, sigma=0.05,
                        order="round_robin", seed=SEED)
        print("sweep mode=%d eta=%g lambda=%g" % (mode, eta, lam), flush=True)
        run = DeviceRun(wl, hdiag=h, wstar=ws, arrivals=order)
        ref_loss, ref_w = _oracle_loss(mode, eta, lam, 0.05)
        if math.isfinite(ref_loss) and np.all(np.isfinite(ref_w)):
            assert_same_bits(run.w, ref_w, "sweep w")
            assert _loss(run.w, h, ws) == ref_loss
        else:
            # a diverged run ends in inf/NaN on both sides (NaN payloads are not compared)
            assert np.array_equal(np.isfinite(run.w), np.isfinite(ref_w))
