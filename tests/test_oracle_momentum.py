"""Pins for the oracle's momentum variant.  The paper only says (footnote in
Section 6) that momentum variants were implemented; the rule pinned here is a
proposal: the classical heavy ball applied to the delay-compensated gradient,
v <- mu*v + g_dc, w <- w - eta*v.  What is pinned is that the oracle computes
exactly that rule - not that it is the authors' rule."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import MODE_A, MODE_C

F32 = np.float32


@pytest.mark.parametrize("mode", [MODE_C, MODE_A])
def test_switching_momentum_on_with_zero_history_changes_nothing_for_one_push(mode):
    rng = np.random.default_rng(0)
    n = 64
    w0 = rng.standard_normal(n).astype(F32)
    g1, g2 = rng.standard_normal((2, n)).astype(F32)
    a = oracle.Server(w0, 2, 0.1, 2.0, mode, 0.9, 1e-7)
    b = oracle.Server(w0, 2, 0.1, 2.0, mode, 0.9, 1e-7)
    b.set_momentum(0.9)
    for sv in (a, b):
        sv.push(1, g1)
    # first push: v = 0.9*0 + g_dc = g_dc, so w agrees
    assert np.array_equal(a.w(), b.w())
    a.push(0, g2)
    b.push(0, g2)
    assert not np.array_equal(a.w(), b.w())           # the second push feels the history


def test_single_worker_is_heavy_ball_sgd():
    """M = 1, zero delay: compensation vanishes, leaving v <- mu v + g, w <- w - eta v."""
    rng = np.random.default_rng(1)
    n, T, eta, mu = 200, 40, F32(0.1), F32(0.9)
    h = rng.uniform(0.05, 1.0, n).astype(F32)
    ws = rng.standard_normal(n).astype(F32)
    w0 = rng.standard_normal(n).astype(F32)
    sv = oracle.Server(w0, 1, eta, 2.0, MODE_A, 0.95, 1e-7)
    sv.set_momentum(mu)
    w, v = w0.copy(), np.zeros(n, dtype=F32)
    for _ in range(T):
        snap = sv.pull(0)
        g = (h * (snap - ws)).astype(F32)
        sv.push(0, g)
        v = ((mu * v).astype(F32) + g).astype(F32)
        w = (w - (eta * v).astype(F32)).astype(F32)
        assert np.array_equal(sv.w(), w)
        assert np.array_equal(sv.vel(), v)


def test_constant_gradient_closed_form():
    """lambda = 0, constant g: v_n = g (1 - mu^n)/(1 - mu), w_n = w_0 - eta * sum_k v_k."""
    eta, mu, g, w0 = 0.05, 0.8, 1.5, 2.0
    sv = oracle.Server(np.array([w0], dtype=F32), 1, eta, 0.0, MODE_C)
    sv.set_momentum(mu)
    e, m = float(F32(eta)), float(F32(mu))
    total = 0.0
    for n in range(1, 60):
        sv.push(0, np.array([g], dtype=F32))
        vn = g * (1 - m ** n) / (1 - m)
        total += vn
        assert abs(float(sv.vel()[0]) - vn) < 1e-5 * vn
        assert abs(float(sv.w()[0]) - (w0 - e * total)) < 1e-4


def test_exact_rational_trace_with_delay():
    rng = np.random.default_rng(3)
    n, M = 8, 3
    eta, lam, mu = Fraction(1, 2), Fraction(1, 4), Fraction(1, 2)
    w0 = (rng.integers(-8, 9, n) / 4).astype(F32)
    sv = oracle.Server(w0, M, float(eta), float(lam), MODE_C)
    sv.set_momentum(float(mu))
    w = [Fraction(float(x)) for x in w0]
    v = [Fraction(0)] * n
    bak = [list(w) for _ in range(M)]
    script = [("push", 0), ("push", 1), ("pull", 0), ("push", 2), ("push", 0), ("pull", 1), ("push", 1)]
    for op, m in script:
        if op == "push":
            g = (rng.choice([-1.0, 1.0], n) * 2.0 ** rng.integers(-1, 2, n)).astype(F32)
            sv.push(m, g)
            for i in range(n):
                gi = Fraction(float(g[i]))
                gdc = gi + lam * gi * gi * (w[i] - bak[m][i])
                v[i] = mu * v[i] + gdc
                w[i] = w[i] - eta * v[i]
        else:
            sv.pull(m)
            bak[m] = list(w)
        assert [Fraction(float(x)) for x in sv.w()] == w, (op, m)
        assert [Fraction(float(x)) for x in sv.vel()] == v


def test_momentum_off_again_and_fold():
    rng = np.random.default_rng(4)
    n = 32
    w0 = rng.standard_normal(n).astype(F32)
    g = rng.standard_normal((3, n)).astype(F32)
    a = oracle.Server(w0, 1, 0.1, 0.04, MODE_C)
    a.set_momentum(0.5)
    a.set_momentum(0.0)                       # off: plain rule again
    b = oracle.Server(w0, 1, 0.1, 0.04, MODE_C)
    a.sync_fold(g, 0.3)
    b.sync_fold(g, 0.3)
    assert np.array_equal(a.w(), b.w())
    # with momentum the fold carries the velocity from gradient to gradient
    c = oracle.Server(w0, 1, 0.1, 0.0, MODE_C)
    c.set_momentum(0.5)
    c.sync_fold(g, 0.3)
    step = F32(F32(0.3) / F32(3))
    w, v = w0.copy(), np.zeros(n, dtype=F32)
    for j in range(3):
        v = ((F32(0.5) * v).astype(F32) + g[j]).astype(F32)
        w = (w - (step * v).astype(F32)).astype(F32)
    assert np.array_equal(c.w(), w)
