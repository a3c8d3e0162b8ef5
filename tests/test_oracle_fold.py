"""Pins for the oracle's synchronous delay-compensated fold (the supplement's
"Large Mini-batch Synchronous SGD with Delay-Compensated Gradient")."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import MODE_A, MODE_C

F32 = np.float32


def test_lambda_zero_is_large_minibatch_ssgd():
    """Without compensation the fold is one synchronous step with the averaged
    gradient: w - eta_hat * (1/J) * sum_j g_j (the supplement's large-batch rule)."""
    rng = np.random.default_rng(0)
    n, J, eta_hat = 301, 8, 0.8
    w0 = rng.standard_normal(n).astype(F32)
    g = rng.standard_normal((J, n)).astype(F32)
    sv = oracle.Server(w0, 1, 0.123, 0.0, MODE_C)
    sv.sync_fold(g, eta_hat)
    step = F32(F32(eta_hat) / F32(J))
    w = w0.copy()
    for j in range(J):                       # same sum, taken one gradient at a time
        w = (w - (step * g[j]).astype(F32)).astype(F32)
    assert np.array_equal(sv.w(), w)
    exact = w0.astype(np.float64) - eta_hat * g.astype(np.float64).mean(axis=0)
    assert np.max(np.abs(sv.w() - exact)) < 1e-5
    assert sv.t == J


@pytest.mark.parametrize("mode", [MODE_C, MODE_A])
def test_single_gradient_is_plain_sgd(mode):
    rng = np.random.default_rng(1)
    n = 100
    w0 = rng.standard_normal(n).astype(F32)
    g = rng.standard_normal((1, n)).astype(F32)
    sv = oracle.Server(w0, 1, 0.5, 2.0, mode, ema_m=0.9, eps=1e-7)
    sv.sync_fold(g, 0.25)
    assert np.array_equal(sv.w(), (w0 - (F32(0.25) * g[0]).astype(F32)).astype(F32))


def test_hand_worked_fold():
    """lambda = 1/4, eta_hat = 1, J = 2 (step 1/2), w_t = 1, g = (2, 4):
    j=0: moved 0      -> w = 1 - 0.5*2 = 0
    j=1: moved 0-1=-1 -> compensated 4 + 0.25*16*(-1) = 0 -> w stays 0."""
    sv = oracle.Server(np.array([1.0], dtype=F32), 1, 9.0, 0.25, MODE_C)
    sv.sync_fold(np.array([[2.0], [4.0]], dtype=F32), 1.0)
    assert float(sv.w()[0]) == 0.0
    # the other order: j=0: w = 1 - 0.5*4 = -1; j=1: moved -2 -> 2 + 0.25*4*(-2) = 0 -> w = -1
    sv = oracle.Server(np.array([1.0], dtype=F32), 1, 9.0, 0.25, MODE_C)
    sv.sync_fold(np.array([[4.0], [2.0]], dtype=F32), 1.0)
    assert float(sv.w()[0]) == -1.0


def test_exact_rational_brute_force():
    rng = np.random.default_rng(2)
    n, J = 8, 4
    lam, eta_hat = Fraction(1, 4), Fraction(2)
    w0 = (rng.integers(-8, 9, n) / 4).astype(F32)
    g = (rng.choice([-1.0, 1.0], (J, n)) * 2.0 ** rng.integers(-1, 2, (J, n))).astype(F32)
    sv = oracle.Server(w0, 1, 0.5, float(lam), MODE_C)
    sv.sync_fold(g, float(eta_hat))
    step = eta_hat / J
    for i in range(n):
        wt = Fraction(float(w0[i]))
        w = wt
        for j in range(J):
            gj = Fraction(float(g[j, i]))
            w = w - step * (gj + lam * gj * gj * (w - wt))
        assert Fraction(float(sv.w()[i])) == w


def test_fold_reproduces_sequential_sgd_when_lambda_g2_is_the_curvature():
    """The supplement's point: with an exact first-order term the fold of J
    same-snapshot gradients equals J sequential SGD steps with learning rate
    eta_hat/J on the samples in the same order.  Quadratic sample loss
    0.5*h*(w - c_j)^2, gradient at w_t: g_j = h (w_t - c_j); choose c_j so that
    g_j = +-2 and lambda = 1/4, h = 1: lambda g_j^2 = h."""
    h, lam, eta_hat, J, w_t = 1.0, 0.25, 2.0, 4, 0.5
    signs = [1.0, -1.0, -1.0, 1.0]
    c = [w_t - s * 2.0 / h for s in signs]
    g = np.array([[h * (w_t - cj)] for cj in c], dtype=F32)
    sv = oracle.Server(np.array([w_t], dtype=F32), 1, 0.0, lam, MODE_C)
    sv.sync_fold(g, eta_hat)
    w = w_t
    for cj in c:                                   # sequential SGD, gradient at the running model
        w = w - (eta_hat / J) * h * (w - cj)
    assert float(sv.w()[0]) == w
    # and uncompensated large-batch SGD lands elsewhere
    plain = w_t - eta_hat * float(np.mean(g))
    assert plain != w


def test_adaptive_fold_advances_mean_square_per_gradient():
    m, eps, lam0 = 0.75, 0.0, 0.25
    sv = oracle.Server(np.array([1.0], dtype=F32), 1, 0.0, lam0, MODE_A, ema_m=m, eps=eps)
    sv.sync_fold(np.array([[2.0], [2.0]], dtype=F32), 1.0)
    # j=0: MS = 0.25*4 = 1, lambda = 0.25, moved 0 -> w = 1 - 0.5*2 = 0
    # j=1: MS = 0.75 + 1 = 1.75, lambda = 0.25/sqrt(1.75), moved -1
    ms = 1.75
    lam = np.float32(lam0) / np.sqrt(np.float32(ms))
    w = 0.0 - 0.5 * (2.0 + float(lam) * 4.0 * (-1.0))
    assert float(sv.ms()[0]) == ms
    assert abs(float(sv.w()[0]) - w) < 1e-6
    assert sv.t == 2


def test_grad_sqnorms_against_a_library_dot_product():
    rng = np.random.default_rng(6)
    g = (rng.standard_normal((5, 100003)) * np.array([[1e-3], [1.0], [30.0], [1e-6], [0.2]])).astype(F32)
    got = oracle.grad_sqnorms(g)
    g64 = g.astype(np.float64)
    ref = np.einsum("ji,ji->j", g64, g64)
    assert np.all(np.abs(got - ref) <= 1e-13 * ref)
    # against exact rational arithmetic on a shorter vector
    from fractions import Fraction
    short = g[:, :2000]
    exact = [sum(Fraction(float(x)) ** 2 for x in row) for row in short]
    for a, e in zip(oracle.grad_sqnorms(short), exact):
        assert abs(Fraction(float(a)) - e) <= e * Fraction(1, 2 ** 52)
    # exact on small integers, and the order it induces
    h = np.array([[3, 4, 0], [1, 1, 1], [0, 0, 2]], dtype=F32)
    assert oracle.grad_sqnorms(h).tolist() == [25.0, 3.0, 4.0]
    assert np.argsort(oracle.grad_sqnorms(h), kind="stable").tolist() == [1, 2, 0]


def test_smallest_first_keeps_the_running_model_closer_to_the_snapshot():
    """The reason the supplement gives for an order: applying the small
    gradients first keeps |wt^j - w_t| smaller along the way (checked on the
    distances themselves, with lambda = 0 so that the steps are the gradients)."""
    rng = np.random.default_rng(7)
    n, J = 256, 6
    g = (rng.standard_normal((J, n)) * rng.uniform(0.1, 3.0, (J, 1))).astype(F32)
    order = np.argsort(oracle.grad_sqnorms(g), kind="stable")

    def path_distances(rows):
        w0 = np.zeros(n, dtype=F32)
        out = []
        for j in range(1, J + 1):
            sv = oracle.Server(w0, 1, 0.0, 0.0, MODE_C)
            sv.sync_fold(rows[:j], 0.1 * j)        # step 0.1 per gradient
            out.append(float(np.linalg.norm(sv.w().astype(np.float64))))
        return np.array(out)

    asc, desc = path_distances(g[order]), path_distances(g[order[::-1]])
    assert np.all(asc[:-1] <= desc[:-1] + 1e-9)
    assert abs(asc[-1] - desc[-1]) < 1e-4            # same end point without compensation


@pytest.mark.parametrize("mode", [MODE_C, MODE_A])
def test_a_fold_delivered_in_parts_is_the_undivided_fold(mode):
    """J = 40 same-snapshot gradients in parts of 16, 16 and 8 against the kept w_t must
    leave the bits of the one-call fold; with the running model as anchor (a mistake the
    interface invites) they must not."""
    rng = np.random.default_rng(21)
    n, J = 700, 40
    w0 = rng.standard_normal(n).astype(F32)
    g = (0.3 * rng.standard_normal((J, n))).astype(F32)
    lam0 = 2.0 if mode == MODE_A else 0.04
    whole = oracle.Server(w0, 1, 0.1, lam0, mode, 0.95, 1e-7)
    whole.sync_fold(g, 2.0)
    parts = oracle.Server(w0, 1, 0.1, lam0, mode, 0.95, 1e-7)
    anchor = parts.w().copy()
    for lo, hi in ((0, 16), (16, 32), (32, 40)):
        parts.sync_fold_part(g[lo:hi], J, 2.0, anchor)
    assert parts.t == whole.t == J
    assert parts.w().tobytes() == whole.w().tobytes()
    assert parts.ms().tobytes() == whole.ms().tobytes()
    wrong = oracle.Server(w0, 1, 0.1, lam0, mode, 0.95, 1e-7)
    for lo, hi in ((0, 16), (16, 32), (32, 40)):
        wrong.sync_fold_part(g[lo:hi], J, 2.0, wrong.w())
    assert wrong.w().tobytes() != whole.w().tobytes()
    # one part that is the whole fold, anchored at the current model, is sync_fold itself
    single = oracle.Server(w0, 1, 0.1, lam0, mode, 0.95, 1e-7)
    single.sync_fold_part(g[:16], 16, 0.8, single.w())
    ref = oracle.Server(w0, 1, 0.1, lam0, mode, 0.95, 1e-7)
    ref.sync_fold(g[:16], 0.8)
    assert single.w().tobytes() == ref.w().tobytes()
