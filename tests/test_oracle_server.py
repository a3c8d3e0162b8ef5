"""Pins for the oracle's server (Algorithm 2, Eq. 4.1, Eq. 18) against what the
paper and plain mathematics fix.  Each check would fail for a plausible slip:
a dropped factor, w_bak - w instead of w - w_bak, the wrong worker's backup,
MeanSquare used before it is refreshed, a pull that copies the wrong way."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import MODE_A, MODE_C

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
F32 = np.float32


def quad_grad(snap, h, wstar):
    """Noise-free gradient of 0.5*sum h (w-wstar)^2 in binary32 (numpy)."""
    return (h * (snap - wstar)).astype(F32)


# --- Section 5, discussion (3): lambda = 0 is ASGD (Eq. 2.2) ----------------
@pytest.mark.parametrize("mode", [MODE_C, MODE_A])
def test_lambda_zero_is_asgd(mode):
    rng = np.random.default_rng(1)
    n, M, T, eta = 257, 5, 60, F32(0.1)
    h = rng.uniform(0.01, 1.0, n).astype(F32)
    wstar = rng.standard_normal(n).astype(F32)
    w0 = rng.standard_normal(n).astype(F32)
    order = rng.integers(0, M, T)
    sv = oracle.Server(w0, M, eta, 0.0, mode, ema_m=0.9, eps=1e-7)
    # independent ASGD: every worker holds the snapshot it last pulled
    w = w0.copy()
    snaps = [w0.copy() for _ in range(M)]
    for m in order:
        g = quad_grad(snaps[m], h, wstar)
        sv.push(int(m), quad_grad(sv.bak(int(m)), h, wstar))
        sv.pull(int(m))
        w = (w - (eta * g).astype(F32)).astype(F32)       # Eq. 2.2
        snaps[m] = w.copy()
        assert np.array_equal(sv.w(), w)
    assert sv.t == T


# --- zero delay: one worker is sequential SGD --------------------------------------
@pytest.mark.parametrize("mode", [MODE_C, MODE_A])
def test_single_worker_is_sequential_sgd(mode):
    rng = np.random.default_rng(2)
    n, T, eta = 300, 80, F32(0.25)
    h = rng.uniform(0.01, 1.0, n).astype(F32)
    wstar = rng.standard_normal(n).astype(F32)
    w0 = rng.standard_normal(n).astype(F32)
    sv = oracle.Server(w0, 1, eta, 2.0, mode, ema_m=0.95, eps=1e-7)
    w = w0.copy()
    for _ in range(T):
        snap = sv.pull(0)
        assert np.array_equal(snap, w)
        g = quad_grad(snap, h, wstar)
        sv.push(0, g)
        w = (w - (eta * g).astype(F32)).astype(F32)
        assert np.array_equal(sv.w(), w)


# --- hand-worked numbers ------------------------------------------------------------
def _golden_rows():
    rows = {}
    for line in open(os.path.join(GOLDEN, "hand_trace_d8_m3.txt")):
        if line.strip() and not line.startswith("#"):
            p = line.split()
            rows[p[0]] = np.array([float(x) for x in p[1:]], dtype=F32)
    return rows


def test_hand_trace_first_two_events():
    r = _golden_rows()
    sv = oracle.Server(r["w0"], 3, 0.5, 0.25, MODE_C)
    sv.push(0, r["g_a"])
    assert np.array_equal(sv.w(), r["w1"])
    assert np.array_equal(sv.pull(0), r["w1"])
    sv.push(1, r["g_b"])
    assert np.array_equal(sv.w(), r["w2"])
    # backups: worker 1's is w1, the others still w0
    assert np.array_equal(sv.bak(0), r["w1"])
    assert np.array_equal(sv.bak(1), r["w0"])
    assert np.array_equal(sv.bak(2), r["w0"])


def _exact_server(w0, M, eta, lam_fn):
    """Algorithm 2 on exact rationals. lam_fn(g) -> lambda*g*g as a Fraction."""
    state = {"w": [Fraction(float(x)) for x in w0]}
    state["bak"] = [list(state["w"]) for _ in range(M)]

    def push(m, g):
        g = [Fraction(float(x)) for x in g]
        state["w"] = [w - eta * (gi + lam_fn(gi) * (w - b))
                      for w, b, gi in zip(state["w"], state["bak"][m], g)]

    def pull(m):
        state["bak"][m] = list(state["w"])

    return state, push, pull


def _dyadic(rng, n, scale=4):
    return (rng.integers(-8, 9, n) / scale).astype(F32)


def _signed_pow2(rng, n):
    """+-2^k, k in -1..2: products with such gradients only shift exponents, so
    the whole trace stays exactly representable in binary32."""
    return (rng.choice([-1.0, 1.0], n) * 2.0 ** rng.integers(-1, 3, n)).astype(F32)


@pytest.mark.parametrize("variant", ["c", "a_stateless"])
def test_brute_force_exact_rational_trace_d8_m3(variant):
    """d = 8, M = 3, a script of pushes and pulls that is *not* the regular
    push-then-pull cycle (late pulls, a worker pushing twice on one backup)."""
    rng = np.random.default_rng(5)
    d, M = 8, 3
    eta, lam0 = Fraction(1, 2), Fraction(1, 4)
    w0 = _dyadic(rng, d)
    if variant == "c":
        sv = oracle.Server(w0, M, float(eta), float(lam0), MODE_C)
        lam_g2 = lambda g: lam0 * g * g
    else:
        # Eq. 18 with m = 0 and eps = 0: MeanSquare = g^2, sqrt = |g|, so
        # lambda_t g^2 = lambda_0 |g| (and 0 when g = 0 needs 0/0 avoided)
        sv = oracle.Server(w0, M, float(eta), float(lam0), MODE_A, ema_m=0.0, eps=0.0)
        lam_g2 = lambda g: lam0 * abs(g)
    st, push, pull = _exact_server(w0, M, eta, lam_g2)
    script = [("push", 0), ("pull", 0), ("push", 1), ("push", 2), ("pull", 2),
              ("push", 0), ("pull", 1), ("push", 2), ("push", 1), ("pull", 0),
              ("push", 0), ("pull", 1), ("pull", 2), ("push", 2)]
    for op, m in script:
        if op == "push":
            g = _signed_pow2(rng, d)
            sv.push(m, g)
            push(m, g)
        else:
            got = sv.pull(m)
            pull(m)
            assert [Fraction(float(x)) for x in got] == st["bak"][m]
        assert [Fraction(float(x)) for x in sv.w()] == st["w"], (op, m)
        for k in range(M):
            assert [Fraction(float(x)) for x in sv.bak(k)] == st["bak"][k]


# --- exact first-order compensation on a quadratic ---------------------------------
def test_compensation_recovers_current_gradient_when_lambda_g2_equals_curvature():
    """Section 3/4: the compensated gradient is g(w_t) + H (w_{t+tau} - w_t) with
    H replaced by lambda g.g.  For a quadratic with curvature h this is the
    exact gradient at the current model whenever lambda g^2 = h; the push then
    equals an SGD step taken at the current model."""
    h, wstar, lam0, eta = 1.0, 3.0, 0.25, 0.5
    b = wstar + 2.0                      # g = h (b - wstar) = 2, lambda g^2 = 1 = h
    for w_now in [-7.0, 0.0, 4.5, 5.0, 12.25]:
        sv = oracle.Server(np.array([b], dtype=F32), 2, eta, lam0, MODE_C)
        # move the model away from the backup with worker 1, lambda-free:
        # worker 1's backup equals w, so its push is a plain step of -eta*g1
        g1 = (b - w_now) / eta
        sv.push(1, np.array([g1], dtype=F32))
        assert float(sv.w()[0]) == w_now
        sv.push(0, np.array([h * (b - wstar)], dtype=F32))
        assert float(sv.w()[0]) == w_now - eta * h * (w_now - wstar)


# --- closed forms ---------------------------------------------------------------------
def test_constant_gradient_fixed_backup_closed_form():
    """With g and w_bak fixed, Eq. 4.1 is the affine recurrence
    (w - b) <- (1 - a)(w - b) - eta g,  a = eta lambda g^2."""
    eta, lam, g, b, w0 = 0.1, 0.04, 3.0, 1.5, -2.0
    sv = oracle.Server(np.array([b], dtype=F32), 2, eta, lam, MODE_C)
    sv.push(1, np.array([(b - w0) / eta], dtype=F32))       # w <- w0, backup 0 stays b
    start = float(sv.w()[0])
    a = float(F32(eta)) * float(F32(lam)) * g * g
    for n in range(1, 40):
        sv.push(0, np.array([g], dtype=F32))
        exact = b + (1 - a) ** n * (start - b) - float(F32(eta)) * g * (1 - (1 - a) ** n) / a
        assert abs(float(sv.w()[0]) - exact) < 2e-6 * max(1.0, abs(exact)), n


def test_mean_square_closed_form_and_lambda():
    """Eq. 18 with constant g from MeanSquare(0) = 0: MeanSquare(n) = g^2 (1 - m^n);
    lambda_n = lambda_0 / sqrt(MeanSquare(n) + eps) drives the step."""
    m, eps, lam0, eta, g = 0.95, 1e-7, 2.0, 0.05, 0.3
    b = 0.25
    sv = oracle.Server(np.array([b], dtype=F32), 2, eta, lam0, MODE_A, ema_m=m, eps=eps)
    # displace w from worker 0's backup through worker 1 with a tiny-gradient push
    # (it also touches MeanSquare; account for it below)
    g1 = -4.0
    sv.push(1, np.array([g1], dtype=F32))
    ms = (1 - float(F32(m))) * g1 * g1
    w = b - float(F32(eta)) * g1
    assert abs(float(sv.ms()[0]) - ms) < 1e-6
    assert abs(float(sv.w()[0]) - w) < 1e-6
    for n in range(1, 60):
        sv.push(0, np.array([g], dtype=F32))
        ms = float(F32(m)) * ms + (1 - float(F32(m))) * g * g
        lam = lam0 / math.sqrt(ms + float(F32(eps)))
        w = w - float(F32(eta)) * (g + lam * g * g * (w - b))
        assert abs(float(sv.ms()[0]) - ms) < 1e-6 * max(ms, 1e-3), n
        assert abs(float(sv.w()[0]) - w) < 1e-5, n
    # pure closed form for the EMA part
    sv2 = oracle.Server(np.zeros(1, dtype=F32), 1, eta, lam0, MODE_A, ema_m=m, eps=eps)
    for n in range(1, 100):
        sv2.push(0, np.array([g], dtype=F32))
        exact = g * g * (1 - float(F32(m)) ** n)
        assert abs(float(sv2.ms()[0]) - exact) < 2e-6 * exact + 1e-9, n


def test_adaptive_exact_square_root_case():
    """Adaptive variant on numbers where sqrt and the division are exact."""
    w0 = np.array([1.0, -3.0], dtype=F32)
    sv = oracle.Server(w0, 2, 0.5, 0.25, MODE_A, ema_m=0.75, eps=0.0)
    # worker 1's backup equals w, so this is a plain step; MeanSquare = 1/4 * g^2 = 1
    sv.push(1, np.array([2.0, -2.0], dtype=F32))
    assert np.array_equal(sv.ms(), np.array([1.0, 1.0], dtype=F32))
    assert np.array_equal(sv.w(), np.array([0.0, -2.0], dtype=F32))
    # worker 0 still holds w0, so w - w_bak = (-1, 1).  Restart MeanSquare at 0 and push
    # g = (4, 8): MeanSquare = 1/4 * (16, 64) = (4, 16), lambda = 0.25 / (2, 4),
    # lambda g^2 = (2, 4), compensated gradient = (4 + 2*(-1), 8 + 4*1) = (2, 12),
    # w = (0, -2) - 0.5 * (2, 12) = (-1, -8)
    sv.set_ms(np.array([0.0, 0.0], dtype=F32))
    sv.push(0, np.array([4.0, 8.0], dtype=F32))
    assert np.array_equal(sv.ms(), np.array([4.0, 16.0], dtype=F32))
    assert np.array_equal(sv.w(), np.array([-1.0, -8.0], dtype=F32))
    # one more on the kept MeanSquare, g = (2, 4): 0.75*(4, 16) + 0.25*(4, 16) = (4, 16) again.
    # Worker 1 never pulled, its backup is still w0 = (1, -3): w - w_bak = (-2, -5);
    # lambda = 0.25/(2, 4); lambda g^2 = (0.5, 1); gdc = (2 - 1, 4 - 5) = (1, -1);
    # w = (-1, -8) - 0.5*(1, -1) = (-1.5, -7.5)
    sv.pull(0)
    sv.push(1, np.array([2.0, 4.0], dtype=F32))
    assert np.array_equal(sv.ms(), np.array([4.0, 16.0], dtype=F32))
    assert np.array_equal(sv.w(), np.array([-1.5, -7.5], dtype=F32))


def test_m_zero_is_stateless():
    """Section 6.2 uses m = 0: MeanSquare(t) = g^2 whatever came before."""
    rng = np.random.default_rng(9)
    n = 64
    w0 = rng.standard_normal(n).astype(F32)
    g0 = rng.standard_normal(n).astype(F32)
    g = rng.standard_normal(n).astype(F32)
    out = []
    for junk in [0.0, 7.5, 1e-3]:
        sv = oracle.Server(w0, 2, 0.1, 2.0, MODE_A, ema_m=0.0, eps=1e-7)
        sv.push(1, g0)
        sv.set_ms(np.full(n, junk, dtype=F32))
        sv.push(0, g)
        out.append((sv.w(), sv.ms()))
        assert np.array_equal(sv.ms(), (g * g).astype(F32))
    assert all(np.array_equal(out[0][0], o[0]) for o in out[1:])


def test_fixed_point_and_pull_semantics():
    rng = np.random.default_rng(4)
    n, M = 100, 4
    wstar = rng.standard_normal(n).astype(F32)
    sv = oracle.Server(wstar, M, 0.1, 2.0, MODE_A, ema_m=0.5, eps=1e-7)
    sv.set_ms(np.full(n, 8.0, dtype=F32))
    sv.push(2, np.zeros(n, dtype=F32))                 # g = 0 at the optimum
    assert np.array_equal(sv.w(), wstar)
    assert np.array_equal(sv.ms(), np.full(n, 4.0, dtype=F32))
    # pull copies w into exactly one backup, bit for bit
    sv.push(1, rng.standard_normal(n).astype(F32))
    w = sv.w()
    before = [sv.bak(k) for k in range(M)]
    got = sv.pull(3)
    assert np.array_equal(got.view(np.uint32), w.view(np.uint32))
    for k in range(M):
        expect = w if k == 3 else before[k]
        assert np.array_equal(sv.bak(k).view(np.uint32), expect.view(np.uint32))
    assert np.array_equal(sv.w(), w)
    with pytest.raises(ValueError):
        sv.push(M, w)
    with pytest.raises(ValueError):
        sv.pull(-1)


def test_round_robin_has_constant_delay_scalar_recurrence():
    """Round-robin arrivals: after the first M pushes every gradient is M-1
    pushes old.  With lambda = 0 and no noise, w_{t+1} = w_t - eta h (w_{t-(M-1)} - wstar),
    the first M gradients all taken at w_0."""
    M, T, eta, h, wstar, w0 = 4, 200, 0.1, 0.7, 1.25, -0.5
    sv = oracle.Server(np.array([w0], dtype=F32), M, eta, 0.0, MODE_C)
    order = np.arange(T) % M
    sv.run(order, np.array([h], dtype=F32), np.array([wstar], dtype=F32), 0.0, seed=1)
    hist = [w0]
    for t in range(T):
        src = hist[t - (M - 1)] if t >= M else w0
        hist.append(hist[-1] - eta * h * (src - wstar))
    assert abs(float(sv.w()[0]) - hist[-1]) < 1e-5
    assert abs(hist[-1] - wstar) < 1e-3              # and it converges


# --- the event loop and the synthetic worker -----------------------------------------
def test_synth_grad_formula_and_noise_key():
    rng = np.random.default_rng(8)
    n = 1003
    snap = rng.standard_normal(n).astype(F32)
    h = rng.uniform(0.001, 1, n).astype(F32)
    wstar = rng.standard_normal(n).astype(F32)
    seed, t, sigma = 424242, 17, F32(0.01)
    g = oracle.synth_grad(snap, h, wstar, sigma, seed, t)
    z = np.concatenate([oracle.normal_quad(seed, t, q) for q in range((n + 3) // 4)])[:n]
    ref = ((h * (snap - wstar)).astype(F32) + (sigma * z).astype(F32)).astype(F32)
    assert np.array_equal(g, ref)
    # sigma = 0 leaves the plain quadratic gradient
    assert np.array_equal(oracle.synth_grad(snap, h, wstar, 0.0, seed, t), quad_grad(snap, h, wstar))
    # bf16 delivery = RNE of the fp32 value, widened
    gb = oracle.synth_grad(snap, h, wstar, sigma, seed, t, as_bf16=True)
    wid = (oracle.bf16_rne(g).astype(np.uint32) << 16).view(F32)
    assert np.array_equal(gb, wid)
    # a subset with global indices reproduces the same elements
    idx = np.array([0, 1, 2, 3, 4, 7, 500, 501, 1002], dtype=np.uint64)
    gs = oracle.synth_grad(snap[idx], h[idx], wstar[idx], sigma, seed, t, gidx=idx)
    assert np.array_equal(gs, g[idx])


@pytest.mark.parametrize("mode,bf16", [(MODE_C, False), (MODE_A, False), (MODE_A, True)])
def test_run_equals_explicit_loop_threads_and_subsets(mode, bf16):
    rng = np.random.default_rng(12)
    n, M, T = 1537, 6, 50
    h = np.exp(rng.uniform(math.log(1e-3), 0, n)).astype(F32)
    wstar = rng.standard_normal(n).astype(F32)
    w0 = np.zeros(n, dtype=F32)
    order = rng.integers(0, M, T)
    kw = dict(ema_m=0.95, eps=1e-7)
    seed, sigma = 99, 0.01
    a = oracle.Server(w0, M, 0.1, 2.0 if mode == MODE_A else 0.04, mode, **kw)
    a.run(order, h, wstar, sigma, seed, as_bf16=bf16)
    b = oracle.Server(w0, M, 0.1, 2.0 if mode == MODE_A else 0.04, mode, **kw)
    for t, m in enumerate(order):
        g = oracle.synth_grad(b.bak(int(m)), h, wstar, sigma, seed, t, as_bf16=bf16)
        b.push(int(m), g)
        b.pull(int(m))
    c = oracle.Server(w0, M, 0.1, 2.0 if mode == MODE_A else 0.04, mode, **kw)
    c.run(order[:20], h, wstar, sigma, seed, as_bf16=bf16, nthreads=3)
    c.run(order[20:], h, wstar, sigma, seed, as_bf16=bf16, nthreads=5)   # resumes at t = 20
    idx = np.sort(rng.choice(n, 200, replace=False)).astype(np.uint64)
    s = oracle.Server(w0[idx], M, 0.1, 2.0 if mode == MODE_A else 0.04, mode, **kw)
    s.run(order, h[idx], wstar[idx], sigma, seed, gidx=idx, as_bf16=bf16)
    assert a.t == b.t == c.t == s.t == T
    for x in (b, c):
        assert np.array_equal(a.w().view(np.uint32), x.w().view(np.uint32))
        assert np.array_equal(a.ms().view(np.uint32), x.ms().view(np.uint32))
        for k in range(M):
            assert np.array_equal(a.bak(k).view(np.uint32), x.bak(k).view(np.uint32))
    assert np.array_equal(a.w()[idx], s.w())
    assert np.array_equal(a.ms()[idx], s.ms())
    assert np.all(np.isfinite(a.w())) and np.all(np.isfinite(a.ms()))


def test_compensation_helps_on_the_quadratic():
    """Behavioural sanity (not a parity pin): on the noise-free quadratic with
    round-robin delay, DC-ASGD-c ends no further from the optimum than ASGD."""
    rng = np.random.default_rng(21)
    n, M, T = 512, 8, 400
    h = np.exp(rng.uniform(math.log(1e-2), 0, n)).astype(F32)
    wstar = rng.standard_normal(n).astype(F32)
    order = np.arange(T) % M
    loss = {}
    for lam in (0.0, 0.04):
        sv = oracle.Server(np.zeros(n, dtype=F32), M, 0.3, lam, MODE_C)
        sv.run(order, h, wstar, 0.0, 5)
        dw = sv.w().astype(np.float64) - wstar
        loss[lam] = 0.5 * float(np.sum(h * dw * dw))
    assert loss[0.04] <= loss[0.0]


def test_set_eta_changes_later_pushes_only():
    """A step schedule (Section 6 divides the learning rate by ten at fixed epochs):
    with one worker and zero delay the run is SGD with the scheduled rates."""
    rng = np.random.default_rng(31)
    n = 50
    w0 = rng.standard_normal(n).astype(F32)
    sv = oracle.Server(w0, 1, 0.5, 0.04, MODE_C)
    w = w0.copy()
    for step, eta in enumerate([0.5, 0.5, 0.05, 0.05, 0.005]):
        sv.set_eta(eta)
        g = rng.standard_normal(n).astype(F32)
        sv.pull(0)
        sv.push(0, g)
        w = (w - (F32(eta) * g).astype(F32)).astype(F32)
        assert np.array_equal(sv.w(), w), step


def test_time_indexed_lambda():
    """Algorithm 2 lists lambda_t as an input: changing it between pushes must equal
    running each stretch with a server built for that value (same state carried over),
    and lambda = 0 for a stretch must make that stretch plain ASGD."""
    rng = np.random.default_rng(12)
    n, M = 500, 3
    w0 = rng.standard_normal(n).astype(F32)
    gs = rng.standard_normal((12, n)).astype(F32)
    order = rng.integers(0, M, 12)
    sv = oracle.Server(w0, M, 0.1, 0.04, MODE_C)
    for t in range(12):
        if t == 4:
            sv.set_lambda(0.0)
        if t == 8:
            sv.set_lambda(0.5)
        before = sv.w().copy()
        bak = sv.bak(int(order[t])).copy()
        sv.push(int(order[t]), gs[t])
        lam = F32(0.04) if t < 4 else F32(0.0) if t < 8 else F32(0.5)
        g = gs[t]
        expect = before - F32(0.1) * (g + (lam * (g * g)) * (before - bak))
        assert np.array_equal(sv.w(), expect.astype(F32)), t
        if 4 <= t < 8:
            assert np.array_equal(sv.w(), (before - F32(0.1) * g).astype(F32))
        sv.pull(int(order[t]))
