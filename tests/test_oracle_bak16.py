"""Pins for the oracle's bfloat16-snapshot mode (a storage variant, not from the
paper): the pulled value is the library conversion of w, the value kept as
w_bak(m) is that same number, and everything else is Algorithm 2 unchanged."""
import os
from fractions import Fraction

import numpy as np
import torch

import oracle

F32 = np.float32
MODE_C, MODE_A = oracle.MODE_C, oracle.MODE_A
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "hand_trace_d8_m3.txt")


def torch_bf16(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=F32)).to(torch.bfloat16).float().numpy()


def test_pull_hands_out_the_library_conversion_and_keeps_it():
    rng = np.random.default_rng(3)
    w0 = (rng.standard_normal(5000) * np.exp(rng.uniform(-20, 20, 5000))).astype(F32)
    sv = oracle.Server(w0, 3, 0.1, 0.0, MODE_C)
    sv.set_backup_bf16()
    for m in range(3):                                   # switching on rounds what is held
        assert sv.bak(m).view(np.uint32).tolist() == torch_bf16(w0).view(np.uint32).tolist()
    g = rng.standard_normal(5000).astype(F32)
    sv.push(1, g)
    got = sv.pull(1)
    assert got.view(np.uint32).tolist() == torch_bf16(sv.w()).view(np.uint32).tolist()
    assert sv.bak(0).view(np.uint32).tolist() == torch_bf16(w0).view(np.uint32).tolist()   # untouched


def test_ties_round_to_even_in_the_pull():
    w0 = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 1 + 2.0 ** -8 + 2.0 ** -20,
                   2.0 ** -130, 3.0e38], dtype=F32)
    sv = oracle.Server(w0, 1, 0.1, 0.0, MODE_C)
    sv.set_backup_bf16()
    want = np.array([1.0, 1 + 2.0 ** -6, -1.0, 1 + 2.0 ** -7, 2.0 ** -130, 3.0e38], dtype=F32)
    want[5] = torch_bf16(w0[5:6])[0]
    assert sv.pull(0).tolist() == want.tolist()


def test_compensation_uses_the_rounded_snapshot_exact_case():
    """One parameter, w = 1 + 2^-10: the snapshot is 1, so w - w_bak = 2^-10 although the
    worker pulled a moment ago.  eta = lambda = 1/2, g = 1: every step is exact."""
    w0 = np.array([1 + 2.0 ** -10], dtype=F32)
    sv = oracle.Server(w0, 1, 0.5, 0.5, MODE_C)
    sv.set_backup_bf16()
    sv.push(0, np.array([1.0], dtype=F32))
    w, b, g, eta, lam = Fraction(1) + Fraction(1, 1024), Fraction(1), Fraction(1), Fraction(1, 2), Fraction(1, 2)
    expect = w - eta * (g + lam * g * g * (w - b))
    assert Fraction(float(sv.w()[0])) == expect == Fraction(1, 2) + Fraction(3, 4096)
    # without the variant the same push sees w - w_bak = 0
    sv32 = oracle.Server(w0, 1, 0.5, 0.5, MODE_C)
    sv32.push(0, np.array([1.0], dtype=F32))
    assert Fraction(float(sv32.w()[0])) == w - eta * g


def test_representable_states_give_the_float32_trajectory():
    """The hand-worked trace only visits values with at most 8 significant bits, so
    rounding the snapshots changes nothing: both modes must reproduce it."""
    rows = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            rows[k] = np.array([float(x) for x in v], dtype=F32)
    for mode16 in (False, True):
        sv = oracle.Server(rows["w0"], 3, 0.5, 0.25, MODE_C)
        if mode16:
            sv.set_backup_bf16()
        sv.push(1, rows["g_a"])
        assert sv.w().tolist() == rows["w1"].tolist()
        pulled = sv.pull(1)
        assert pulled.tolist() == torch_bf16(pulled).tolist(), "precondition: representable"
        sv.push(2, rows["g_b"])
        assert sv.w().tolist() == rows["w2"].tolist()


def test_lambda_zero_ignores_the_snapshot_format():
    rng = np.random.default_rng(4)
    w0 = rng.standard_normal(300).astype(F32)
    a = oracle.Server(w0, 4, 0.1, 0.0, MODE_C)
    b = oracle.Server(w0, 4, 0.1, 0.0, MODE_C)
    b.set_backup_bf16()
    for t in range(20):
        g = rng.standard_normal(300).astype(F32)
        m = int(rng.integers(0, 4))
        for sv in (a, b):
            sv.push(m, g)
            sv.pull(m)
    assert a.w().tolist() == b.w().tolist()
    assert not np.array_equal(a.bak(0), b.bak(0))


def test_worker_gradient_is_taken_at_the_rounded_snapshot_and_training_still_works():
    """run() computes each gradient from the stored backup, i.e. from the rounded
    snapshot; on the synthetic quadratic the final loss stays close to the float32 run."""
    rng = np.random.default_rng(5)
    n, M, T = 4000, 4, 400
    h = np.exp(rng.uniform(np.log(1e-2), 0.0, n)).astype(F32)
    wstar = rng.standard_normal(n).astype(F32)
    order = rng.integers(0, M, T).astype(np.int32)
    loss = {}
    for mode16 in (False, True):
        sv = oracle.Server(np.zeros(n, dtype=F32), M, 0.1, 2.0, MODE_A, 0.95, 1e-7)
        if mode16:
            sv.set_backup_bf16()
        sv.run(order, h, wstar, 0.01, 99)
        d = sv.w().astype(np.float64) - wstar
        loss[mode16] = 0.5 * float(np.sum(h * d * d))
        if mode16:
            for m in range(M):
                assert sv.bak(m).tolist() == torch_bf16(sv.bak(m)).tolist()
    start = 0.5 * float(np.sum(h * wstar.astype(np.float64) ** 2))
    assert loss[False] < 0.05 * start
    assert abs(loss[True] - loss[False]) < 0.05 * loss[False] + 1e-3 * start
