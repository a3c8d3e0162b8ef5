"""Pins for the oracle's random-number side: Philox4x32-10, the arithmetic-only
Box-Muller transform, and bf16 rounding.  None of these compare the oracle
with itself: Philox is checked against published known answers and a second,
independently written implementation; the normals against Box-Muller
evaluated with libm in double; bf16 against torch's conversion."""
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --- a second Philox4x32-10, written on Python/numpy integers ---------------
def philox_py(ctr, key):
    """ctr: uint64 array [..., 4] holding 32-bit words, key: [..., 2]."""
    c = [np.asarray(ctr[..., i], dtype=np.uint64) for i in range(4)]
    k = [np.asarray(key[..., i], dtype=np.uint64) for i in range(2)]
    mask = np.uint64(0xFFFFFFFF)
    for rnd in range(10):
        prod0 = np.uint64(0xD2511F53) * c[0]
        prod1 = np.uint64(0xCD9E8D57) * c[2]
        c = [(prod1 >> np.uint64(32)) ^ c[1] ^ k[0], prod1 & mask,
             (prod0 >> np.uint64(32)) ^ c[3] ^ k[1], prod0 & mask]
        k = [(k[0] + np.uint64(0x9E3779B9)) & mask, (k[1] + np.uint64(0xBB67AE85)) & mask]
    return np.stack(c, axis=-1).astype(np.uint32)


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        got = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in got] == v[6:10]
        got_py = philox_py(np.array(v[0:4], dtype=np.uint64), np.array(v[4:6], dtype=np.uint64))
        assert [int(x) for x in got_py] == v[6:10]


def test_philox_matches_second_implementation():
    rng = np.random.default_rng(7)
    ctr = rng.integers(0, 1 << 32, size=(5000, 4), dtype=np.uint64)
    key = rng.integers(0, 1 << 32, size=(5000, 2), dtype=np.uint64)
    # include the structured counters the gradient noise actually uses
    ctr[:1000, 0] = np.arange(1000)
    ctr[:1000, 1] = 17
    ctr[:1000, 2] = 0
    ctr[:1000, 3] = 0
    ref = philox_py(ctr, key)
    for i in range(ctr.shape[0]):
        got = oracle.philox4x32_10(ctr[i], key[i])
        assert np.array_equal(got, ref[i]), i


# --- Box-Muller --------------------------------------------------------------
def box_muller_f64(xa, xb):
    u = ((np.asarray(xa, dtype=np.uint64) >> np.uint64(8)) + np.uint64(1)).astype(np.float64) / 2.0**24
    ang = 2.0 * math.pi * (np.asarray(xb, dtype=np.uint64) >> np.uint64(8)).astype(np.float64) / 2.0**24
    r = np.sqrt(-2.0 * np.log(u))
    return r * np.cos(ang), r * np.sin(ang)


def test_normal_pair_against_libm_double():
    rng = np.random.default_rng(11)
    xa = rng.integers(0, 1 << 32, size=40000, dtype=np.uint64)
    xb = rng.integers(0, 1 << 32, size=40000, dtype=np.uint64)
    z = np.array([oracle.normal_pair(a, b) for a, b in zip(xa, xb)], dtype=np.float64)
    z0, z1 = box_muller_f64(xa, xb)
    # polynomial truncation ~2e-9 relative plus a handful of binary32 roundings
    tol = 4e-6
    assert np.max(np.abs(z[:, 0] - z0)) < tol
    assert np.max(np.abs(z[:, 1] - z1)) < tol


def test_normal_pair_corner_words():
    # smallest/largest u, every octant boundary of the angle and its neighbours
    xas = [0x00000000, 0x000000FF, 0x00000100, 0x7FFFFFFF, 0x80000000, 0xB504F300,
           0xB504F400, 0xFFFFFE00, 0xFFFFFF00, 0xFFFFFFFF]
    js = []
    for octant in range(8):
        base = octant * 0x200000
        js += [base, base + 1, base + 0x1FFFFF, (base + 0x200000) & 0xFFFFFF,
               base + 0x100000]
    for xa in xas:
        for j in js:
            xb = (j << 8) | 0x5A
            z = oracle.normal_pair(xa, xb).astype(np.float64)
            z0, z1 = box_muller_f64(np.array([xa]), np.array([xb]))
            assert abs(z[0] - z0[0]) < 4e-6, (hex(xa), hex(j))
            assert abs(z[1] - z1[0]) < 4e-6, (hex(xa), hex(j))
    # u = 1 gives radius 0; u = 2^-24 gives the largest radius sqrt(48 ln 2)
    assert np.all(oracle.normal_pair(0xFFFFFFFF, 0x12345678) == 0.0)
    zmax = oracle.normal_pair(0, 0)
    assert abs(float(zmax[0]) - math.sqrt(48.0 * math.log(2.0))) < 4e-6
    assert abs(float(zmax[1])) < 1e-6


def test_normal_quad_uses_counter_q_t_0_tag_and_is_standard_normal():
    seed = 0x1234_5678_9ABC_DEF0
    key = np.array([seed & 0xFFFFFFFF, seed >> 32], dtype=np.uint64)
    ts, qs = np.meshgrid(np.arange(40), np.arange(1500), indexing="ij")
    ctr = np.stack([qs.ravel(), ts.ravel(), np.zeros(qs.size, np.int64),
                    np.zeros(qs.size, np.int64)], axis=-1).astype(np.uint64)
    x = philox_py(ctr, np.broadcast_to(key, (ctr.shape[0], 2))).astype(np.uint64)
    a0, a1 = box_muller_f64(x[:, 0], x[:, 1])
    b0, b1 = box_muller_f64(x[:, 2], x[:, 3])
    ref = np.stack([a0, a1, b0, b1], axis=-1)
    got = np.array([oracle.normal_quad(seed, t, q) for t, q in zip(ts.ravel(), qs.ravel())],
                   dtype=np.float64)
    assert np.max(np.abs(got - ref)) < 4e-6
    flat = got.ravel()
    n = flat.size
    assert abs(flat.mean()) < 5.0 / math.sqrt(n)
    assert abs(flat.var() - 1.0) < 5.0 * math.sqrt(2.0 / n)
    assert abs((flat ** 3).mean()) < 5.0 * math.sqrt(15.0 / n)
    assert abs((flat ** 4).mean() - 3.0) < 5.0 * math.sqrt(96.0 / n)
    assert np.max(np.abs(flat)) <= math.sqrt(48.0 * math.log(2.0)) + 1e-5
    # a different tag or seed gives a different stream
    assert not np.array_equal(oracle.normal_quad(seed, 3, 5, 0), oracle.normal_quad(seed, 3, 5, 1))
    assert not np.array_equal(oracle.normal_quad(seed, 3, 5, 0), oracle.normal_quad(seed + 1, 3, 5, 0))


# --- bf16 ------------------------------------------------------------------------
def test_bf16_round_to_nearest_even_against_torch():
    torch = pytest.importorskip("torch")
    hi = np.arange(0, 0x10000, dtype=np.uint32)
    hi = hi[(hi & 0x7F80) != 0x7F80]            # finite inputs only
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x1234, 0xC000],
                    dtype=np.uint32)
    bits = ((hi[:, None] << 16) | lows[None, :]).ravel().astype(np.uint32)
    x = bits.view(np.float32)
    got = oracle.bf16_rne(x)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    rng = np.random.default_rng(3)
    y = (rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))).astype(np.float32)
    ref = torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.bf16_rne(y), ref)


def test_bf16_ties_go_to_even():
    def f(bits):
        return np.array([bits], dtype=np.uint32).view(np.float32)
    assert int(oracle.bf16_rne(f(0x3F808000))[0]) == 0x3F80      # tie, even stays
    assert int(oracle.bf16_rne(f(0x3F818000))[0]) == 0x3F82      # tie, odd goes up
    assert int(oracle.bf16_rne(f(0x3F808001))[0]) == 0x3F81      # above the tie
    assert int(oracle.bf16_rne(f(0x3F807FFF))[0]) == 0x3F80      # below the tie
