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


def test_philox_matches_second_implementation_on_a_million_counters():
    rng = np.random.default_rng(70)
    n = 1 << 20
    ctr = rng.integers(0, 1 << 32, size=(n, 4), dtype=np.uint64)
    key = rng.integers(0, 1 << 32, size=(n, 2), dtype=np.uint64)
    # a quarter of them shaped like the gradient noise's counters: (i/4, t, 0, 0), one key
    k = n // 4
    ctr[:k, 0] = np.arange(k) * 97 % (1 << 26)
    ctr[:k, 1] = np.arange(k) % 4000
    ctr[:k, 2:] = 0
    key[:k] = [160908326 + 2, 0]
    # and the corners of the word range
    ctr[k:k + 4] = [[0, 0, 0, 0], [0xFFFFFFFF] * 4, [0, 0xFFFFFFFF, 0, 0xFFFFFFFF], [1, 0, 0, 0]]
    key[k:k + 4] = [[0, 0], [0xFFFFFFFF, 0xFFFFFFFF], [0xFFFFFFFF, 0], [0, 1]]
    got = oracle.philox4x32_10_many(ctr, key)
    assert np.array_equal(got, philox_py(ctr, key))
    # the array entry point is the single-counter one in a loop
    for i in (0, 1, k, k + 1, n - 1):
        assert np.array_equal(got[i], oracle.philox4x32_10(ctr[i], key[i]))


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


# --- the noise transform once more, on numpy float32 arrays -----------------------
# Written from the definition of the transform (not from the oracle's source):
# every line is one binary32 operation on arrays, which numpy evaluates with
# one IEEE rounding each, so the result must be the oracle's bits.
def normal_pairs_np(xa, xb):
    f = np.float32
    xa = np.asarray(xa, dtype=np.uint32)
    xb = np.asarray(xb, dtype=np.uint32)
    # radius: u = ((xa >> 8) + 1) / 2^24 in (0, 1]
    k = (xa >> np.uint32(8)) + np.uint32(1)
    u = k.astype(f) * f(2.0 ** -24)
    ub = u.view(np.uint32)
    e = (ub >> np.uint32(23)).astype(np.int32) - 127
    mt = ((ub & np.uint32(0x007FFFFF)) | np.uint32(0x3F800000)).view(f)
    big = mt > f(1.41421354)
    mt = np.where(big, mt * f(0.5), mt)
    e = np.where(big, e + 1, e)
    num = mt - f(1.0)
    den = mt + f(1.0)
    s = num / den
    s2 = s * s
    p = np.full(s.shape, f(0.11111111))
    p = p * s2
    p = p + f(0.14285715)
    p = p * s2
    p = p + f(0.2)
    p = p * s2
    p = p + f(0.33333334)
    p = p * s2
    p = p + f(1.0)
    twos = f(2.0) * s
    lm = twos * p
    el = e.astype(f) * f(0.69314718)
    lnu = el + lm
    arg = f(-2.0) * lnu
    r = np.sqrt(arg)
    # angle 2*pi*j/2^24 folded to [0, pi/4]
    j = xb >> np.uint32(8)
    quadrant = j >> np.uint32(22)
    rr = j & np.uint32(0x3FFFFF)
    swap = rr > np.uint32(0x200000)
    rr = np.where(swap, np.uint32(0x400000) - rr, rr)
    x = rr.astype(f) * f(float.fromhex("0x1.921fb6p-22"))
    x2 = x * x
    sp = np.full(x.shape, f(2.7557319e-6))
    sp = sp * x2
    sp = sp - f(1.9841270e-4)
    sp = sp * x2
    sp = sp + f(8.3333333e-3)
    sp = sp * x2
    sp = sp - f(0.16666667)
    sp = sp * x2
    sp = sp + f(1.0)
    sn = x * sp
    cp = np.full(x.shape, f(-2.7557319e-7))
    cp = cp * x2
    cp = cp + f(2.4801587e-5)
    cp = cp * x2
    cp = cp - f(1.3888889e-3)
    cp = cp * x2
    cp = cp + f(4.1666668e-2)
    cp = cp * x2
    cp = cp - f(0.5)
    cp = cp * x2
    cs = cp + f(1.0)
    sn, cs = np.where(swap, cs, sn), np.where(swap, sn, cs)
    C = np.select([quadrant == 0, quadrant == 1, quadrant == 2], [cs, -sn, -cs], sn)
    S = np.select([quadrant == 0, quadrant == 1, quadrant == 2], [sn, cs, -sn], -cs)
    z0 = r * C
    z1 = r * S
    assert z0.dtype == f and z1.dtype == f
    return np.stack([z0, z1], axis=-1)


def corner_words():
    xas = [0x00000000, 0x000000FF, 0x00000100, 0x7FFFFFFF, 0x80000000, 0xB504F300,
           0xB504F400, 0xB504F200, 0x6A09E600, 0x6A09E700, 0xFFFFFE00, 0xFFFFFF00, 0xFFFFFFFF]
    js = []
    for octant in range(8):
        base = octant * 0x200000
        js += [base, base + 1, base + 0x1FFFFF, (base + 0x200000) & 0xFFFFFF, base + 0x100000]
    xa, xb = np.meshgrid(np.array(xas, dtype=np.uint32),
                         (np.array(js, dtype=np.uint32) << np.uint32(8)) | np.uint32(0x5A))
    return xa.ravel(), xb.ravel()


def test_normal_pair_bit_for_bit_against_numpy_float32():
    rng = np.random.default_rng(23)
    n = 1 << 18
    xa = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    xb = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    # small u (large radius), u near the fold of the mantissa, angles next to octant edges
    xa[:4096] = rng.integers(0, 1 << 14, size=4096, dtype=np.uint64).astype(np.uint32)
    xa[4096:8192] = (0xB504F3 + rng.integers(-600, 600, size=4096)).astype(np.uint32) << np.uint32(8)
    edge = (rng.integers(0, 8, size=8192) * 0x200000 + rng.integers(-40, 40, size=8192)) % (1 << 24)
    xb[:8192] = edge.astype(np.uint32) << np.uint32(8)
    ca, cb = corner_words()
    xa, xb = np.concatenate([xa, ca]), np.concatenate([xb, cb])
    got = oracle.normal_pairs(xa, xb)
    want = normal_pairs_np(xa, xb)
    bad = np.flatnonzero((got.view(np.uint32) != want.view(np.uint32)).any(axis=1))
    assert bad.size == 0, (bad.size, hex(int(xa[bad[0]])), hex(int(xb[bad[0]])), got[bad[0]], want[bad[0]])
    # the array entry point is the scalar one in a loop
    for i in (0, 5000, n - 1, n + 3):
        assert np.array_equal(oracle.normal_pair(int(xa[i]), int(xb[i])).view(np.uint32),
                              got[i].view(np.uint32))


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
