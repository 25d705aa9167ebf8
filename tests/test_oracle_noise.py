"""Pins for the oracle's noise generator (paper §3.2 Eq. 3; docs/NOISE_SPEC.md N1-N6).

Each test checks the oracle against something other than itself: published known answers, the
algebraic inverse of the Philox round, libm in fp64, the textbook Box-Muller formula, closed-form
moments, or exhaustive enumeration of the rounding uniform.
"""
import math
import os

import numpy as np
import pytest
from scipy import stats

HERE = os.path.dirname(os.path.abspath(__file__))
M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def test_philox_known_answers(oracle):
    n = 0
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]
        n += 1
    assert n == 3


def _philox_forward(ctr, key):
    """Philox4x32-10 in plain Python integers, written from the published round (N1): a third
    implementation next to the C oracle and the HIP kernels."""
    c0, c1, c2, c3 = (int(v) for v in ctr)
    k0, k1 = (int(v) for v in key)
    for rnd in range(10):
        if rnd:
            k0, k1 = (k0 + W0) & MASK, (k1 + W1) & MASK
        p0, p1 = M0 * c0, M1 * c2
        c0, c1, c2, c3 = (p1 >> 32) ^ c1 ^ k0, p1 & MASK, (p0 >> 32) ^ c3 ^ k1, p0 & MASK
    return [c0, c1, c2, c3]


def test_philox_against_big_integer_python(oracle):
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        assert _philox_forward(v[0:4], v[4:6]) == v[6:10]
    rng = np.random.default_rng(7)
    cases = [([0, 0, 0, 0], [0, 1]), ([1, 0, 0, 0], [0, 0]), ([0, 0, 0, 1], [0, 0]), ([MASK, 0, MASK, 0], [MASK, 0])]
    cases += [([int(x) for x in rng.integers(0, 1 << 32, size=4)], [int(x) for x in rng.integers(0, 1 << 32, size=2)])
              for _ in range(500)]
    for ctr, key in cases:
        assert [int(x) for x in oracle.philox4x32_10(ctr, key)] == _philox_forward(ctr, key)
    # the tensor stream: counter (pair lo, pair hi, tensor id, 0), key (seed lo, seed hi)
    seed, tid = 0x0123456789ABCDEF, 77
    w = oracle.noise_words(seed, tid, (1 << 32) - 3, 6)
    for j in range(6):
        pair = (1 << 32) - 3 + j
        assert [int(x) for x in w[j]] == _philox_forward([pair & MASK, pair >> 32, tid, 0], [seed & MASK, seed >> 32])


def _philox_decrypt(out, key):
    """Inverse of the 10-round bijection, from the round's algebra (uses the modular inverses of
    the multipliers, which the forward direction never touches)."""
    inv0, inv1 = pow(M0, -1, 1 << 32), pow(M1, -1, 1 << 32)
    c = [int(x) for x in out]
    for rnd in range(9, -1, -1):
        k0 = (key[0] + rnd * W0) & MASK
        k1 = (key[1] + rnd * W1) & MASK
        c0 = (c[3] * inv0) & MASK          # lo32(M0*c0) = n3
        c2 = (c[1] * inv1) & MASK          # lo32(M1*c2) = n1
        c1 = c[0] ^ ((M1 * c2) >> 32) ^ k0
        c3 = c[2] ^ ((M0 * c0) >> 32) ^ k1
        c = [c0, c1, c2, c3]
    return c


def test_philox_is_the_keyed_bijection(oracle):
    rng = np.random.default_rng(1)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 1 << 32, size=4)]
        key = [int(x) for x in rng.integers(0, 1 << 32, size=2)]
        out = oracle.philox4x32_10(ctr, key)
        assert _philox_decrypt(out, key) == ctr


def test_counter_and_key_layout(oracle):
    seed = 0xFEDCBA9876543210
    tid = 0x1234567
    for pair_begin in (0, 5, (1 << 32) - 2, (1 << 40) + 17):
        w = oracle.noise_words(seed, tid, pair_begin, 4)
        for j in range(4):
            pair = pair_begin + j
            ref = oracle.philox4x32_10([pair & MASK, pair >> 32, tid, 0], [seed & MASK, seed >> 32])
            assert (w[j] == ref).all()
    # different tensor / seed give different streams
    assert (oracle.noise_words(seed, tid, 0, 8) != oracle.noise_words(seed, tid + 1, 0, 8)).any()
    assert (oracle.noise_words(seed, tid, 0, 8) != oracle.noise_words(seed + 1, tid, 0, 8)).any()


def test_philox_words_uniform(oracle):
    w = oracle.noise_words(42, 3, 0, 250000).reshape(-1)
    # each bit is set half the time (4 sigma of a binomial with n = 1e6)
    for b in range(32):
        frac = ((w >> np.uint32(b)) & 1).mean()
        assert abs(frac - 0.5) < 4 * 0.5 / math.sqrt(w.size)
    u = (w >> np.uint32(8)).astype(np.float64) / 2 ** 24
    assert stats.kstest(u[:200000], "uniform").pvalue > 1e-4


def test_ln_polynomial_against_libm(oracle):
    rng = np.random.default_rng(2)
    ms = np.unique(np.concatenate([
        np.arange(1, 4097), (1 << 24) - np.arange(0, 4097), 1 << np.arange(0, 25),
        (1 << np.arange(1, 25)) - 1, (np.sqrt(2.0) * (1 << np.arange(0, 24))).astype(np.int64),
        (np.sqrt(2.0) * (1 << np.arange(0, 24))).astype(np.int64) + 1,
        rng.integers(1, (1 << 24) + 1, size=20000)]))
    worst = 0.0
    for m in ms:
        m = int(m)
        got = oracle.ln_u1(m)
        ref = math.log(m) - 24 * math.log(2.0)
        if m == 1 << 24:
            assert got == 0.0
            continue
        assert got < 0.0
        worst = max(worst, abs(got - ref) / abs(ref))
    assert worst < 5e-7, worst


def test_sincos_polynomials_against_libm(oracle):
    fs = np.concatenate([np.arange(0, 1 << 24, 4099), [0, 1, (1 << 24) - 1, 1 << 23]]) / float(1 << 24)
    worst = 0.0
    for f in fs:
        s, c = oracle.sincos_quarter(float(np.float32(f)))
        worst = max(worst, abs(s - math.sin(math.pi / 2 * f)), abs(c - math.cos(math.pi / 2 * f)))
        assert 0.0 <= s <= 1.0 and 0.0 <= c <= 1.0
    assert worst < 2.5e-7, worst


def test_gauss_is_textbook_box_muller_of_the_words(oracle):
    seed, tid, n_pairs = 987654321987, 11, 50000
    w = oracle.noise_words(seed, tid, 0, n_pairs).astype(np.uint64)
    g = oracle.noise_gauss(seed, tid, 0, 2 * n_pairs).astype(np.float64)
    u1 = ((w[:, 0] >> 8) + 1) / 2.0 ** 24
    theta = 2 * math.pi * (w[:, 1] >> 6).astype(np.float64) / 2.0 ** 26   # (q + f)/4 of a turn
    r = np.sqrt(-2 * np.log(u1))
    assert np.abs(g[0::2] - r * np.cos(theta)).max() < 5e-6
    assert np.abs(g[1::2] - r * np.sin(theta)).max() < 5e-6
    # element addressing: odd start, arbitrary window
    g2 = oracle.noise_gauss(seed, tid, 12345, 777)
    assert (g2 == g[12345:12345 + 777].astype(np.float32)).all()


def test_gauss_distribution(oracle):
    g = oracle.noise_gauss(31337, 5, 0, 2_000_000).astype(np.float64)
    n = g.size
    assert abs(g.mean()) < 4 / math.sqrt(n)
    assert abs(g.var() - 1) < 4 * math.sqrt(2 / n)
    assert abs(stats.skew(g)) < 4 * math.sqrt(6 / n)
    assert abs(stats.kurtosis(g)) < 4 * math.sqrt(24 / n)
    assert stats.kstest(g[:500000], "norm").pvalue > 1e-4
    assert abs(np.corrcoef(g[0::2], g[1::2])[0, 1]) < 4 / math.sqrt(n / 2)
    assert np.abs(g).max() <= math.sqrt(2 * 24 * math.log(2)) + 1e-5
    tail = (np.abs(g) > 3).mean()
    assert abs(tail - 0.0026998) < 4 * math.sqrt(0.0027 / n)


@pytest.mark.parametrize("sigma", [1.0, 0.5, 2.0])
def test_delta_is_eq3_of_the_gaussian(oracle, sigma):
    # sigma a power of two: sigma*eps is exact, so the fp64 statement of Eq. 3 must agree exactly
    seed, tid, n = 2024, 9, 200000
    w = oracle.noise_words(seed, tid, 0, n // 2).astype(np.uint64)
    g = oracle.noise_gauss(seed, tid, 0, n).astype(np.float64)
    d = oracle.noise_delta(seed, tid, 0, n, sigma).astype(np.int64)
    ub = np.empty(n)
    ub[0::2] = (w[:, 2] >> 8) / 2.0 ** 24
    ub[1::2] = (w[:, 3] >> 8) / 2.0 ** 24
    t = sigma * g
    ref = np.floor(t) + (ub < (t - np.floor(t)))
    ref = np.clip(ref, -8, 7).astype(np.int64)
    assert (d == ref).all()


def test_delta_expectation_given_eps(oracle):
    # E[delta | eps] = sigma*eps: enumerate the rounding uniform on a regular grid of its 24 bits
    grid = np.arange(0, 1 << 24, 1 << 12, dtype=np.uint64)          # 4096 values of w>>8
    for eps, sigma in [(0.3, 1.0), (-0.3, 1.0), (1.75, 1.0), (-2.125, 0.7), (0.0, 1.0), (-1.0, 1.0),
                       (2.5, 0.01), (-2.5, 0.01)]:
        e32 = float(np.float32(eps))
        t = float(np.float32(sigma) * np.float32(e32))
        vals = np.array([oracle.delta_from_gauss(e32, int(v) << 8, sigma) for v in grid])
        assert set(np.unique(vals)) <= {math.floor(t), math.floor(t) + 1}
        assert abs(vals.mean() - t) <= 1.0 / 4096 + 1e-7


def test_delta_moments_and_range(oracle):
    n = 2_000_000
    d = oracle.noise_delta(777, 1, 0, n, 1.0).astype(np.float64)
    assert abs(d.mean()) < 4 * math.sqrt(1.17 / n)
    # Var(delta) = sigma^2 + E[fr(1-fr)], and the fractional part is uniform to ~1e-8 at sigma = 1
    assert abs(d.var() - (1 + 1 / 6)) < 0.01
    assert d.min() >= -6 and d.max() <= 6
    assert (oracle.noise_delta(777, 1, 0, 100000, 0.0) == 0).all()
    small = oracle.noise_delta(777, 1, 0, n, 0.01).astype(np.float64)
    assert set(np.unique(small)) <= {-1.0, 0.0, 1.0}
    assert abs(small.mean()) < 4 * math.sqrt(0.008 / n)
    assert abs(np.abs(small).mean() - 0.01 * math.sqrt(2 / math.pi)) < 4 * math.sqrt(0.008 / n)
    big = oracle.noise_delta(777, 1, 0, n, 4.0)
    assert big.min() == -8 and big.max() == 7                      # the 4-bit container


def test_delta_window_addressing(oracle):
    full = oracle.noise_delta(5, 2, 0, 4096, 1.0)
    for begin, cnt in [(1, 100), (2, 3), (999, 1001), (4095, 1)]:
        assert (oracle.noise_delta(5, 2, begin, cnt, 1.0) == full[begin:begin + cnt]).all()


def test_from_words_matches_generated_stream(oracle):
    seed, tid, n = 99, 4, 20000
    w = oracle.noise_words(seed, tid, 0, n)
    eps, delta = oracle.noise_from_words(w, 1.0)
    assert (eps.reshape(-1) == oracle.noise_gauss(seed, tid, 0, 2 * n)).all()
    assert (delta.reshape(-1) == oracle.noise_delta(seed, tid, 0, 2 * n, 1.0)).all()


def test_radius_is_correctly_rounded_sqrt_for_every_input(oracle):
    # eps0 with angle word 0 is r * CP0; sweep a slice of all 2^24 radius inputs and compare r with
    # the fp64 square root of the oracle's own ln value, rounded once to fp32
    ms = np.arange(1, (1 << 24) + 1, 257, dtype=np.uint64)
    words = np.zeros((ms.size, 4), dtype=np.uint32)
    words[:, 0] = ((ms - 1) << 8).astype(np.uint32)
    eps, _ = oracle.noise_from_words(words, 1.0)
    cp0 = np.float32(float.fromhex("0x1.fffffep-1"))
    L = np.array([oracle.ln_u1(int(m)) for m in ms[::97]], dtype=np.float32)
    r = np.sqrt((np.float32(-2.0) * L).astype(np.float64)).astype(np.float32)
    assert (eps[::97, 0] == r * cp0).all()
    assert (eps[:, 1] == 0).all()                      # sin(0) = 0: the odd lane is r * 0


# ---- an independent numpy-float32 implementation of N3-N5 of docs/NOISE_SPEC.md -------------------
# Written from the definition's text and coefficient tables (hex-float column), vectorised, with the
# fused multiply-add emulated exactly: the product of two fp32 values is exact in fp64, the fp64
# addition's rounding error is recovered with the two-sum identity, and a sum that lands exactly on
# an fp32 rounding boundary while the exact value does not is nudged off it before the final
# rounding, so that rounding once (fma) and rounding twice (fp64 then fp32) cannot differ.

def _f32(x):
    return np.asarray(x, dtype=np.float32)


def _fma32(a, b, c):
    a, b, c = (np.asarray(v, dtype=np.float32).astype(np.float64) for v in (a, b, c))
    p = a * b
    s = p + c
    bb = s - p
    err = (p - (s - bb)) + (c - bb)
    on_boundary = (s.view(np.uint64) & np.uint64(0x1FFFFFFF)) == np.uint64(0x10000000)
    toward = np.where(err > 0, np.inf, -np.inf)
    s = np.where(on_boundary & (err != 0), np.nextafter(s, toward), s)
    return s.astype(np.float32)


_H = float.fromhex
_LN2 = _f32(_H("0x1.62e430p-1"))
_LP = [_f32(_H(h)) for h in ("-0x1.000060p-1", "0x1.5559f0p-2", "-0x1.ff7476p-3", "0x1.976dd8p-3", "-0x1.6049d0p-3",
                             "0x1.4d64acp-3", "-0x1.a7d988p-4")]
_SP = [_f32(_H(h)) for h in ("0x1.921fb6p+0", "-0x1.4abbc4p-1", "0x1.4668f2p-4", "-0x1.32535ap-8", "0x1.3e17cap-13")]
_CP = [_f32(_H(h)) for h in ("0x1.fffffep-1", "-0x1.3bd3a6p+0", "0x1.03bd06p-2", "-0x1.54f61ap-6", "0x1.c1f064p-11")]


def _numpy_noise(words, sigma):
    """(eps [n,2] float32, delta [n,2] int64) of n Philox word quadruples, per N3-N6."""
    w = np.asarray(words, dtype=np.uint32).reshape(-1, 4)
    m = (w[:, 0] >> np.uint32(8)) + np.uint32(1)
    q = w[:, 1] >> np.uint32(30)
    f = ((w[:, 1] >> np.uint32(6)) & np.uint32(0xFFFFFF)).astype(np.float32) * _f32(2.0 ** -24)
    ub = [(w[:, 2] >> np.uint32(8)).astype(np.float32) * _f32(2.0 ** -24),
          (w[:, 3] >> np.uint32(8)).astype(np.float32) * _f32(2.0 ** -24)]
    # ln
    ix = m.astype(np.float32).view(np.uint32) - np.uint32(0x3F3504F3)
    e = (ix >> np.uint32(23)).astype(np.int64)
    t = ((ix & np.uint32(0x007FFFFF)) + np.uint32(0x3F3504F3)).view(np.float32) - _f32(1.0)
    p = np.full_like(t, _LP[6])
    for k in (5, 4, 3, 2, 1, 0):
        p = _fma32(p, t, _LP[k])
    l1 = _fma32(t * t, p, t)
    L = _fma32((e - 24).astype(np.float32), _LN2, l1)
    r = np.sqrt(_f32(-2.0) * L)
    # sin / cos of the first-quadrant angle
    z = f * f
    sp = np.full_like(z, _SP[4])
    cp = np.full_like(z, _CP[4])
    for k in (3, 2, 1, 0):
        sp = _fma32(sp, z, _SP[k])
        cp = _fma32(cp, z, _CP[k])
    s = f * sp
    c1 = np.select([q == 0, q == 1, q == 2], [cp, -s, -cp], s)
    s1 = np.select([q == 0, q == 1, q == 2], [s, cp, -s], -cp)
    eps = np.stack([r * c1, r * s1], axis=1).astype(np.float32)
    delta = np.empty(eps.shape, dtype=np.int64)
    for lane in range(2):
        tt = _f32(sigma) * eps[:, lane]
        fl = np.floor(tt)
        fr = tt - fl
        delta[:, lane] = np.clip(fl.astype(np.int64) + (ub[lane] < fr), -8, 7)
    return eps, delta


def test_fma_emulation_is_exact():
    # against exact rational arithmetic, on operands that provoke double rounding
    from fractions import Fraction
    rng = np.random.default_rng(3)
    a = rng.standard_normal(4000).astype(np.float32)
    b = rng.standard_normal(4000).astype(np.float32)
    c = (-(a.astype(np.float64) * b.astype(np.float64))).astype(np.float32)     # heavy cancellation
    c[::2] = rng.standard_normal(2000).astype(np.float32)
    # exact ties of the fp32 result grid: 1 + 2^-24 (+ a crumb that must break the tie)
    a = np.concatenate([a, _f32([1.0, 1.0, 1.0, 3.0])])
    b = np.concatenate([b, _f32([2.0 ** -24, 2.0 ** -24 + 2.0 ** -47, 2.0 ** -24 - 2.0 ** -48, 2.0 ** -24])])
    c = np.concatenate([c, _f32([1.0, 1.0, 1.0, 1.0 + 2.0 ** -23])])
    got = _fma32(a, b, c)

    def round_f32(x):          # nearest-even rounding of a rational to fp32 (normal range)
        if x == 0:
            return 0.0
        sign, x = (-1, -x) if x < 0 else (1, x)
        e = 0
        while x >= 2:
            x, e = x / 2, e + 1
        while x < 1:
            x, e = x * 2, e - 1
        scaled = x * (1 << 23)
        n = int(scaled)
        rem = scaled - n
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n & 1):
            n += 1
        return sign * float(Fraction(n, 1 << 23) * Fraction(2) ** e)

    for i in range(a.size):
        exact = Fraction(float(a[i])) * Fraction(float(b[i])) + Fraction(float(c[i]))
        assert float(got[i]) == round_f32(exact), i


@pytest.mark.parametrize("sigma", [1.0, 0.37, 2.5, 0.01])
def test_numpy_float32_reimplementation_matches_bit_for_bit(oracle, sigma):
    seed, tid, n = 0xA5A5A5A55A5A5A5A, 21, 60000
    w = oracle.noise_words(seed, tid, 12345, n)
    eps_ref, delta_ref = oracle.noise_from_words(w, sigma)
    eps, delta = _numpy_noise(w, sigma)
    assert (eps.view(np.uint32) == eps_ref.view(np.uint32)).all()
    assert (delta == delta_ref).all()
    # edge inputs: smallest and largest radius uniform, every quadrant, angle 0 and just below 1
    edge = np.array([[r, a, 0x80000000, 0x7FFFFF00] for r in (0, 0xFF, 0xFFFFFF00, 0xFFFFFFFF, 0x80000000)
                     for a in (0, 0x3FFFFFC0, 0x40000000, 0x7FFFFFFF, 0x80000040, 0xC0000000, 0xFFFFFFFF)], dtype=np.uint32)
    eps_ref, delta_ref = oracle.noise_from_words(edge, sigma)
    eps, delta = _numpy_noise(edge, sigma)
    assert (eps.view(np.uint32) == eps_ref.view(np.uint32)).all() and (delta == delta_ref).all()
