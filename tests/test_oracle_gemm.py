"""Pins for the oracle's perturbed quantised GEMM (paper Alg. 1 inner loop, §3.2 Eq. 4, App. A.1).

Special cases that reduce to a library matmul, brute-force loops on tiny layers, and the W8A8
integer path against a numpy statement of symmetric per-token quantisation.
"""
import numpy as np
import pytest

import workloads as wl


def _dequant(oracle, w):
    q = w.unpacked().astype(np.float64)
    s = wl.f16_bits_to_f32(w.scales).astype(np.float64)
    if w.group_size:
        s = np.repeat(s, w.group_size, axis=1)
    else:
        s = s[:, None]
    return q * s


def _bf16_ulp_diff(a_bits, b_bits):
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, 0x8000 - b, b)  # monotone map of sign-magnitude patterns
    return np.abs(key(a_bits) - key(b_bits))


@pytest.mark.parametrize("bits,group", [(4, 32), (4, 128), (8, 0)])
def test_sigma_zero_is_a_plain_matmul(oracle, bits, group):
    out_f, in_f, N, T = 48, 256, 3, 5
    qw, sc, qmin, qmax = wl.random_tensor(10 + bits, out_f, in_f, bits, group)
    w = oracle.Tensor(qw, sc, out_f, in_f, bits, group, qmin, qmax, 4)
    rng = np.random.default_rng(0)
    x = wl.f32_to_bf16_bits(rng.standard_normal((N, T, in_f)).astype(np.float32))
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    y = oracle.perturbed_qgemm(w, seeds, 0.0, x)
    ref = wl.bf16_bits_to_f32(x).astype(np.float64) @ _dequant(oracle, w).T
    ref_bits = wl.f32_to_bf16_bits(ref.astype(np.float32))
    d = _bf16_ulp_diff(y, ref_bits)
    assert d.max() <= 1 and (d > 0).mean() < 0.01
    # mask = 0 is the same as sigma = 0, member by member
    y_mask = oracle.perturbed_qgemm(w, seeds, 1.0, x, perturb_mask=np.array([0, 1, 0], dtype=np.uint8))
    y_pert = oracle.perturbed_qgemm(w, seeds, 1.0, x)
    assert (y_mask[0] == y[0]).all() and (y_mask[2] == y[2]).all() and (y_mask[1] == y_pert[1]).all()
    assert (y_pert != y).mean() > 0.5


@pytest.mark.parametrize("bits,group", [(4, 4), (8, 0)])
def test_perturbed_brute_force_tiny(oracle, bits, group):
    out_f, in_f, N, T, sigma, tid = 8, 8, 4, 3, 1.0, 21
    qw, sc, qmin, qmax = wl.random_tensor(3, out_f, in_f, bits, group)
    if bits == 8:
        qmin, qmax = -3, 3   # tight range so that the gate fires on a tiny layer
        qw = np.clip(qw, qmin, qmax).astype(np.int8)
    w = oracle.Tensor(qw, sc, out_f, in_f, bits, group, qmin, qmax, tid)
    rng = np.random.default_rng(5)
    x = wl.f32_to_bf16_bits(rng.standard_normal((N, T, in_f)).astype(np.float32))
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    y = oracle.perturbed_qgemm(w, seeds, sigma, x)
    q = w.unpacked()
    s = wl.f16_bits_to_f32(w.scales).astype(np.float64)
    xf = wl.bf16_bits_to_f32(x).astype(np.float64)
    gated = 0
    for i in range(N):
        delta = oracle.noise_delta(int(seeds[i]), tid, 0, out_f * in_f, sigma).reshape(out_f, in_f)
        for n in range(out_f):
            wp = []
            for k in range(in_f):
                v = int(q[n, k]) + int(delta[n, k])
                if qmin <= v <= qmax:
                    wp.append(v)
                else:
                    wp.append(int(q[n, k]))
                    gated += 1
            for t in range(T):
                acc = 0.0
                for k in range(in_f):
                    sc_nk = s[n, k // group] if group else s[n]
                    acc += sc_nk * xf[i, t, k] * wp[k]
                ref = wl.f32_to_bf16_bits(np.array([acc], dtype=np.float32))[0]
                assert _bf16_ulp_diff(np.array([y[i, t, n]]), np.array([ref]))[0] <= 1
    assert gated > 0


def test_row_subset_equals_full(oracle):
    out_f, in_f, N, T = 64, 128, 2, 4
    qw, sc, qmin, qmax = wl.random_tensor(8, out_f, in_f, 4, 32)
    w = oracle.Tensor(qw, sc, out_f, in_f, 4, 32, qmin, qmax, 2)
    rng = np.random.default_rng(9)
    x = wl.f32_to_bf16_bits(rng.standard_normal((N, T, in_f)).astype(np.float32))
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    full = oracle.perturbed_qgemm(w, seeds, 1.0, x)
    rows = np.array([0, 7, 33, 63], dtype=np.int32)
    part = oracle.perturbed_qgemm(w, seeds, 1.0, x, rows=rows)
    assert (part[:, :, rows] == full[:, :, rows]).all()
    other = np.setdiff1d(np.arange(out_f), rows)
    assert (part[:, :, other] == 0).all()


def test_w8a8_integer_path(oracle):
    out_f, in_f, N, T, tid = 16, 64, 2, 6, 77
    qw, sc, qmin, qmax = wl.random_tensor(12, out_f, in_f, 8, 0)
    w = oracle.Tensor(qw, sc, out_f, in_f, 8, 0, qmin, qmax, tid)
    rng = np.random.default_rng(4)
    xf = rng.standard_normal((N, T, in_f)).astype(np.float32)
    xf[1, 2, :] = 0.0                                               # an all-zero token
    x = wl.f32_to_bf16_bits(xf)
    xv = wl.bf16_bits_to_f32(x)
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    y = oracle.perturbed_qgemm(w, seeds, 1.0, x, act_mode=1)
    # symmetric dynamic per-token int8 (scale = max|x| / 127), exact integer accumulation
    a = (np.abs(xv).max(axis=2) / np.float32(127.0)).astype(np.float32)
    a = np.where(a == 0, np.float32(1), a)
    xq = np.clip(np.rint(xv / a[:, :, None]), -127, 127).astype(np.int64)
    q = w.unpacked().astype(np.int64)
    s = wl.f16_bits_to_f32(w.scales)
    for i in range(N):
        delta = oracle.noise_delta(int(seeds[i]), tid, 0, out_f * in_f, 1.0).reshape(out_f, in_f).astype(np.int64)
        v = q + delta
        wp = np.where((v >= qmin) & (v <= qmax), v, q)
        acc = xq[i] @ wp.T                                          # [T,out] exact
        ref = (acc.astype(np.float32) * a[i][:, None]) * s[None, :]
        assert (wl.f32_to_bf16_bits(ref.astype(np.float32)) == y[i]).all()
    assert (y[1, 2] == 0).all() or (y[1, 2] == 0x8000).all() or set(np.unique(y[1, 2])) <= {0, 0x8000}
    # act_mode 1 needs int8 weights with one scale per row
    qw4, sc4, a4, b4 = wl.random_tensor(1, 8, 64, 4, 32)
    w4 = oracle.Tensor(qw4, sc4, 8, 64, 4, 32, a4, b4, 1)
    with pytest.raises(ValueError):
        oracle.perturbed_qgemm(w4, seeds, 1.0, x[:, :, :64], act_mode=1)


def test_int4_nibble_order(oracle):
    # element 2b sits in the low nibble of byte b, element 2b+1 in the high nibble
    out_f, in_f = 2, 8
    q = np.array([[-8, 7, 1, -1, 0, 3, -4, 5], [2, -2, 6, -6, 7, -8, 0, 1]])
    packed = wl.pack_int4(q)
    assert packed[0, 0] == ((7 << 4) | 0x8) and packed[0, 1] == ((0xF << 4) | 1)
    sc = wl.f16_bits(np.ones((out_f, 1), dtype=np.float32))
    w = oracle.Tensor(packed, sc, out_f, in_f, 4, 8, -8, 7, 1)
    assert (w.unpacked() == q).all()
    # one-hot activations read the weights back through the oracle GEMM
    x = wl.f32_to_bf16_bits(np.eye(in_f, dtype=np.float32)[None])   # N=1, T=in_f
    y = wl.bf16_bits_to_f32(oracle.perturbed_qgemm(w, [1], 0.0, x))[0]
    assert (y.T == q).all()


def test_output_rounding_is_nearest_even_bfloat16(oracle):
    """The final rounding to bfloat16 on exact ties and next to them, against hand-placed values:
    with unit weights and scale 1 the output is x0 + x1 exactly, and x1 = 2^-8 puts it half-way
    between two bfloat16 neighbours of x0 in [1, 2). Truncation, round-half-up and round-half-away
    each miss at least one of the cases."""
    one = wl.pack_int4(np.ones((1, 2), dtype=np.int64))
    scale = wl.f16_bits(np.ones((1, 1), dtype=np.float32))
    w = oracle.Tensor(one, scale, 1, 2, 4, 2, -8, 7, 1)
    cases = [
        (0x3F80, 0x3B80, 0x3F80),   # 1 + 2^-8: tie, lower neighbour 1.0 is even
        (0x3F81, 0x3B80, 0x3F82),   # 1 + 2^-7 + 2^-8: tie, upper neighbour is even
        (0xBF80, 0xBB80, 0xBF80),   # the same two, negated
        (0xBF81, 0xBB80, 0xBF82),
        (0x3F80, 0x3B81, 0x3F81),   # just above the tie: up
        (0x3F81, 0x3B7F, 0x3F81),   # just below the tie: down
        (0x3F80, 0x3A80, 0x3F80),   # a quarter of a step: down
        (0x3F80, 0x3BC0, 0x3F81),   # three quarters of a step: up
    ]
    x = np.array([[[a, b]] for a, b, _ in cases], dtype=np.uint16)            # [N=8, T=1, in=2]
    y = oracle.perturbed_qgemm(w, np.zeros(len(cases), dtype=np.uint64), 0.0, x)
    assert [int(v) for v in y.reshape(-1)] == [c for _, _, c in cases]
    # the exact values behind the table, restated in rationals
    from fractions import Fraction
    def val(bits):
        return Fraction(float(wl.bf16_bits_to_f32(np.array([bits], dtype=np.uint16))[0]))
    for a, b, c in cases:
        exact = val(a) + val(b)
        lo_hi = sorted([val(c), val(c ^ 1)], key=lambda v: abs(v - exact))
        assert abs(val(c) - exact) <= abs(lo_hi[1] - exact)
