"""Pins for the oracle's Full-Residual step with a binary16 residual (paper Alg. 1: residuals
initialised as FP16; §4 residual ablation: the Full-Residual variant stores FP16 residuals).

The half conversions are checked against numpy's float16 (a different implementation); the step is
tied to the fp32-residual step (pinned in test_oracle_update.py) through cases where the two must
agree exactly, and to numpy's rounding where they differ.
"""
import numpy as np
import pytest

import workloads as wl
from test_oracle_update import _tensor, _dyadic_fitness


def test_half_decoding_all_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    for h in range(0, 65536, 7):           # every 7th pattern plus the edges below: ~9400 calls
        got = np.float32(oracle.f16_to_f32(h))
        assert (np.isnan(got) and np.isnan(ref[h])) or got.view(np.uint32) == ref[h].view(np.uint32), h
    for h in (0x0000, 0x8000, 0x0001, 0x03FF, 0x0400, 0x7BFF, 0xFBFF, 0x7C00, 0xFC00, 0x3C00, 0xBC00):
        assert np.float32(oracle.f16_to_f32(h)).view(np.uint32) == ref[h].view(np.uint32), hex(h)


def test_half_encoding_rounds_to_nearest_even_and_saturates(oracle):
    rng = np.random.default_rng(5)
    vals = np.concatenate([
        rng.standard_normal(3000).astype(np.float32),                       # residual-sized values
        (rng.standard_normal(2000) * 1e-4).astype(np.float32),              # near and inside the subnormal range
        (rng.standard_normal(500) * 1e-7).astype(np.float32),
        (rng.standard_normal(1500) * 3000).astype(np.float32),
        np.float32([0.0, -0.0, 0.5, -0.5, 65504.0, -65504.0, 65503.9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -24,
                    2.0 ** -14, 2.0 ** -14 - 2.0 ** -25]),
    ])
    # exact ties between neighbouring halves: (2m+1) * 2^-12 around 1.0 and in the subnormals
    m = np.arange(1024, 1100)
    vals = np.concatenate([vals, ((2 * m + 1) * 2.0 ** -11).astype(np.float32), ((2 * m[:20] - 2047) * 2.0 ** -25).astype(np.float32)])
    vals = vals[np.abs(vals) <= 65504.0]
    ref = vals.astype(np.float16).view(np.uint16)
    for v, r in zip(vals, ref):
        assert oracle.f32_to_f16_sat(v) == int(r), (float(v), hex(int(r)))
    # beyond the largest finite half: saturate, never infinity
    for v, r in ((65520.0, 0x7BFF), (1e6, 0x7BFF), (-65520.0, 0xFBFF), (-3e9, 0xFBFF), (np.inf, 0x7BFF), (-np.inf, 0xFBFF)):
        assert oracle.f32_to_f16_sat(v) == r


@pytest.mark.parametrize("bits", [4, 8])
def test_dyadic_run_equals_fp32_residual_run(oracle, bits):
    # c = 2^-4, fitnesses multiples of 2^-3, gamma = 1: every residual is a multiple of 2^-7 below
    # 16 in magnitude, exactly representable in binary16, so both variants must walk identically
    out_f, in_f, N, steps = 16, 64, 8, 12
    w16 = _tensor(oracle, 2, out_f, in_f, bits, 32 if bits == 4 else 0, qmin=-8 if bits == 4 else -5,
                  qmax=7 if bits == 4 else 5)
    w32 = w16.copy()
    rng = np.random.default_rng(7)
    seeds = rng.integers(0, 2 ** 63, size=(steps, N), dtype=np.uint64)
    fit = _dyadic_fitness(rng, steps, N)
    e32 = np.zeros((out_f, in_f), dtype=np.float32)
    e16 = np.zeros((out_f, in_f), dtype=np.uint16)
    s32 = np.zeros(2, dtype=np.uint64)
    s16 = np.zeros(2, dtype=np.uint64)
    for t in range(steps):
        oracle.update_full_residual(w32, seeds[t], fit[t], 1.0, 0.5, 1.0, e32, stats=s32)
        oracle.update_full_residual_f16(w16, seeds[t], fit[t], 1.0, 0.5, 1.0, e16, stats=s16)
        assert np.abs(e32).max() < 16
        assert (w16.qweight == w32.qweight).all()
        assert (e16.view(np.float16).astype(np.float32) == e32).all()
    assert (s16 == s32).all() and s16[0] > 0 and s16[1] > 0
    assert (e16 != 0).any()


def test_general_step_is_fp32_step_on_decoded_residual_then_rounded(oracle):
    out_f, in_f, N, steps = 12, 40, 6, 8
    w16 = _tensor(oracle, 9, out_f, in_f, 4, 0)
    rng = np.random.default_rng(23)
    seeds = rng.integers(0, 2 ** 63, size=(steps, N), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(steps)])
    sigma, alpha, gamma = 1.0, 1.5, 0.9
    e16 = np.zeros((out_f, in_f), dtype=np.uint16)
    inexact = 0
    for t in range(steps):
        ref_w = w16.copy()
        ref_e = e16.view(np.float16).astype(np.float32)          # numpy decodes
        oracle.update_full_residual(ref_w, seeds[t], fit[t], sigma, alpha, gamma, ref_e)
        oracle.update_full_residual_f16(w16, seeds[t], fit[t], sigma, alpha, gamma, e16)
        assert (w16.qweight == ref_w.qweight).all()
        assert (e16 == ref_e.astype(np.float16).view(np.uint16)).all()    # numpy rounds
        inexact += int((e16.view(np.float16).astype(np.float32) != ref_e).sum())
    assert inexact > 100          # the rounding to half really happens in this run


def test_gated_residual_saturates_at_largest_half(oracle):
    out_f, in_f, N = 4, 32, 4
    w = _tensor(oracle, 1, out_f, in_f, 4, 0, lo=7, hi=7)      # every weight on the upper edge
    seeds = np.arange(1, N + 1, dtype=np.uint64)
    fit = np.float32([1.5, -0.5, -1.5, 0.5])
    e16 = np.zeros((out_f, in_f), dtype=np.uint16)
    g = oracle.aggregate(w, seeds, fit, 1.0)
    alpha = 4e6                                                 # c = 1e6: |u| = 1e6 |g|
    before = w.qweight.copy()
    oracle.update_full_residual_f16(w, seeds, fit, 1.0, alpha, 0.9, e16)
    e = e16.view(np.float16).astype(np.float32)
    big = np.abs(g) >= 1.0
    assert big.any() and (e[big] == np.sign(g[big]) * 65504.0).all()
    assert (w.qweight == before)[big.reshape(out_f, -1, 2).all(axis=2)].all()      # gated: bytes untouched
    assert np.isfinite(e).all()
