"""Pins for the oracle's stateless baselines (paper §5: W ← W + Q(α ĝ), Eq. 9-10): deterministic
rounding stagnates (pinned in test_oracle_update.py), stochastic rounding is unbiased per step but
its errors add up as a random walk, while error feedback keeps the deviation from the ideal
trajectory at one residual."""
import numpy as np
import pytest

import workloads as wl
from test_oracle_update import _tensor


def _uniforms(oracle, round_seed, tensor_id, n_pairs):
    """Rounding uniforms of the step, from the raw Philox routine: stream tag 1, words 2 and 3."""
    ub = np.empty((n_pairs, 2), dtype=np.float32)
    key = (round_seed & 0xFFFFFFFF, round_seed >> 32)
    for p in range(n_pairs):
        w = oracle.philox4x32_10((p & 0xFFFFFFFF, p >> 32, tensor_id, 1), key)
        ub[p, 0] = np.float32(w[2] >> 8) * np.float32(2.0 ** -24)
        ub[p, 1] = np.float32(w[3] >> 8) * np.float32(2.0 ** -24)
    return ub.reshape(-1)


def test_step_is_floor_plus_bernoulli_of_the_fraction(oracle):
    out_f, in_f, N = 4, 32, 6
    w = _tensor(oracle, 3, out_f, in_f, 8, 0, lo=-3, hi=3)        # interior: the gate cannot fire
    rng = np.random.default_rng(1)
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    fit = oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32))
    sigma, alpha, round_seed = 1.0, 4.0, 0x0123456789ABCDEF
    g = oracle.aggregate(w, seeds, fit, sigma).reshape(-1)
    u = (np.float32(alpha / (N * sigma)) * g).astype(np.float32)
    before = w.unpacked().reshape(-1).copy()
    oracle.update_stochastic_rounding(w, seeds, fit, sigma, alpha, round_seed)
    step = w.unpacked().reshape(-1) - before
    fl = np.floor(u)
    assert ((step == fl) | (step == fl + 1)).all()
    ub = _uniforms(oracle, round_seed, w.tensor_id, out_f * in_f // 2)
    assert (step == fl + (ub < (u - fl))).all()
    assert (step != np.rint(u)).any()                              # not round-to-nearest in disguise
    # the rounding stream is not the perturbation stream of the same seed
    assert (oracle.philox4x32_10((0, 0, 3, 1), (5, 0)) != oracle.philox4x32_10((0, 0, 3, 0), (5, 0))).all()


def test_integer_updates_are_applied_exactly(oracle):
    out_f, in_f, N = 4, 16, 4
    w = _tensor(oracle, 4, out_f, in_f, 8, 0, lo=-3, hi=3)
    seeds = np.arange(10, 10 + N, dtype=np.uint64)
    fit = np.float32([2, -1, 1, -2])
    g = oracle.aggregate(w, seeds, fit, 1.0)                      # integers
    for round_seed in (1, 2, 99):
        wc = w.copy()
        oracle.update_stochastic_rounding(wc, seeds, fit, 1.0, float(N), round_seed)   # c = 1
        assert (wc.unpacked() - w.unpacked() == g).all()
    assert (g != 0).any()


def test_unbiased_over_rounding_seeds(oracle):
    out_f, in_f, N, trials = 2, 32, 6, 600
    w = _tensor(oracle, 5, out_f, in_f, 8, 0, lo=-3, hi=3)
    rng = np.random.default_rng(2)
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    fit = oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32))
    alpha = 1.2
    u = (np.float32(alpha / N) * oracle.aggregate(w, seeds, fit, 1.0)).astype(np.float64)
    acc = np.zeros_like(u)
    for r in range(trials):
        wc = w.copy()
        oracle.update_stochastic_rounding(wc, seeds, fit, 1.0, alpha, 1000 + r)
        acc += wc.unpacked() - w.unpacked()
    fr = u - np.floor(u)
    tol = 4.5 * np.sqrt(fr * (1 - fr) / trials) + 1e-9
    assert (np.abs(acc / trials - u) <= tol).all()
    assert (fr > 0.05).any()


def test_random_walk_against_error_feedback(oracle):
    # the same population every step: a constant signal u = c·g with |u| < 1/2 per element
    out_f, in_f, N, steps = 8, 64, 8, 64
    w_sr = _tensor(oracle, 6, out_f, in_f, 8, 0, lo=-2, hi=2)
    w_ef = w_sr.copy()
    w0 = w_sr.unpacked().astype(np.float64)
    rng = np.random.default_rng(3)
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    fit = oracle.normalize_fitness(np.arange(N, dtype=np.float32))
    g = oracle.aggregate(w_sr, seeds, fit, 1.0)
    alpha = float(0.4 * N / np.abs(g).max())
    u = (np.float32(alpha / N) * g).astype(np.float64)
    e = np.zeros((out_f, in_f), dtype=np.float32)
    for t in range(steps):
        oracle.update_stochastic_rounding(w_sr, seeds, fit, 1.0, alpha, 77 + t)
        oracle.update_full_residual(w_ef, seeds, fit, 1.0, alpha, 1.0, e)
    ideal = steps * u
    err_ef = w_ef.unpacked() - w0 - ideal
    err_sr = w_sr.unpacked() - w0 - ideal
    assert np.abs(err_ef).max() <= 0.5 + 1e-3                       # one residual (Eq. 13)
    fr = u - np.floor(u)
    predicted = np.sqrt((steps * fr * (1 - fr)).mean())             # random-walk RMS
    rms_sr = np.sqrt((err_sr ** 2).mean())
    assert 0.75 * predicted <= rms_sr <= 1.25 * predicted
    assert rms_sr > 3 * np.sqrt((err_ef ** 2).mean())


def test_range_edge_is_masked_and_counted(oracle):
    out_f, in_f, N = 4, 32, 4
    w = _tensor(oracle, 7, out_f, in_f, 4, 0, lo=7, hi=7)
    seeds = np.arange(1, N + 1, dtype=np.uint64)
    fit = np.float32([1.5, -0.5, -1.5, 0.5])
    g = oracle.aggregate(w, seeds, fit, 1.0)
    stats = oracle.update_stochastic_rounding(w, seeds, fit, 1.0, 8.0 * N, 5)     # c = 8: steps of several units
    after = w.unpacked()
    assert after.max() <= 7 and after.min() >= -8
    up = g > 0.2                                                   # u >= 1.6: Δ >= 1 whatever the uniform
    assert up.any() and (after[up] == 7).all()
    assert stats[1] >= up.sum() and stats[0] == (after != 7).sum()


def test_a_zero_update_is_never_counted_as_gated(oracle):
    """Eq. 4 masks an update that would leave the range; with nothing to mask nothing is counted,
    also where the stored weight itself lies outside [qmin, qmax] (a -8 nibble under the symmetric
    range [-7, 7] of App. A.1). Both update rules use the same counter rule."""
    out_f, in_f, N = 4, 32, 4
    q = np.full((out_f, in_f), -8, dtype=np.int64)
    q[:, ::3] = 2
    seeds = np.arange(1, N + 1, dtype=np.uint64)
    mk = lambda: oracle.Tensor(wl.pack_int4(q), None, out_f, in_f, 4, 0, -7, 7, 3)   # noqa: E731
    # zero fitness: every update is zero -> no change, nothing gated
    for call in (lambda w: oracle.update_stochastic_rounding(w, seeds, np.zeros(N, np.float32), 1.0, 2.0, 5),
                 lambda w: oracle.update(w, seeds, np.zeros(N, np.float32), None, None, 1.0, 2.0, 0.9)):
        w = mk()
        stats = call(w)
        assert (stats == 0).all() and (w.unpacked() == q).all()
    # non-zero fitness: exactly the elements whose rounded update is non-zero and masked are counted
    fit = np.float32([1.5, -0.5, -1.5, 0.5])
    w = mk()
    g = oracle.aggregate(w, seeds, fit, 1.0)
    u = (np.float32(2.0 / N) * g).astype(np.float32)
    d = np.rint(u).astype(np.int64)
    stats = oracle.update(w, seeds, fit, None, None, 1.0, 2.0, 0.9)
    ok = (q + d >= -7) & (q + d <= 7)
    assert stats[0] == ((d != 0) & ok).sum() and stats[1] == ((d != 0) & ~ok).sum() and stats[1] > 0
    assert (w.unpacked() == np.where(ok, q + d, q)).all()
    # the stochastic rule on the same tensor: Δ is floor or floor + 1; the counter follows the Δ taken
    w = mk()
    stats = oracle.update_stochastic_rounding(w, seeds, fit, 1.0, 2.0, 9)
    step = w.unpacked() - q
    ub = _uniforms(oracle, 9, 3, out_f * in_f // 2).reshape(out_f, in_f)
    d = (np.floor(u) + (ub < (u - np.floor(u)))).astype(np.int64)
    ok = (q + d >= -7) & (q + d <= 7)
    assert (step == np.where(ok, d, 0)).all()
    assert stats[0] == ((d != 0) & ok).sum() and stats[1] == ((d != 0) & ~ok).sum() and stats[1] > 0
