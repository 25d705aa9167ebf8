"""Pins for the oracle's error-feedback update and seed replay (paper §3.2 Eq. 5-8, Alg. 1,
§3.3 Alg. 2, §5 Eq. 11-13).

Invariants the paper states or implies: the telescoping identity W_T + e_T = W_0 + Σ α ĝ_t
(bit-exact for dyadic inputs), |e| <= 1/2, stagnation of stateless rounding, replayed residual =
stored residual when the window covers the whole history and no gate fires, truncation ~ γ^K,
zero fitness variance gives zero update, masked (not saturated) range edges.
"""
import numpy as np
import pytest

import workloads as wl


def _tensor(oracle, seed, out_f, in_f, bits, group, lo=None, hi=None, qmin=None, qmax=None, tid=3):
    rng = np.random.default_rng(seed)
    if qmin is None:
        qmin, qmax = (-8, 7) if bits == 4 else (-127, 127)
    lo = qmin if lo is None else lo
    hi = qmax if hi is None else hi
    q = rng.integers(lo, hi + 1, size=(out_f, in_f))
    qw = wl.pack_int4(q) if bits == 4 else q.astype(np.int8)
    return oracle.Tensor(qw, None, out_f, in_f, bits, group, qmin, qmax, tid)


def _dyadic_fitness(rng, steps, N):
    return (rng.integers(-16, 17, size=(steps, N)) / 8.0).astype(np.float32)


def test_aggregate_is_eq5_sum(oracle):
    w = _tensor(oracle, 1, 4, 16, 8, 0)
    rng = np.random.default_rng(0)
    N = 6
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    fit = rng.standard_normal(N).astype(np.float32)
    g = oracle.aggregate(w, seeds, fit, 1.0)
    deltas = np.stack([oracle.noise_delta(int(s), w.tensor_id, 0, 64, 1.0) for s in seeds]).astype(np.float64)
    ref = (fit.astype(np.float64)[:, None] * deltas).sum(axis=0).reshape(4, 16)
    assert np.abs(g - ref).max() < 1e-5
    # dyadic fitnesses: every partial sum is exact, so the fp32 chain equals the exact sum
    fit2 = _dyadic_fitness(rng, 1, N)[0]
    g2 = oracle.aggregate(w, seeds, fit2, 1.0)
    ref2 = (fit2.astype(np.float64)[:, None] * deltas).sum(axis=0).reshape(4, 16)
    assert (g2.astype(np.float64) == ref2).all()


@pytest.mark.parametrize("bits", [4, 8])
def test_telescoping_identity_bit_exact(oracle, bits):
    # N=8, sigma=1, alpha=0.5 -> c = 2^-4; fitnesses multiples of 2^-3; gamma = 1: all dyadic, so
    # (W_T - W_0) + e_T == c * sum_t g_t holds exactly, at the range edges too (gated delta in both)
    out_f, in_f, N, steps = 16, 64, 8, 12
    w = _tensor(oracle, 2, out_f, in_f, bits, 32 if bits == 4 else 0, qmin=-8 if bits == 4 else -5,
                qmax=7 if bits == 4 else 5)
    w0 = w.unpacked().copy()
    rng = np.random.default_rng(7)
    seeds = rng.integers(0, 2 ** 63, size=(steps, N), dtype=np.uint64)
    fit = _dyadic_fitness(rng, steps, N)
    e = np.zeros((out_f, in_f), dtype=np.float32)
    gsum = np.zeros((out_f, in_f), dtype=np.float64)
    stats = np.zeros(2, dtype=np.uint64)
    never_gated = np.ones((out_f, in_f), dtype=bool)
    for t in range(steps):
        before = w.unpacked()
        u, stats = oracle.update_full_residual(w, seeds[t], fit[t], 1.0, 0.5, 1.0, e, want_u=True, stats=stats)
        g = oracle.aggregate(w, seeds[t], fit[t], 1.0).astype(np.float64)
        gsum += g
        applied = w.unpacked() - before
        never_gated &= (applied == np.rint(u))
        assert (e == u - applied.astype(np.float32)).all()                 # Eq. 8
    lhs = (w.unpacked() - w0).astype(np.float64) + e.astype(np.float64)
    assert (lhs == gsum / 16.0).all()                                       # Eq. 13 (gamma = 1)
    assert np.abs(e[never_gated]).max() <= 0.5                              # |e| <= grid/2
    assert stats[0] > 0 and stats[1] > 0 and (~never_gated).any()
    assert w.unpacked().min() >= w.qmin and w.unpacked().max() <= w.qmax


def test_stateless_rounding_stagnates_but_feedback_moves(oracle):
    out_f, in_f, N, steps = 8, 64, 8, 40
    w_stateless = _tensor(oracle, 3, out_f, in_f, 8, 0, lo=-2, hi=2)
    w_feedback = w_stateless.copy()
    w0 = w_stateless.unpacked().copy()
    rng = np.random.default_rng(11)
    # the same population every step: a constant sub-threshold signal c*g, |c*g| < 1/2 everywhere
    seeds = np.tile(rng.integers(0, 2 ** 63, size=(1, N), dtype=np.uint64), (steps, 1))
    fit = np.tile(oracle.normalize_fitness(np.arange(N, dtype=np.float32)), (steps, 1))
    sigma, gamma = 1.0, 0.9
    g = oracle.aggregate(w_stateless, seeds[0], fit[0], sigma)
    alpha = float(0.4 * N * sigma / np.abs(g).max())
    c = alpha / (N * sigma)
    for t in range(steps):
        g = oracle.aggregate(w_stateless, seeds[t], fit[t], sigma)
        assert np.abs(c * g).max() < 0.5
        oracle.update(w_stateless, seeds[t], fit[t], None, None, sigma, alpha, gamma)      # hist_len = 0
        lo = max(0, t - 16)
        oracle.update(w_feedback, seeds[t], fit[t], seeds[lo:t], fit[lo:t], sigma, alpha, gamma)
    assert (w_stateless.unpacked() == w0).all()
    assert (w_feedback.unpacked() != w0).any()


def test_replay_equals_stored_residual_when_window_covers_history(oracle):
    # interior weights (|W| <= 2 in a +-127 range): no gate, so Alg. 2's proxy residual is Alg. 1's e
    out_f, in_f, N, steps = 8, 32, 6, 10
    w_full = _tensor(oracle, 4, out_f, in_f, 8, 0, lo=-2, hi=2)
    w_replay = w_full.copy()
    rng = np.random.default_rng(13)
    seeds = rng.integers(0, 2 ** 63, size=(steps, N), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(steps)])
    sigma, alpha, gamma = 1.0, 1.5, 0.9
    e = np.zeros((out_f, in_f), dtype=np.float32)
    moved = 0
    for t in range(steps):
        rep = oracle.replay_residual(w_replay, seeds[:t], fit[:t], N, sigma, alpha, gamma)
        assert (rep == e).all()
        before = w_full.unpacked()
        oracle.update_full_residual(w_full, seeds[t], fit[t], sigma, alpha, gamma, e)
        oracle.update(w_replay, seeds[t], fit[t], seeds[:t], fit[:t], sigma, alpha, gamma)
        assert (w_full.unpacked() == w_replay.unpacked()).all()
        moved += int((w_full.unpacked() != before).sum())
    assert moved > 50


def test_replay_closed_form_without_rounding(oracle):
    out_f, in_f, N, K = 4, 32, 8, 6
    w = _tensor(oracle, 5, out_f, in_f, 8, 0, lo=-2, hi=2)
    rng = np.random.default_rng(17)
    seeds = rng.integers(0, 2 ** 63, size=(K, N), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(K)])
    sigma, alpha, gamma = 1.0, 0.02, 0.9
    c = alpha / (N * sigma)
    rep = oracle.replay_residual(w, seeds, fit, N, sigma, alpha, gamma).astype(np.float64)
    ref = np.zeros((out_f, in_f))
    for j in range(K):
        ref += c * gamma ** (K - 1 - j) * oracle.aggregate(w, seeds[j], fit[j], sigma).astype(np.float64)
    assert np.abs(ref).max() < 0.5
    assert np.abs(rep - ref).max() < 1e-6


def test_window_truncation_decays_like_gamma_to_the_K(oracle):
    out_f, in_f, N, steps = 4, 64, 8, 60
    w = _tensor(oracle, 6, out_f, in_f, 8, 0, lo=-2, hi=2)
    rng = np.random.default_rng(19)
    seeds = rng.integers(0, 2 ** 63, size=(steps, N), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(steps)])
    sigma, alpha, gamma = 1.0, 0.02, 0.9          # small alpha: no rounding fires, pure decay
    full = oracle.replay_residual(w, seeds, fit, N, sigma, alpha, gamma)
    errs = []
    for K in (10, 20, 40):
        part = oracle.replay_residual(w, seeds[steps - K:], fit[steps - K:], N, sigma, alpha, gamma)
        errs.append(np.abs(part - full).max())
    scale = np.abs(full).max()
    assert errs[0] > errs[1] > errs[2]
    for K, err in zip((10, 20, 40), errs):
        assert err <= 3 * scale * gamma ** K / (1 - gamma) + 1e-7


def test_zero_fitness_variance_gives_zero_update(oracle):
    fit = oracle.normalize_fitness(np.full(8, 3.25, dtype=np.float32))
    assert (fit == 0).all()
    assert (oracle.normalize_fitness(np.array([1.5], dtype=np.float32)) == 0).all()
    w = _tensor(oracle, 7, 8, 32, 4, 32)
    w0 = w.unpacked().copy()
    rng = np.random.default_rng(23)
    seeds = rng.integers(0, 2 ** 63, size=(5, 8), dtype=np.uint64)
    zeros = np.zeros((5, 8), dtype=np.float32)
    stats = oracle.update(w, seeds[4], zeros[4], seeds[:4], zeros[:4], 1.0, 0.5, 0.9)
    assert (w.unpacked() == w0).all() and stats[0] == 0 and stats[1] == 0
    assert (oracle.replay_residual(w, seeds[:4], zeros[:4], 8, 1.0, 0.5, 0.9) == 0).all()


def test_normalize_fitness_is_population_zscore(oracle):
    rng = np.random.default_rng(29)
    r = (rng.standard_normal(30) * 3 + 2).astype(np.float32)
    f = oracle.normalize_fitness(r)
    ref = (r.astype(np.float64) - r.astype(np.float64).mean()) / r.astype(np.float64).std()
    assert np.abs(f - ref).max() < 1e-6
    assert abs(f.astype(np.float64).mean()) < 1e-6 and abs(f.astype(np.float64).std() - 1) < 1e-6


def test_gate_masks_at_the_range_edges(oracle):
    # 4x8 INT4 layer holding every nibble value twice; one strong member pushes |u| past 1.5 so
    # that rounded updates of +-1 and +-2 occur. Mask, not saturate: 6 + 2 stays 6.
    q = np.tile(np.arange(-8, 8), 2).reshape(4, 8)
    w = oracle.Tensor(wl.pack_int4(q), None, 4, 8, 4, 8, -8, 7, 5)
    N, sigma, alpha, gamma = 4, 1.0, 6.0, 0.9
    rng = np.random.default_rng(31)
    seen_masked_two = False
    for trial in range(200):
        w.qweight[:] = wl.pack_int4(q)
        seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
        fit = oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32))
        g = oracle.aggregate(w, seeds, fit, sigma)
        u = (np.float32(alpha / (N * sigma)) * g).astype(np.float32)     # hist_len = 0: u = c*g exactly one op
        d = np.rint(u).astype(np.int64)
        ok = (q + d >= -8) & (q + d <= 7)
        expect = np.where(ok, q + d, q)
        stats = oracle.update(w, seeds, fit, None, None, sigma, alpha, gamma)
        assert (w.unpacked() == expect).all()
        assert stats[0] == (ok & (d != 0)).sum() and stats[1] == (~ok).sum()
        seen_masked_two |= bool(((np.abs(d) >= 2) & ~ok & (np.abs(q + np.sign(d)) <= 7) & (q + np.sign(d) >= -8)).any())
    assert seen_masked_two


def test_replay_gates_against_current_weights(oracle):
    # a weight on qmax with a positive simulated update keeps u as its proxy residual (Alg. 2)
    out_f, in_f, N = 2, 16, 4
    q = np.full((out_f, in_f), 7)
    q[1] = 0
    w = oracle.Tensor(wl.pack_int4(q), None, out_f, in_f, 4, 16, -8, 7, 8)
    rng = np.random.default_rng(37)
    seeds = rng.integers(0, 2 ** 63, size=(1, N), dtype=np.uint64)
    fit = oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32))[None]
    sigma, alpha, gamma = 1.0, 4.0, 0.9
    u = (np.float32(alpha / (N * sigma)) * oracle.aggregate(w, seeds[0], fit[0], sigma)).astype(np.float32)
    rep = oracle.replay_residual(w, seeds, fit, N, sigma, alpha, gamma)
    d = np.rint(u)
    edge_pos = d[0] > 0
    assert edge_pos.any()
    assert (rep[0][edge_pos] == u[0][edge_pos]).all()                     # masked: residual keeps u
    assert (rep[0][~edge_pos] == (u[0] - d[0])[~edge_pos]).all()
    assert (rep[1] == (u[1] - d[1])).all()                                # interior row: plain Eq. 8


def test_row_subset_update_equals_full(oracle):
    out_f, in_f, N, K = 32, 64, 5, 3
    w_full = _tensor(oracle, 9, out_f, in_f, 4, 32)
    w_part = w_full.copy()
    w0 = w_full.unpacked().copy()
    rng = np.random.default_rng(41)
    seeds = rng.integers(0, 2 ** 63, size=(K + 1, N), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(K + 1)])
    args = (1.0, 1.2, 0.9)
    oracle.update(w_full, seeds[K], fit[K], seeds[:K], fit[:K], *args)
    rows = np.array([0, 5, 31], dtype=np.int32)
    oracle.update(w_part, seeds[K], fit[K], seeds[:K], fit[:K], *args, rows=rows)
    assert (w_part.unpacked()[rows] == w_full.unpacked()[rows]).all()
    other = np.setdiff1d(np.arange(out_f), rows)
    assert (w_part.unpacked()[other] == w0[other]).all()
    assert (w_full.unpacked() != w0).any()


def test_invalid_arguments(oracle):
    w = _tensor(oracle, 10, 4, 16, 4, 16)
    seeds = np.arange(4, dtype=np.uint64)
    fit = np.zeros(4, dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.update(w, seeds, fit, None, None, 0.0, 0.5, 0.9)           # sigma = 0: c undefined
    with pytest.raises(ValueError):
        oracle.replay_residual(w, None, None, 4, -1.0, 0.5, 0.9)
