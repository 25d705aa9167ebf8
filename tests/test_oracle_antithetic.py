"""Pins for antithetic perturbation pairs in the oracle (paper App. A.1: "antithetic perturbation
pairs"): members 2j and 2j+1 share one seed and use +δ_j and -δ_j. Everything else is Eq. 4-8
unchanged, so each pin restates the pair semantics against the separately pinned single-member
primitives (noise_delta, the non-antithetic GEMM of the unperturbed weights)."""
import numpy as np

import workloads as wl


def _tensor(oracle, seed, out_f, in_f, bits, group, scales=True):
    qw, sc, qmin, qmax = wl.random_tensor(seed, out_f, in_f, bits, group)
    return oracle.Tensor(qw, sc if scales else None, out_f, in_f, bits, group, qmin, qmax, 31)


def test_aggregate_is_the_signed_sum(oracle):
    w = _tensor(oracle, 1, 4, 32, 8, 0, scales=False)
    rng = np.random.default_rng(0)
    N = 10
    pair_seeds = rng.integers(0, 2 ** 63, size=N // 2, dtype=np.uint64)
    fit = (rng.integers(-16, 17, size=N) / 8.0).astype(np.float32)      # dyadic: the fp32 chain is exact
    g = oracle.aggregate(w, pair_seeds, fit, 1.0, antithetic=True)
    ref = np.zeros(4 * 32)
    for j, s in enumerate(pair_seeds):
        d = oracle.noise_delta(int(s), w.tensor_id, 0, 4 * 32, 1.0).astype(np.float64)
        ref += (float(fit[2 * j]) - float(fit[2 * j + 1])) * d
    assert (g.reshape(-1).astype(np.float64) == ref).all()
    # a symmetric fitness (F+ == F-) carries no signal: the estimate vanishes identically
    sym = np.repeat(fit[::2], 2)
    assert (oracle.aggregate(w, pair_seeds, sym, 1.0, antithetic=True) == 0).all()


def test_gemm_odd_members_use_the_negated_perturbation(oracle):
    out_f, in_f, N, T = 16, 64, 6, 5
    w = _tensor(oracle, 2, out_f, in_f, 4, 32)
    rng = np.random.default_rng(3)
    x = wl.f32_to_bf16_bits(rng.standard_normal((N, T, in_f)).astype(np.float32))
    pair_seeds = rng.integers(0, 2 ** 63, size=N // 2, dtype=np.uint64)
    y = oracle.perturbed_qgemm(w, pair_seeds, 1.0, x, antithetic=True)
    # even members: identical to the plain call with that seed
    plain = oracle.perturbed_qgemm(w, np.repeat(pair_seeds, 2), 1.0, x)
    assert (y[0::2] == plain[0::2]).all()
    # odd members: the unperturbed GEMM of the explicitly mirrored, gated weights
    q = w.unpacked()
    for j, s in enumerate(pair_seeds):
        d = oracle.noise_delta(int(s), w.tensor_id, 0, out_f * in_f, 1.0).reshape(out_f, in_f).astype(np.int64)
        v = q - d
        mirrored = np.where((v >= w.qmin) & (v <= w.qmax), v, q)
        wm = oracle.Tensor(wl.pack_int4(mirrored), w.scales, out_f, in_f, 4, 32, w.qmin, w.qmax, w.tensor_id)
        ref = oracle.perturbed_qgemm(wm, [0], 0.0, x[2 * j + 1:2 * j + 2])
        assert (y[2 * j + 1] == ref[0]).all()
    assert (y[1::2] != plain[1::2]).any()


def test_update_matches_explicit_signed_members(oracle):
    # hist_len = 0: u = c * g is a single fp32 multiply of the (pinned) aggregate, c = alpha / (N sigma)
    w = _tensor(oracle, 4, 16, 64, 4, 32, scales=False)
    q0 = w.unpacked().copy()
    rng = np.random.default_rng(5)
    N = 8
    pair_seeds = rng.integers(0, 2 ** 63, size=N // 2, dtype=np.uint64)
    fit = oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32))
    alpha, sigma = 3.0, 1.0
    g = oracle.aggregate(w, pair_seeds, fit, sigma, antithetic=True)
    u = (np.float32(alpha / (N * sigma)) * g).astype(np.float32)
    d = np.rint(u).astype(np.int64)
    ok = (q0 + d >= w.qmin) & (q0 + d <= w.qmax)
    oracle.update(w, pair_seeds, fit, None, None, sigma, alpha, 0.9, antithetic=True)
    assert (w.unpacked() == np.where(ok, q0 + d, q0)).all()
    assert (w.unpacked() != q0).any()


def test_replay_equals_stored_residual_with_pairs(oracle):
    # interior int8 weights: replaying the whole history reproduces the residual of a step-by-step run
    qw = np.random.default_rng(6).integers(-2, 3, size=(8, 32)).astype(np.int8)
    w = oracle.Tensor(qw, None, 8, 32, 8, 0, -127, 127, 9)
    rng = np.random.default_rng(7)
    N, steps = 6, 6
    seeds = rng.integers(0, 2 ** 63, size=(steps, N // 2), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(steps)])
    sigma, alpha, gamma = 1.0, 1.5, 0.9
    c = np.float32(alpha / (N * sigma))
    e = np.zeros((8, 32), dtype=np.float32)
    moved = 0
    for t in range(steps):
        # explicitly stored residual, advanced with the (separately pinned) aggregate
        g = oracle.aggregate(w, seeds[t], fit[t], sigma, antithetic=True)
        u = (c * g + np.float32(gamma) * e).astype(np.float32)   # unfused; the oracle fuses the multiply-add
        before = w.unpacked()
        oracle.update(w, seeds[t], fit[t], seeds[:t], fit[:t], sigma, alpha, gamma, antithetic=True)
        applied = (w.unpacked() - before).astype(np.float32)
        assert np.abs(applied - np.rint(u)).max() <= 1        # fused vs unfused u can differ at a rounding tie
        e = (u - applied).astype(np.float32)
        moved += int((applied != 0).sum())
        # replaying the whole history on the new weights returns that residual
        rep = oracle.replay_residual(w, seeds[:t + 1], fit[:t + 1], N, sigma, alpha, gamma, antithetic=True)
        assert np.abs(rep - e).max() < 1e-6
    assert moved > 20
