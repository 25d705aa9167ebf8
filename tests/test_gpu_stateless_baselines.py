"""GPU parity for the stateless stochastic-rounding baseline (paper §5, Eq. 9-10) and the comparison
the section argues: on one synthetic objective and the same kernels, deterministic stateless
rounding stagnates, stochastic stateless rounding drifts as a random walk, error feedback with seed
replay makes progress."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(oracle):
    import torch
    import paper_2602_03120_amd as qes
    import gpu_util
    assert torch.cuda.is_available()
    return dict(torch=torch, qes=qes, u=gpu_util, oracle=oracle)


@pytest.mark.parametrize("bits,out_f,in_f,N,steps,alpha", [(4, 256, 256, 8, 4, 1.5), (4, 7, 34, 5, 3, 3.0),
                                                           (8, 1024, 1024, 5, 2, 1.5), (4, 2048, 1024, 4, 2, 1.5),
                                                           (8, 2048, 2048, 2, 1, 1.5), (4, 64, 64, 30, 3, 40.0)])
def test_steps_match_oracle(env, bits, out_f, in_f, N, steps, alpha):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    qw, _, qmin, qmax = wl.random_tensor(700 + out_f, out_f, in_f, bits, 0)
    ot = oracle.Tensor(qw, None, out_f, in_f, bits, 0, qmin, qmax, 31)
    dt = u.device_tensor(ot)
    rng = np.random.default_rng(out_f + 2)
    seeds = rng.integers(0, 2 ** 63, size=(steps, N), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(steps)])
    round_seeds = rng.integers(0, 2 ** 64, size=steps, dtype=np.uint64)
    stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
    ref_stats = np.zeros(2, dtype=np.uint64)
    for t in range(steps):
        qes.update_stochastic_rounding(dt, seeds[t], fit[t], 1.0, alpha, int(round_seeds[t]), stats=stats)
        ref_stats = oracle.update_stochastic_rounding(ot, seeds[t], fit[t], 1.0, alpha, int(round_seeds[t]),
                                                      stats=ref_stats)
        assert (dt.qweight.cpu().numpy().view(np.uint8) == ot.qweight.view(np.uint8)).all(), t
    assert (stats.cpu().numpy().view(np.uint64) == ref_stats).all()
    assert ref_stats[0] > 0 and (out_f * in_f < 10000 or ref_stats[1] > 0)


def test_stored_weights_outside_the_range_are_not_counted_as_gated(env):
    """-8 nibbles under the symmetric range [-7, 7]: an element whose update is zero is never
    counted (Eq. 4 masks updates), for both update rules; weights and counters equal the oracle's."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    out_f, in_f, N = 64, 96, 6
    rng = np.random.default_rng(4)
    q = rng.integers(-7, 8, size=(out_f, in_f))
    q[rng.random((out_f, in_f)) < 0.3] = -8
    seeds = rng.integers(0, 2 ** 63, size=N, dtype=np.uint64)
    for fit in (np.zeros(N, np.float32), oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32))):
        for rule in ("stochastic", "feedback"):
            ot = oracle.Tensor(wl.pack_int4(q), None, out_f, in_f, 4, 0, -7, 7, 8)
            dt = u.device_tensor(ot)
            stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
            if rule == "stochastic":
                qes.update_stochastic_rounding(dt, seeds, fit, 1.0, 2.0, 123, stats=stats)
                ref = oracle.update_stochastic_rounding(ot, seeds, fit, 1.0, 2.0, 123)
            else:
                qes.update(dt, seeds, fit, None, None, 1.0, 2.0, 0.9, stats=stats)
                ref = oracle.update(ot, seeds, fit, None, None, 1.0, 2.0, 0.9)
            assert (dt.qweight.cpu().numpy().view(np.uint8) == ot.qweight.view(np.uint8)).all(), rule
            assert (stats.cpu().numpy().view(np.uint64) == ref).all(), (rule, stats, ref)
            assert (ref == 0).all() if not fit.any() else ref[1] > 0


def test_argument_errors(env):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    qw, _, qmin, qmax = wl.random_tensor(1, 16, 32, 4, 0)
    dt = u.device_tensor(oracle.Tensor(qw, None, 16, 32, 4, 0, qmin, qmax, 1))
    with pytest.raises(qes.QesError):
        qes.update_stochastic_rounding(dt, np.arange(4, dtype=np.uint64), np.zeros(4, np.float32), 0.0, 0.5, 1)
    with pytest.raises(qes.QesError):
        qes.update_stochastic_rounding(dt, np.arange(4, dtype=np.uint64), np.full(4, np.nan, np.float32), 1.0, 0.5, 1)


def test_feedback_progresses_where_stateless_rounding_stalls_or_drifts(env):
    """A 32x64 INT4 layer, 16 members, -MSE against a teacher layer's outputs, sub-threshold step
    size: 100 iterations of evaluation (perturbed qGEMM) + update for the three update rules."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    out_f, in_f, N, T, group, iters, K = 32, 64, 16, 32, 32, 100, 8
    sigma, alpha, gamma = 1.0, 0.3, 0.9
    rng = np.random.default_rng(0)
    q_star = rng.integers(-6, 7, size=(out_f, in_f))
    q0 = np.clip(q_star + rng.integers(-2, 3, size=q_star.shape), -8, 7)
    sc = wl.f16_bits(rng.uniform(0.02, 0.05, size=(out_f, in_f // group)).astype(np.float32))
    x1 = wl.f32_to_bf16_bits(rng.standard_normal((1, T, in_f)).astype(np.float32))
    xd = u.to_dev(np.repeat(x1, N, axis=0)).view(torch.bfloat16)
    seeds = rng.integers(0, 2 ** 63, size=(iters, N), dtype=np.uint64)

    def outputs(dt, member_seeds, s):
        y = torch.empty((N, T, out_f), dtype=torch.bfloat16, device=u.DEV)
        qes.perturbed_qgemm(dt, member_seeds, s, xd, y)
        return y.float().cpu().numpy().astype(np.float64)

    def device_tensor(q):
        return u.device_tensor(oracle.Tensor(wl.pack_int4(q), sc, out_f, in_f, 4, group, -8, 7, 7))

    target = outputs(device_tensor(q_star), seeds[0], 0.0)[0]
    loss = lambda dt: float(((outputs(dt, seeds[0], 0.0)[0] - target) ** 2).mean())
    final, changed = {}, {}
    for rule in ("feedback", "deterministic", "stochastic"):
        dt = device_tensor(q0.copy())
        stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
        start = loss(dt)
        hist = np.zeros((0, N), dtype=np.float32)
        for it in range(iters):
            mse = ((outputs(dt, seeds[it], sigma) - target[None]) ** 2).mean(axis=(1, 2))
            fit = qes.normalize_fitness((-mse).astype(np.float32))
            lo = max(0, it - K)
            if rule == "feedback":
                qes.update(dt, seeds[it], fit, seeds[lo:it], hist[lo:it], sigma, alpha, gamma, stats=stats)
            elif rule == "deterministic":
                qes.update(dt, seeds[it], fit, None, None, sigma, alpha, gamma, stats=stats)   # hist_len = 0
            else:
                qes.update_stochastic_rounding(dt, seeds[it], fit, sigma, alpha, 1000 + it, stats=stats)
            hist = np.concatenate([hist, fit[None]], axis=0)
        final[rule] = loss(dt) / start
        changed[rule] = int(stats.cpu().numpy()[0])
    assert changed["deterministic"] == 0 and final["deterministic"] == 1.0     # stagnation: W_T = W_0
    assert changed["feedback"] > 100 and final["feedback"] < 0.93              # progress
    assert changed["stochastic"] > 10 * changed["feedback"] and final["stochastic"] > 1.2   # noise floor
