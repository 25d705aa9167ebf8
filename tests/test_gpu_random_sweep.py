"""Seeded random sweep of small shapes through the C ABI against the oracle: many combinations of
format, group size, ragged out / in / T, population (odd, even, smaller than a round), history
length, masks, zeroed scales and range edges that the hand-picked cases of the other files may not
hit together. Every case is a deterministic function of its index."""
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


def _tensor(oracle, rng, with_scales):
    bits = int(rng.choice([4, 8]))
    in_f = 32 * int(rng.integers(1, 13))                       # 32 .. 384
    out_f = int(rng.integers(1, 150))
    if bits == 4:
        group = int(rng.choice([g for g in (0, 32, 64, 128) if g == 0 or in_f % g == 0]))
        qmin, qmax = (-8, 7) if rng.random() < 0.7 else (-7, 7)
    else:
        group = 0
        qmin, qmax = (-127, 127) if rng.random() < 0.7 else (-5, 5)
    q = rng.integers(qmin, qmax + 1, size=(out_f, in_f))
    qw = wl.pack_int4(q) if bits == 4 else q.astype(np.int8)
    sc = None
    if with_scales:
        shape = (out_f, in_f // group) if group else (out_f,)
        scf = rng.uniform(0.005, 0.02, size=shape).astype(np.float32)
        scf[rng.random(shape) < 0.05] = 0.0                     # a few dead groups / rows
        sc = wl.f16_bits(scf)
    return oracle.Tensor(qw, sc, out_f, in_f, bits, group, qmin, qmax, int(rng.integers(1, 2 ** 31)))


@pytest.mark.parametrize("case", range(24))
def test_update_family(env, case):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    rng = np.random.default_rng(1000 + case)
    ot = _tensor(oracle, rng, with_scales=False)
    dt = u.device_tensor(ot)
    antithetic = bool(case % 3 == 1)
    N = int(rng.integers(1, 12)) * (2 if antithetic else 1)
    K = int(rng.integers(0, 6))
    sigma = float(rng.choice([0.5, 1.0, 1.2, 1.5, 3.0]))
    alpha = float(rng.choice([0.3, 1.5, 6.0])) * N / 8.0
    gamma = float(rng.choice([0.0, 0.5, 0.9, 1.0]))
    seeds = rng.integers(0, 2 ** 64, size=(K + 1, N // 2 if antithetic else N), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(K + 1)])
    res = torch.full((ot.out_features, ot.in_features), 3.0, dtype=torch.float32, device=u.DEV)
    qes.replay_residual(dt, seeds[:K], fit[:K], N, sigma, alpha, gamma, res, antithetic=antithetic)
    ref_res = oracle.replay_residual(ot, seeds[:K], fit[:K], N, sigma, alpha, gamma, antithetic=antithetic)
    assert (res.cpu().numpy().view(np.uint32) == ref_res.view(np.uint32)).all()
    stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
    qes.update(dt, seeds[K], fit[K], seeds[:K], fit[:K], sigma, alpha, gamma, stats=stats, antithetic=antithetic)
    ref_stats = oracle.update(ot, seeds[K], fit[K], seeds[:K], fit[:K], sigma, alpha, gamma, antithetic=antithetic)
    assert (dt.qweight.cpu().numpy().view(np.uint8) == ot.qweight.view(np.uint8)).all()
    assert (stats.cpu().numpy().view(np.uint64) == ref_stats).all()


@pytest.mark.parametrize("case", range(24))
def test_gemm(env, case):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    rng = np.random.default_rng(2000 + case)
    ot = _tensor(oracle, rng, with_scales=True)
    dt = u.device_tensor(ot)
    antithetic = bool(case % 3 == 2)
    N = int(rng.integers(1, 6)) * (2 if antithetic else 1)
    T = int(rng.choice([1, 5, 16, 17, 48, 64, 100, 129, 200, 260]))
    act = 1 if (ot.bits == 8 and case % 2 == 0) else 0
    sigma = float(rng.choice([0.0, 0.7, 1.0, 2.0]))
    x = wl.f32_to_bf16_bits((rng.standard_normal((N, T, ot.in_features)) * rng.choice([0.1, 1.0, 30.0])).astype(np.float32))
    if case % 5 == 0:
        x[0, 0, :] = 0                                          # an all-zero token (W8A8: scale falls back to 1)
    seeds = rng.integers(0, 2 ** 64, size=N // 2 if antithetic else N, dtype=np.uint64)
    mask = (rng.random(N) < 0.8).astype(np.uint8)
    y = torch.full((N, T, ot.out_features), float("nan"), dtype=torch.bfloat16, device=u.DEV)
    nb = qes.gemm_workspace_bytes(dt, N, T, act)
    ws = torch.empty(nb, dtype=torch.uint8, device=u.DEV) if nb else None
    qes.perturbed_qgemm(dt, seeds, sigma, u.to_dev(x).view(torch.bfloat16), y, act_mode=act, perturb_mask=mask,
                        workspace=ws, antithetic=antithetic)
    got = y.view(torch.int16).cpu().numpy().view(np.uint16)
    ref = oracle.perturbed_qgemm(ot, seeds, sigma, x, act_mode=act, perturb_mask=mask, antithetic=antithetic)
    if act == 1:
        assert (got == ref).all()
    else:
        ok, worst = u.bf16_close(got, ref)
        assert ok, worst
