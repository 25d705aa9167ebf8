"""GPU parity for antithetic perturbation pairs (paper App. A.1): members 2j and 2j+1 share a seed
and use +δ_j / -δ_j. Same bars as the plain entry points: integer weights, counters and fp32
residuals identical to the oracle, bf16 GEMM outputs within 1e-2, W8A8 outputs identical."""
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


def _history(rng, oracle, K, N):
    seeds = rng.integers(0, 2 ** 63, size=(K + 1, N // 2), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(K + 1)])
    return seeds, fit


@pytest.mark.parametrize("bits,out_f,in_f,K,N,sigma", [(4, 256, 256, 4, 8, 1.0), (4, 33, 70, 3, 6, 1.0),
                                                      (8, 1024, 1024, 2, 4, 1.0), (4, 2048, 1024, 1, 6, 2.5),
                                                      (4, 1024, 4096, 1, 6, 1.0),
                                                      (4, 64, 128, 0, 30, 1.0)])
def test_update_and_replay(env, bits, out_f, in_f, K, N, sigma):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    qw, _, qmin, qmax = wl.random_tensor(300 + out_f, out_f, in_f, bits, 0)
    ot = oracle.Tensor(qw, None, out_f, in_f, bits, 0, qmin, qmax, 12)
    seeds, fit = _history(np.random.default_rng(out_f + N), oracle, K, N)
    dt = u.device_tensor(ot)
    res = torch.zeros((out_f, in_f), dtype=torch.float32, device=u.DEV)
    qes.replay_residual(dt, seeds[:K], fit[:K], N, sigma, 1.5, 0.9, res, antithetic=True)
    ref_res = oracle.replay_residual(ot, seeds[:K], fit[:K], N, sigma, 1.5, 0.9, antithetic=True)
    assert (res.cpu().numpy().view(np.uint32) == ref_res.view(np.uint32)).all()
    stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
    qes.update(dt, seeds[K], fit[K], seeds[:K], fit[:K], sigma, 1.5, 0.9, stats=stats, antithetic=True)
    ref_stats = oracle.update(ot, seeds[K], fit[K], seeds[:K], fit[:K], sigma, 1.5, 0.9, antithetic=True)
    assert (dt.qweight.cpu().numpy().view(np.uint8) == ot.qweight.view(np.uint8)).all()
    assert (stats.cpu().numpy().view(np.uint64) == ref_stats).all() and ref_stats[0] > 0


# up to 128 tokens per member one workgroup serves both members of a pair from one draw; longer
# token counts regenerate the draw per member: both paths, every tile height of the shared one
@pytest.mark.parametrize("bits,group,out_f,in_f,N,T,act,off", [
    (4, 128, 200, 384, 4, 64, 0, (3,)), (4, 32, 64, 256, 8, 16, 0, (7,)), (8, 0, 96, 224, 6, 33, 0, (5,)),
    (8, 0, 128, 256, 2, 300, 1, (1,)),          # per-member path, int8 activations
    (4, 128, 200, 384, 4, 128, 0, (0,)),        # shared draw, tallest tile; the +δ member of pair 0 unperturbed
    (8, 0, 128, 224, 4, 100, 1, (2, 3)),        # shared draw, int8 activations, ragged tokens and k; pair 1 unperturbed
    (4, 64, 96, 512, 6, 130, 0, ()),            # just past the shared-draw limit
    (8, 0, 80, 128, 2, 7, 0, (0, 1)),           # a single pair, both members unperturbed
])
def test_gemm(env, bits, group, out_f, in_f, N, T, act, off):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    qw, sc, qmin, qmax = wl.random_tensor(out_f + T, out_f, in_f, bits, group)
    ot = oracle.Tensor(qw, sc, out_f, in_f, bits, group, qmin, qmax, 44)
    rng = np.random.default_rng(T)
    x = wl.f32_to_bf16_bits(rng.standard_normal((N, T, in_f)).astype(np.float32))
    pair_seeds = rng.integers(0, 2 ** 63, size=N // 2, dtype=np.uint64)
    mask = np.ones(N, dtype=np.uint8)
    mask[list(off)] = 0                                     # these members run on the base weights
    dt = u.device_tensor(ot)
    y = torch.empty((N, T, out_f), dtype=torch.bfloat16, device=u.DEV)
    nbytes = qes.gemm_workspace_bytes(dt, N, T, act)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=u.DEV) if nbytes else None
    qes.perturbed_qgemm(dt, pair_seeds, 1.0, u.to_dev(x).view(torch.bfloat16), y, act_mode=act, perturb_mask=mask,
                        workspace=ws, antithetic=True)
    got = y.view(torch.int16).cpu().numpy().view(np.uint16)
    ref = oracle.perturbed_qgemm(ot, pair_seeds, 1.0, x, act_mode=act, perturb_mask=mask, antithetic=True)
    if act == 1:
        assert (got == ref).all()
    else:
        ok, worst = u.bf16_close(got, ref)
        assert ok, worst
        if 1 not in off:
            # the mirrored members really differ from the +δ evaluation of the same seed
            plus = oracle.perturbed_qgemm(ot, np.repeat(pair_seeds, 2), 1.0, x, perturb_mask=mask)
            assert not u.bf16_close(got[1:2], plus[1:2])[0]


def test_odd_population_is_refused(env):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    qw, _, qmin, qmax = wl.random_tensor(1, 16, 32, 4, 0)
    dt = u.device_tensor(oracle.Tensor(qw, None, 16, 32, 4, 0, qmin, qmax, 1))
    import ctypes
    import paper_2602_03120_amd.binding as b
    d = dt.desc()
    seeds = np.zeros(2, dtype=np.uint64)
    fit = np.zeros(3, dtype=np.float32)
    rc = b._load().qes_update_antithetic(ctypes.byref(d), seeds.ctypes.data, fit.ctypes.data, None, None, 0, 3, 1.0, 0.5,
                                         0.9, None, None)
    assert rc == -1
