"""GPU parity on the benchmark configurations themselves (workloads.CONFIGS), through the C ABI.

Configs 1 and 2 run their whole multi-iteration loop in lock step: each ABI call is compared on
identical inputs, and the fitness vector, computed from the ORACLE's GEMM outputs, is fed to both
the GPU update and the oracle update, so the weights stay bit-identical and the next iteration's
GEMM is again compared on identical weights. Nothing the GPU produced ever enters the oracle.
Configs 1 and 2 are checked in full, on every row of every iteration. The big configs (3, 4, 5:
real N, T and K, in the batched launches bench.py times) are checked on sampled output rows, which
the counter-based noise makes exact: first row, last row and seeded random rows of every tensor of
every layer, plus the whole first layer of config 3 for the update. Where the oracle follows only
some rows, its copy of the other rows goes stale and is never read.
"""
import os

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


def _tensors(env, cfg, layer):
    oracle, u = env["oracle"], env["u"]
    out = []
    for li, spec in enumerate(cfg.linears):
        ot = oracle.Tensor(wl.make_qweight(cfg, layer, li), wl.make_scales(cfg, layer, li), spec.out_features,
                           spec.in_features, cfg.bits, cfg.group_size, cfg.qmin, cfg.qmax, cfg.tensor_id(layer, li))
        out.append((spec, ot, u.device_tensor(ot)))
    return out


def _activations(env, cfg):
    torch, u = env["torch"], env["u"]
    xs = {}
    for spec in cfg.linears:
        if spec.x_key not in xs:
            xb = wl.make_activations(cfg, spec.x_key, spec.in_features)
            xs[spec.x_key] = (xb, u.to_dev(xb).view(torch.bfloat16))
    return xs


def _gemm(env, cfg, dt, seeds, xd, ws):
    torch, qes, u = env["torch"], env["qes"], env["u"]
    y = torch.empty((cfg.N, cfg.T, dt.out_features), dtype=torch.bfloat16, device=u.DEV)
    qes.perturbed_qgemm(dt, seeds, cfg.sigma, xd, y, act_mode=cfg.act_mode, workspace=ws)
    return y.view(torch.int16).cpu().numpy().view(np.uint16)


def _packed_rows(ot, arr, rows):
    """Rows of a packed weight array (uint8 [out,in/2] or int8 [out,in])."""
    return arr.reshape(ot.out_features, -1)[rows]


@pytest.mark.parametrize("cfg_index,n_random_rows", [(1, None), (2, None)])
def test_lock_step_iterations(env, cfg_index, n_random_rows):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    cfg = wl.CONFIGS[cfg_index]
    tensors = _tensors(env, cfg, 0)
    xs = _activations(env, cfg)
    targets = [wl.bf16_bits_to_f32(wl.make_target(cfg, li)).astype(np.float64) for li in range(len(cfg.linears))]
    seeds = wl.make_seeds(cfg, cfg.iters)
    rows = [None if n_random_rows is None else wl.sample_rows(cfg, 0, li, n_random_rows)
            for li in range(len(cfg.linears))]
    hist_fit = np.zeros((0, cfg.N), dtype=np.float32)
    moved = 0
    for it in range(cfg.iters):
        # ---- population evaluation: every linear, every member, compared column by column
        mse = np.zeros(cfg.N)
        for li, (spec, ot, dt) in enumerate(tensors):
            xb, xd = xs[spec.x_key]
            y = _gemm(env, cfg, dt, seeds[it], xd, None)
            ref = oracle.perturbed_qgemm(ot, seeds[it], cfg.sigma, xb, rows=rows[li])
            sel = slice(None) if rows[li] is None else rows[li]
            ok, worst = u.bf16_close(y[:, :, sel], ref[:, :, sel])
            assert ok, (it, spec.name, worst)
            rf = wl.bf16_bits_to_f32(ref[:, :, sel]).astype(np.float64)
            mse += ((rf - targets[li][None][:, :, sel]) ** 2).mean(axis=(1, 2))
        # fitness = -MSE over the columns the oracle evaluated (mean over the layers), z-scored;
        # taken from the oracle's outputs for both sides
        fit = oracle.normalize_fitness((-mse / len(tensors)).astype(np.float32))
        assert (fit == qes.normalize_fitness((-mse / len(tensors)).astype(np.float32))).all()
        # ---- update with the history seen so far (window K), both sides
        lo = max(0, it - cfg.K)
        for li, (spec, ot, dt) in enumerate(tensors):
            before = _packed_rows(ot, ot.qweight, slice(None) if rows[li] is None else rows[li]).copy()
            qes.update(dt, seeds[it], fit, seeds[lo:it], hist_fit[lo:it], cfg.sigma, cfg.alpha, cfg.gamma)
            oracle.update(ot, seeds[it], fit, seeds[lo:it], hist_fit[lo:it], cfg.sigma, cfg.alpha, cfg.gamma,
                          rows=rows[li])
            got = dt.qweight.cpu().numpy()
            sel = slice(None) if rows[li] is None else rows[li]
            assert (_packed_rows(ot, got, sel) == _packed_rows(ot, ot.qweight, sel)).all(), (it, spec.name)
            moved += int((_packed_rows(ot, ot.qweight, sel) != before).sum())
        hist_fit = np.concatenate([hist_fit, fit[None]], axis=0)
    assert moved > 0


@pytest.mark.parametrize("cfg_index", [3, 4, 5])
def test_full_size_layer_sampled_rows(env, cfg_index):
    """One full-size layer of the big configurations in the launch configuration bench.py times:
    every tensor shape with the real N, T and K, the layer's GEMMs in one batched call and its
    updates in one batched call, checked on sampled rows of every tensor."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    cfg = wl.CONFIGS[cfg_index]
    seeds = wl.make_seeds(cfg, cfg.K + 1)
    fits = np.stack([oracle.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + 1)])
    ots, dts, rows = [], [], []
    for li, spec in enumerate(cfg.linears):
        ot = oracle.Tensor(wl.make_qweight(cfg, 0, li), wl.make_scales(cfg, 0, li), spec.out_features,
                           spec.in_features, cfg.bits, cfg.group_size, cfg.qmin, cfg.qmax, cfg.tensor_id(0, li))
        ots.append(ot)
        dts.append(u.device_tensor(ot))
        rows.append(wl.sample_rows(cfg, 0, li, 10))
    xs_host, xs_dev = {}, {}
    for spec in cfg.linears:
        if spec.x_key not in xs_host:
            xs_host[spec.x_key] = wl.make_activations(cfg, spec.x_key, spec.in_features)
            xs_dev[spec.x_key] = u.to_dev(xs_host[spec.x_key]).view(torch.bfloat16)
    xs = [xs_dev[spec.x_key] for spec in cfg.linears]
    ys = [torch.empty((cfg.N, cfg.T, spec.out_features), dtype=torch.bfloat16, device=u.DEV) for spec in cfg.linears]
    # ---- the layer's GEMMs in one call; sampled output columns, all members and tokens
    nbytes = qes.gemm_batch_workspace_bytes(dts, xs, cfg.N, cfg.T, cfg.act_mode)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=u.DEV) if nbytes else None
    qes.perturbed_qgemm_batch(dts, seeds[cfg.K], cfg.sigma, xs, ys, act_mode=cfg.act_mode, workspace=ws)
    for li, spec in enumerate(cfg.linears):
        sel = torch.from_numpy(rows[li].astype(np.int64)).to(u.DEV)
        got = ys[li].index_select(2, sel).view(torch.int16).cpu().numpy().view(np.uint16)
        ref = oracle.perturbed_qgemm(ots[li], seeds[cfg.K], cfg.sigma, xs_host[spec.x_key], act_mode=cfg.act_mode,
                                     rows=rows[li])[:, :, rows[li]]
        if cfg.act_mode == 1:
            assert (got == ref).all(), spec.name
        else:
            ok, worst = u.bf16_close(got, ref)
            assert ok, (spec.name, worst)
    del ws, ys, xs, xs_dev, xs_host
    # ---- replayed residual per tensor, sampled rows (fp32, compared exactly)
    for li, spec in enumerate(cfg.linears):
        res = torch.empty((spec.out_features, spec.in_features), dtype=torch.float32, device=u.DEV)
        qes.replay_residual(dts[li], seeds[:cfg.K], fits[:cfg.K], cfg.N, cfg.sigma, cfg.alpha, cfg.gamma, res)
        res_rows = res[torch.from_numpy(rows[li].astype(np.int64)).to(u.DEV)].cpu().numpy()
        del res
        ref_res = np.zeros((spec.out_features, spec.in_features), dtype=np.float32)
        oracle.replay_residual(ots[li], seeds[:cfg.K], fits[:cfg.K], cfg.N, cfg.sigma, cfg.alpha, cfg.gamma,
                               rows=rows[li], residual=ref_res)
        assert (res_rows.view(np.uint32) == ref_res[rows[li]].view(np.uint32)).all(), spec.name
    # ---- the layer's updates in one call with the full window; sampled rows, bit-exact packed weights
    stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
    qes.update_batch(dts, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha, cfg.gamma,
                     stats=stats)
    for li, spec in enumerate(cfg.linears):
        oracle.update(ots[li], seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha, cfg.gamma,
                      rows=rows[li])
        got = dts[li].qweight.cpu().numpy()
        assert (_packed_rows(ots[li], got, rows[li]) == _packed_rows(ots[li], ots[li].qweight, rows[li])).all(), spec.name
    assert int(stats[0]) > 0


@pytest.mark.parametrize("cfg_index", [3, 4, 5])
def test_every_layer_sampled_rows(env, cfg_index):
    """Every layer of the big stacks (28 or 32 layers of 7 tensors, each with its own tensor id and
    weights) through the batched launches bench.py times, with the real N, T and K: GEMM and update
    checked on the first row, the last row and eight seeded rows of every tensor. W8A8 outputs and all
    integer weights must be identical, bf16 outputs within the GEMM tolerance."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    cfg = wl.CONFIGS[cfg_index]
    seeds = wl.make_seeds(cfg, cfg.K + 1)
    fits = np.stack([oracle.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + 1)])
    xs_host = {}
    for spec in cfg.linears:
        if spec.x_key not in xs_host:
            xs_host[spec.x_key] = wl.make_activations(cfg, spec.x_key, spec.in_features)
    xs_dev = {k: u.to_dev(v).view(torch.bfloat16) for k, v in xs_host.items()}
    xs = [xs_dev[spec.x_key] for spec in cfg.linears]
    ys = [torch.empty((cfg.N, cfg.T, spec.out_features), dtype=torch.bfloat16, device=u.DEV) for spec in cfg.linears]
    ws, ws_ready = None, False
    for layer in range(cfg.n_layers):
        print("config %d layer %d" % (cfg_index, layer), flush=True)
        ots = [oracle.Tensor(wl.make_qweight(cfg, layer, li), wl.make_scales(cfg, layer, li), spec.out_features,
                             spec.in_features, cfg.bits, cfg.group_size, cfg.qmin, cfg.qmax, cfg.tensor_id(layer, li))
               for li, spec in enumerate(cfg.linears)]
        dts = [u.device_tensor(ot) for ot in ots]
        rows = [wl.sample_rows(cfg, layer, li, 8) for li in range(len(cfg.linears))]
        if not ws_ready:
            nbytes = qes.gemm_batch_workspace_bytes(dts, xs, cfg.N, cfg.T, cfg.act_mode)
            ws = torch.empty(nbytes, dtype=torch.uint8, device=u.DEV) if nbytes else None
            ws_ready = True
        qes.perturbed_qgemm_batch(dts, seeds[cfg.K], cfg.sigma, xs, ys, act_mode=cfg.act_mode, workspace=ws)
        qes.update_batch(dts, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha, cfg.gamma)
        for li, spec in enumerate(cfg.linears):
            assert rows[li][0] == 0 and rows[li][-1] == spec.out_features - 1 and rows[li].size >= 8
            sel = torch.from_numpy(rows[li].astype(np.int64)).to(u.DEV)
            got = ys[li].index_select(2, sel).view(torch.int16).cpu().numpy().view(np.uint16)
            ref = oracle.perturbed_qgemm(ots[li], seeds[cfg.K], cfg.sigma, xs_host[spec.x_key], act_mode=cfg.act_mode,
                                         rows=rows[li])[:, :, rows[li]]
            if cfg.act_mode == 1:
                assert (got == ref).all(), (layer, spec.name)
            else:
                ok, worst = u.bf16_close(got, ref)
                assert ok, (layer, spec.name, worst)
            oracle.update(ots[li], seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha,
                          cfg.gamma, rows=rows[li])
            got_w = dts[li].qweight.view(spec.out_features, -1).index_select(0, sel).cpu().numpy()
            assert (got_w == _packed_rows(ots[li], ots[li].qweight, rows[li])).all(), (layer, spec.name)


def test_config_3_layer_0_updated_in_full(env):
    """Every element of the seven tensors of config 3's first layer (46.8 M parameters) through one
    batched update with the full window (K = 16, N = 30), against the oracle's update of all rows."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    cfg = wl.CONFIGS[3]
    seeds = wl.make_seeds(cfg, cfg.K + 1)
    fits = np.stack([oracle.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + 1)])
    ots = [oracle.Tensor(wl.make_qweight(cfg, 0, li), None, spec.out_features, spec.in_features, cfg.bits, cfg.group_size,
                         cfg.qmin, cfg.qmax, cfg.tensor_id(0, li)) for li, spec in enumerate(cfg.linears)]
    dts = [u.device_tensor(ot) for ot in ots]
    stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
    qes.update_batch(dts, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha, cfg.gamma,
                     stats=stats)
    ref_stats = np.zeros(2, dtype=np.uint64)
    for ot, dt, spec in zip(ots, dts, cfg.linears):
        print("config 3 layer 0 %s" % spec.name, flush=True)
        ref_stats = oracle.update(ot, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha,
                                  cfg.gamma, stats=ref_stats)
        assert (dt.qweight.cpu().numpy() == ot.qweight).all(), spec.name
    assert (stats.cpu().numpy().view(np.uint64) == ref_stats).all() and ref_stats[0] > 0


@pytest.mark.skipif(os.environ.get("QES_LONG_TESTS") != "1",
                    reason="five minutes of oracle time: run with QES_LONG_TESTS=1 (and -s to see its progress lines)")
def test_config_5_layer_0_in_full(env):
    """Every output and every element of the headline configuration's first layer (seven tensors,
    218 M parameters, N=32, T=128, K=32): the batched GEMM against the oracle on all columns, all
    members and tokens, then the batched update with the full window against the oracle's update of
    all rows, counters included."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    cfg = wl.CONFIGS[5]
    seeds = wl.make_seeds(cfg, cfg.K + 1)
    fits = np.stack([oracle.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + 1)])
    ots = [oracle.Tensor(wl.make_qweight(cfg, 0, li), wl.make_scales(cfg, 0, li), spec.out_features, spec.in_features,
                         cfg.bits, cfg.group_size, cfg.qmin, cfg.qmax, cfg.tensor_id(0, li))
           for li, spec in enumerate(cfg.linears)]
    dts = [u.device_tensor(ot) for ot in ots]
    xs_host = {}
    for spec in cfg.linears:
        if spec.x_key not in xs_host:
            xs_host[spec.x_key] = wl.make_activations(cfg, spec.x_key, spec.in_features)
    xs_dev = {k: u.to_dev(v).view(torch.bfloat16) for k, v in xs_host.items()}
    xs = [xs_dev[spec.x_key] for spec in cfg.linears]
    ys = [torch.empty((cfg.N, cfg.T, spec.out_features), dtype=torch.bfloat16, device=u.DEV) for spec in cfg.linears]
    qes.perturbed_qgemm_batch(dts, seeds[cfg.K], cfg.sigma, xs, ys)
    for li, spec in enumerate(cfg.linears):
        print("config 5 layer 0 GEMM %s" % spec.name, flush=True)
        ref = oracle.perturbed_qgemm(ots[li], seeds[cfg.K], cfg.sigma, xs_host[spec.x_key])
        ok, worst = u.bf16_close(ys[li].view(torch.int16).cpu().numpy().view(np.uint16), ref)
        assert ok, (spec.name, worst)
    stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
    qes.update_batch(dts, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha, cfg.gamma,
                     stats=stats)
    ref_stats = np.zeros(2, dtype=np.uint64)
    for ot, dt, spec in zip(ots, dts, cfg.linears):
        print("config 5 layer 0 update %s" % spec.name, flush=True)
        ref_stats = oracle.update(ot, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha,
                                  cfg.gamma, stats=ref_stats)
        assert (dt.qweight.cpu().numpy() == ot.qweight).all(), spec.name
    assert (stats.cpu().numpy().view(np.uint64) == ref_stats).all() and ref_stats[0] > 0


def test_largest_tensor_indexing(env):
    """A tensor just under the ABI's 2^33-element limit (4.3 GB of packed INT4, 2^32 - 2^20 pairs):
    element offsets need 64 bits and pair indices all 32. GEMM, replay and update on the first, the
    last and random rows; the oracle follows only those rows."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    out_f, in_f = 65536, 131040
    assert out_f * in_f < 2 ** 33 and out_f * in_f // 2 > 2 ** 32 - 2 ** 21
    rng = np.random.default_rng(77)
    qw = rng.integers(0, 256, size=(out_f, in_f // 2), dtype=np.uint8)
    sc = wl.f16_bits(rng.uniform(0.005, 0.02, size=(out_f, in_f // 32)).astype(np.float32))
    ot = oracle.Tensor(qw, sc, out_f, in_f, 4, 32, -8, 7, 4000000000)          # a tensor id above 2^31 as well
    dt = qes.Tensor(torch.from_numpy(qw).to(u.DEV), u.to_dev(sc), out_f, in_f, 4, 32, -8, 7, 4000000000)
    rows = np.unique(np.concatenate([[0, 1, out_f - 1, 32768, 32769], rng.integers(0, out_f, size=4)])).astype(np.int32)
    sel = torch.from_numpy(rows.astype(np.int64)).to(u.DEV)
    N, T, K = 2, 16, 1
    seeds = rng.integers(0, 2 ** 64, size=(K + 1, N), dtype=np.uint64)
    fit = np.float32([[1.0, -1.0], [-1.0, 1.0]])
    x = wl.f32_to_bf16_bits(rng.standard_normal((N, T, in_f)).astype(np.float32))
    y = torch.empty((N, T, out_f), dtype=torch.bfloat16, device=u.DEV)
    qes.perturbed_qgemm(dt, seeds[K], 1.0, u.to_dev(x).view(torch.bfloat16), y)
    got = y.index_select(2, sel).view(torch.int16).cpu().numpy().view(np.uint16)
    ref = oracle.perturbed_qgemm(ot, seeds[K], 1.0, x, rows=rows)[:, :, rows]
    ok, worst = u.bf16_close(got, ref)
    assert ok, worst
    stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
    before = qw[rows].copy()                      # the oracle updates qw in place
    qes.update(dt, seeds[K], fit[K], seeds[:K], fit[:K], 1.0, 2.0, 0.9, stats=stats)
    oracle.update(ot, seeds[K], fit[K], seeds[:K], fit[:K], 1.0, 2.0, 0.9, rows=rows)
    got_rows = dt.qweight.view(out_f, in_f // 2).index_select(0, sel).cpu().numpy()
    assert (got_rows == ot.qweight[rows]).all()
    assert int(stats[0]) > 2 ** 32 and (got_rows != before).any()      # the counters are 64-bit too


def test_maximum_population_and_history(env):
    """N = 1024 members and hist_len = 256 generations (the ABI's limits) on a small tensor."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    N, K = 1024, 256
    qw, sc, qmin, qmax = wl.random_tensor(77, 8, 64, 4, 32)
    ot = oracle.Tensor(qw, sc, 8, 64, 4, 32, qmin, qmax, 3)
    dt = u.device_tensor(ot)
    rng = np.random.default_rng(123)
    seeds = rng.integers(0, 2 ** 63, size=(K + 1, N), dtype=np.uint64)
    fits = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(K + 1)])
    stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
    qes.update(dt, seeds[K], fits[K], seeds[:K], fits[:K], 1.0, 8.0, 0.9, stats=stats)
    ref_stats = oracle.update(ot, seeds[K], fits[K], seeds[:K], fits[:K], 1.0, 8.0, 0.9)
    assert (dt.qweight.cpu().numpy() == ot.qweight).all()
    assert (stats.cpu().numpy().view(np.uint64) == ref_stats).all() and ref_stats[0] > 0
    # one more member or generation than the limit is refused
    with pytest.raises(qes.QesError):
        qes.update(dt, np.zeros(N + 1, np.uint64), np.zeros(N + 1, np.float32), None, None, 1.0, 0.5, 0.9)
    with pytest.raises(qes.QesError):
        qes.update(dt, seeds[K], fits[K], np.zeros((K + 1, N), np.uint64), np.zeros((K + 1, N), np.float32), 1.0, 0.5,
                   0.9)
    # GEMM with 1024 members of one token each
    x = wl.f32_to_bf16_bits(rng.standard_normal((N, 1, 64)).astype(np.float32))
    y = torch.empty((N, 1, 8), dtype=torch.bfloat16, device=u.DEV)
    qes.perturbed_qgemm(dt, seeds[0], 1.0, u.to_dev(x).view(torch.bfloat16), y)
    ref = oracle.perturbed_qgemm(ot, seeds[0], 1.0, x)
    ok, worst = u.bf16_close(y.view(torch.int16).cpu().numpy().view(np.uint16), ref)
    assert ok, worst
