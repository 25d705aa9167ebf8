"""GPU parity for qes_perturbed_qgemm_batch: the linears of a layer in one launch give the same
outputs, bit for bit, as one qes_perturbed_qgemm call per tensor (whose parity with the oracle is
the subject of test_gpu_gemm.py), and match the oracle directly within the GEMM tolerance."""
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


def _layer(env, specs, N, T, seed):
    """specs: (bits, group, out, in, x_key). Tensors with the same x_key share one activation tensor."""
    torch, u, oracle = env["torch"], env["u"], env["oracle"]
    rng = np.random.default_rng(seed)
    xs_host, ots, dts, xs = {}, [], [], []
    for idx, (bits, group, out_f, in_f, key) in enumerate(specs):
        qw, sc, qmin, qmax = wl.random_tensor(seed * 10 + idx, out_f, in_f, bits, group)
        ot = oracle.Tensor(qw, sc, out_f, in_f, bits, group, qmin, qmax, 60 + idx)
        if key not in xs_host:
            xb = wl.f32_to_bf16_bits(rng.standard_normal((N, T, in_f)).astype(np.float32))
            xs_host[key] = (xb, u.to_dev(xb).view(torch.bfloat16))
        ots.append((ot, xs_host[key][0]))
        dts.append(u.device_tensor(ot))
        xs.append(xs_host[key][1])
    return ots, dts, xs


def _outputs(env, dts, N, T):
    torch, u = env["torch"], env["u"]
    return [torch.full((N, T, d.out_features), 7.0, dtype=torch.bfloat16, device=u.DEV) for d in dts]


@pytest.mark.parametrize("N,T,act,antithetic", [(6, 16, 0, False), (5, 64, 0, False), (3, 300, 0, False), (8, 100, 0, True),
                                                (4, 200, 0, True), (6, 64, 1, False), (4, 40, 1, True),
                                                (6, 256, 0, True), (4, 256, 1, True), (2, 257, 0, True)])
def test_batch_equals_single_calls_and_oracle(env, N, T, act, antithetic):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    if act == 0:
        specs = [(4, 128, 200, 384, "h"), (4, 128, 72, 384, "h"), (8, 0, 96, 224, "a"), (4, 32, 64, 256, "b"),
                 (8, 0, 16, 384, "h"), (4, 128, 384, 128, "i")]
    else:
        specs = [(8, 0, 128, 256, "h"), (8, 0, 40, 256, "h"), (8, 0, 200, 224, "a"), (8, 0, 64, 256, "h2")]
    ots, dts, xs = _layer(env, specs, N, T, 3 + T)
    rng = np.random.default_rng(T)
    seeds = rng.integers(0, 2 ** 63, size=N // 2 if antithetic else N, dtype=np.uint64)
    mask = np.ones(N, dtype=np.uint8)
    mask[1] = 0
    y_batch, y_single = _outputs(env, dts, N, T), _outputs(env, dts, N, T)
    nb = qes.gemm_batch_workspace_bytes(dts, xs, N, T, act)
    assert (nb > 0) == (act == 1)
    ws = torch.empty(nb, dtype=torch.uint8, device=u.DEV) if nb else None
    qes.perturbed_qgemm_batch(dts, seeds, 1.0, xs, y_batch, act_mode=act, perturb_mask=mask, workspace=ws,
                              antithetic=antithetic)
    for d, x, y in zip(dts, xs, y_single):
        n1 = qes.gemm_workspace_bytes(d, N, T, act)
        w1 = torch.empty(n1, dtype=torch.uint8, device=u.DEV) if n1 else None
        qes.perturbed_qgemm(d, seeds, 1.0, x, y, act_mode=act, perturb_mask=mask, workspace=w1, antithetic=antithetic)
    for yb, ys in zip(y_batch, y_single):
        assert torch.equal(yb.view(torch.int16), ys.view(torch.int16))
    # and directly against the oracle: the first and the last tensor of the list
    for k in (0, len(dts) - 1):
        ot, xb = ots[k]
        ref = oracle.perturbed_qgemm(ot, seeds, 1.0, xb, act_mode=act, perturb_mask=mask, antithetic=antithetic)
        got = y_batch[k].view(torch.int16).cpu().numpy().view(np.uint16)
        if act == 1:
            assert (got == ref).all()
        else:
            ok, worst = u.bf16_close(got, ref)
            assert ok, (k, worst)


def test_shared_input_is_quantised_once(env):
    """W8A8: the workspace of a batch holds one quantised copy per distinct activation tensor."""
    torch, qes, u = env["torch"], env["qes"], env["u"]
    specs = [(8, 0, 128, 256, "h"), (8, 0, 40, 256, "h"), (8, 0, 64, 256, "h")]
    _, dts, xs = _layer(env, specs, 4, 32, 9)
    one = qes.gemm_workspace_bytes(dts[0], 4, 32, 1)
    assert one <= qes.gemm_batch_workspace_bytes(dts, xs, 4, 32, 1) < 2 * one


def test_batch_argument_errors(env):
    torch, qes, u = env["torch"], env["qes"], env["u"]
    specs = [(8, 0, 128, 256, "h"), (8, 0, 40, 256, "h")]
    _, dts, xs = _layer(env, specs, 4, 32, 11)
    ys = _outputs(env, dts, 4, 32)
    seeds = np.arange(4, dtype=np.uint64)
    with pytest.raises(ValueError):
        qes.perturbed_qgemm_batch([], seeds, 1.0, [], [])
    with pytest.raises(qes.QesError):                    # W8A8 without its workspace
        qes.perturbed_qgemm_batch(dts, seeds, 1.0, xs, ys, act_mode=1)
    with pytest.raises(ValueError):                      # an output of the wrong shape
        qes.perturbed_qgemm_batch(dts, seeds, 1.0, xs, [ys[0], ys[0]])


def test_refused_w8a8_call_leaves_the_workspace_untouched(env):
    """Every check that can refuse a call precedes the first launch: a W8A8 batch that passes the
    per-tensor checks but exceeds the launch's work-queue limit (4096 descriptors of one 16384-row
    tensor, 1024 members: 2^27 queue slots) returns QES_ERR_UNSUPPORTED before its activations are
    quantised into the workspace. All descriptors alias the same valid buffers."""
    torch, qes, u = env["torch"], env["qes"], env["u"]
    out_f, in_f, N, T = 16384, 32, 1024, 1
    qw = torch.zeros((out_f, in_f), dtype=torch.int8, device=u.DEV)
    sc = torch.ones(out_f, dtype=torch.float16, device=u.DEV)
    t = qes.Tensor(qw, sc, out_f, in_f, 8, 0, -127, 127, 5)
    x = torch.ones((N, T, in_f), dtype=torch.bfloat16, device=u.DEV)
    y = torch.zeros((N, T, out_f), dtype=torch.bfloat16, device=u.DEV)
    n = 4096
    nbytes = qes.gemm_batch_workspace_bytes([t] * n, [x] * n, N, T, 1)
    assert nbytes > 0
    ws = torch.full((nbytes,), 0xAB, dtype=torch.uint8, device=u.DEV)
    with pytest.raises(qes.QesError) as err:
        qes.perturbed_qgemm_batch([t] * n, np.arange(N, dtype=np.uint64), 1.0, [x] * n, [y] * n, act_mode=1, workspace=ws)
    assert err.value.status == -2
    torch.cuda.synchronize()
    assert bool((ws == 0xAB).all()) and bool((y == 0).all())
    # the single-tensor call on the same buffers is accepted and does write the workspace
    small = qes.gemm_workspace_bytes(t, N, T, 1)
    qes.perturbed_qgemm(t, np.arange(N, dtype=np.uint64), 1.0, x, y, act_mode=1, workspace=ws[:small])
    torch.cuda.synchronize()
    assert not bool((ws[:small] == 0xAB).all())
