"""Bit-exact parity of the bf16-MFMA perturbed GEMM on inputs whose arithmetic is exact.

With activations that are small integers, scales that are powers of two (or zero) and
in_features·max|x|·max|w'| < 2^24, every product, every fp32 partial sum and every change of the
accumulators' scale unit is exact, so the kernel's result before the output rounding is the same
real number the oracle forms in fp64, and both round it to bfloat16 once, to nearest even. The
outputs must then be identical bit for bit, which pins what the 1e-2 tolerance of the other GEMM
tests cannot: the in-kernel pair indexing, the gate of every single element, the k tails, clamped
rows, the first and last substep, in every tile height, in the paired (antithetic) kernel and in the
batched launch. One mis-indexed or mis-gated δ changes an output by at least one grid step here.
"""
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


def _exact_tensor(oracle, seed, out_f, in_f, bits, group, qmin=None, qmax=None, dead_scales=False):
    rng = np.random.default_rng(seed)
    if qmin is None:
        qmin, qmax = (-8, 7) if bits == 4 else (-127, 127)
    q = rng.integers(qmin, qmax + 1, size=(out_f, in_f), dtype=np.int64)
    # plenty of elements on both range edges so that the gate fires in every row
    edge = rng.random((out_f, in_f))
    q = np.where(edge < 0.15, qmin, np.where(edge > 0.85, qmax, q))
    qw = wl.pack_int4(q) if bits == 4 else q.astype(np.int8)
    shape = (out_f, in_f // group) if group else (out_f,)
    sc = np.exp2(-rng.integers(3, 10, size=shape)).astype(np.float32)
    if dead_scales:
        sc = np.where(rng.random(shape) < 0.2, 0.0, sc).astype(np.float32)
    return oracle.Tensor(qw, wl.f16_bits(sc), out_f, in_f, bits, group, qmin, qmax, 1000 + seed)


def _exact_activations(seed, N, T, in_f, amax):
    rng = np.random.default_rng(seed + 1)
    return wl.f32_to_bf16_bits(rng.integers(-amax, amax + 1, size=(N, T, in_f)).astype(np.float32))


# (bits, group, out, in, N, T, amax): every tile height (T <= 16, 32, 64, 128, 256, 512 tokens per
# pass, and more than one pass), ragged out (not a multiple of the 64-row tile) and ragged T, one to
# 28 substeps, group sizes 32 / 64 / 128 / per row, both weight widths
CASES = [
    (4, 32, 80, 256, 3, 16, 4),
    (4, 32, 64, 32, 2, 1, 4),            # a single substep, a single token
    (4, 128, 200, 384, 3, 17, 4),        # 32-token tile, ragged
    (4, 128, 72, 896, 2, 40, 3),         # 64-token tile, 28 substeps
    (4, 64, 64, 192, 2, 100, 4),         # 128-token tile
    (4, 128, 130, 256, 2, 200, 4),       # 256-token tile
    (4, 32, 64, 160, 2, 300, 4),         # 512-token tile
    (4, 128, 64, 256, 1, 600, 4),        # two passes over the tokens
    (4, 0, 96, 224, 3, 33, 4),           # int4 with one scale per row
    (8, 0, 96, 224, 3, 33, 2),           # int8 weights, bf16 activations
    (8, 0, 70, 1024, 2, 130, 2),         # int8, 256-token tile, long rows: 1024*2*127 < 2^24
]


def _gpu(env, ot, seeds, x_bits, sigma=1.0, mask=None, antithetic=False):
    torch, qes, u = env["torch"], env["qes"], env["u"]
    N, T, _ = x_bits.shape
    y = torch.full((N, T, ot.out_features), float("nan"), dtype=torch.bfloat16, device=u.DEV)
    qes.perturbed_qgemm(u.device_tensor(ot), seeds, sigma, u.to_dev(x_bits).view(torch.bfloat16), y, perturb_mask=mask,
                        antithetic=antithetic)
    return y.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("bits,group,out_f,in_f,N,T,amax", CASES)
def test_identical_outputs(env, bits, group, out_f, in_f, N, T, amax):
    oracle = env["oracle"]
    seed = out_f + in_f + T
    ot = _exact_tensor(oracle, seed, out_f, in_f, bits, group, dead_scales=(group == 128))
    x = _exact_activations(seed, N, T, in_f, amax)
    seeds = np.random.default_rng(seed).integers(0, 2 ** 63, size=N, dtype=np.uint64)
    ref = oracle.perturbed_qgemm(ot, seeds, 1.0, x)
    got = _gpu(env, ot, seeds, x)
    assert (got == ref).all(), int((got != ref).sum())
    assert (ref != oracle.perturbed_qgemm(ot, seeds, 0.0, x)).mean() > 0.3       # the noise is in the outputs


@pytest.mark.parametrize("sigma", [0.3, 2.0, 5.0])
def test_identical_outputs_other_sigmas(env, sigma):
    """Small σ (most δ zero), and σ large enough for |δ| up to the 4-bit container's clamp."""
    oracle = env["oracle"]
    ot = _exact_tensor(oracle, 5, 100, 256, 4, 64)
    x = _exact_activations(5, 3, 48, 256, 4)
    seeds = np.arange(11, 14, dtype=np.uint64)
    assert (_gpu(env, ot, seeds, x, sigma=sigma) == oracle.perturbed_qgemm(ot, seeds, sigma, x)).all()


def test_symmetric_range_and_masks(env):
    """qmin = -7 (App. A.1's symmetric grid) with stored -8 nibbles absent, members switched off."""
    oracle = env["oracle"]
    ot = _exact_tensor(oracle, 8, 90, 128, 4, 32, qmin=-7, qmax=7)
    x = _exact_activations(8, 5, 20, 128, 4)
    seeds = np.arange(1, 6, dtype=np.uint64)
    mask = np.array([1, 0, 1, 1, 0], dtype=np.uint8)
    ref = oracle.perturbed_qgemm(ot, seeds, 1.0, x, perturb_mask=mask)
    assert (_gpu(env, ot, seeds, x, mask=mask) == ref).all()


# paired kernel: one workgroup serves members 2j and 2j+1 from one draw (up to 128 tokens per member
# in single launches); above that the mirrored member regenerates the draw with the opposite sign
@pytest.mark.parametrize("bits,group,out_f,in_f,N,T,amax", [(4, 32, 80, 256, 4, 16, 4), (4, 128, 200, 384, 2, 50, 4),
                                                            (4, 64, 64, 192, 6, 128, 4), (8, 0, 96, 224, 4, 33, 2),
                                                            (4, 128, 70, 256, 2, 200, 4), (4, 32, 64, 160, 2, 300, 4)])
def test_identical_outputs_antithetic(env, bits, group, out_f, in_f, N, T, amax):
    oracle = env["oracle"]
    seed = out_f + in_f + T + 1
    ot = _exact_tensor(oracle, seed, out_f, in_f, bits, group)
    x = _exact_activations(seed, N, T, in_f, amax)
    seeds = np.random.default_rng(seed).integers(0, 2 ** 63, size=N // 2, dtype=np.uint64)
    mask = np.ones(N, dtype=np.uint8)
    mask[N - 1] = 0                                     # one member of the last pair on the base weights
    ref = oracle.perturbed_qgemm(ot, seeds, 1.0, x, perturb_mask=mask, antithetic=True)
    assert (_gpu(env, ot, seeds, x, mask=mask, antithetic=True) == ref).all()


@pytest.mark.parametrize("N,T,antithetic", [(3, 40, False), (4, 100, True), (4, 256, True), (2, 300, False)])
def test_identical_outputs_batched(env, N, T, antithetic):
    """A layer's linears in one launch (per-XCD work queues, a tensor found by bisection, the paired
    256-token tile that only the batched call uses): every tensor identical to the oracle."""
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    specs = [(4, 128, 200, 384, "h"), (4, 128, 72, 384, "h"), (8, 0, 96, 224, "a"), (4, 32, 64, 256, "b"),
             (8, 0, 16, 384, "h"), (4, 128, 384, 128, "i")]
    xs_host, ots, xs = {}, [], []
    for idx, (bits, group, out_f, in_f, key) in enumerate(specs):
        ots.append(_exact_tensor(oracle, 50 + idx, out_f, in_f, bits, group))
        if key not in xs_host:
            xs_host[key] = _exact_activations(60 + idx, N, T, in_f, 2 if bits == 8 or key == "h" else 4)
        xs.append(xs_host[key])
    dts = [u.device_tensor(ot) for ot in ots]
    xd = {k: u.to_dev(v).view(torch.bfloat16) for k, v in xs_host.items()}
    ys = [torch.full((N, T, ot.out_features), float("nan"), dtype=torch.bfloat16, device=u.DEV) for ot in ots]
    seeds = np.random.default_rng(T).integers(0, 2 ** 63, size=N // 2 if antithetic else N, dtype=np.uint64)
    qes.perturbed_qgemm_batch(dts, seeds, 1.0, [xd[s[4]] for s in specs], ys, antithetic=antithetic)
    for ot, xb, y in zip(ots, xs, ys):
        ref = oracle.perturbed_qgemm(ot, seeds, 1.0, xb, antithetic=antithetic)
        got = y.view(torch.int16).cpu().numpy().view(np.uint16)
        assert (got == ref).all(), (ot.out_features, ot.in_features)
