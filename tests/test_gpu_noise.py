"""GPU parity: the HIP noise generator against the CPU oracle, bit for bit (paper §3.2 Eq. 3)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(oracle):
    import torch
    import paper_2602_03120_amd as qes
    from gpu_util import DEV, from_dev
    assert torch.cuda.is_available()
    return dict(torch=torch, qes=qes, DEV=DEV, from_dev=from_dev, oracle=oracle)


SEEDS = [0, 1, 0xFFFFFFFFFFFFFFFF, 0x0123456789ABCDEF, 7919 << 40]


@pytest.mark.parametrize("pair_begin,n_pairs", [(0, 1), (0, 257), (5, 100003), ((1 << 32) - 100, 1000),
                                                ((1 << 45) + 3, 4099)])
def test_words_bit_exact(env, pair_begin, n_pairs):
    torch, qes, oracle = env["torch"], env["qes"], env["oracle"]
    for seed in SEEDS:
        out = torch.zeros(n_pairs * 4, dtype=torch.int32, device=env["DEV"])
        qes.noise_words(seed, 0xABCDEF01, pair_begin, n_pairs, out)
        got = env["from_dev"](out, np.uint32).reshape(n_pairs, 4)
        ref = oracle.noise_words(seed, 0xABCDEF01, pair_begin, n_pairs)
        assert (got == ref).all()


@pytest.mark.parametrize("elem_begin,n", [(0, 2), (1, 1), (3, 100001), (1 << 20, 1 << 20), ((1 << 33) + 1, 5000)])
def test_gauss_bit_exact(env, elem_begin, n):
    torch, qes, oracle = env["torch"], env["qes"], env["oracle"]
    for seed in SEEDS[:3]:
        out = torch.zeros(n, dtype=torch.float32, device=env["DEV"])
        qes.noise_gauss(seed, 17, elem_begin, n, out)
        got = env["from_dev"](out, np.uint32)
        ref = oracle.noise_gauss(seed, 17, elem_begin, n).view(np.uint32)
        assert (got == ref).all()


@pytest.mark.parametrize("sigma", [0.0, 0.001, 0.01, 0.3, 0.7, 1.0, 1.2, 2.5, 4.0])
def test_delta_bit_exact(env, sigma):
    torch, qes, oracle = env["torch"], env["qes"], env["oracle"]
    n = 1_000_003
    for seed, begin in [(11, 0), (0x0123456789ABCDEF, 12345)]:
        out = torch.zeros(n, dtype=torch.int8, device=env["DEV"])
        qes.noise_delta(seed, 3, begin, n, sigma, out)
        got = env["from_dev"](out, np.int8)
        ref = oracle.noise_delta(seed, 3, begin, n, sigma)
        assert (got == ref).all()


def test_noise_argument_errors(env):
    torch, qes = env["torch"], env["qes"]
    out = torch.zeros(16, dtype=torch.int8, device=env["DEV"])
    with pytest.raises(qes.QesError):
        qes.noise_delta(1, 1, 0, 16, -1.0, out)
    with pytest.raises(qes.QesError):
        qes.noise_delta(1, 1, 0, 16, float("nan"), out)
    qes.noise_delta(1, 1, 0, 0, 1.0, out)          # empty request is a no-op


@pytest.mark.parametrize("sweep", ["radius", "angle"])
def test_every_radius_and_angle_input(env, sweep):
    """All 2^24 radius inputs (with a few angle words) and all 2^24 angle fractions (with every
    quadrant, random radius words): Gaussians and perturbations identical to the oracle's."""
    torch, qes, oracle = env["torch"], env["qes"], env["oracle"]
    rng = np.random.default_rng(5)
    chunk = 1 << 22
    for c0 in range(0, 1 << 24, chunk):
        j = np.arange(c0, c0 + chunk, dtype=np.uint64)
        words = rng.integers(0, 1 << 32, size=(chunk, 4), dtype=np.uint64).astype(np.uint32)
        if sweep == "radius":
            words[:, 0] = ((j << 8) | (words[:, 0] & 0xFF)).astype(np.uint32)
            words[: chunk // 2, 1] = 0
        else:
            words[:, 1] = (((j & 3) << 30) | (j << 6) & 0x3FFFFFC0 | (words[:, 1] & 0x3F)).astype(np.uint32)
        wd = torch.from_numpy(words.view(np.int32)).to(env["DEV"])
        eps = torch.empty((chunk, 2), dtype=torch.float32, device=env["DEV"])
        dl = torch.empty((chunk, 2), dtype=torch.int8, device=env["DEV"])
        qes.noise_from_words(wd, chunk, 1.0, eps, dl)
        ref_eps, ref_dl = oracle.noise_from_words(words, 1.0)
        assert (env["from_dev"](eps, np.uint32) == ref_eps.view(np.uint32)).all()
        assert (env["from_dev"](dl, np.int8) == ref_dl).all()
