"""Host threads calling the library at the same time, each on a stream of its own.

The library keeps no state between calls except its ring of staging slots (the (seed, fitness)
records of a call travel through one of eight pinned/device slot pairs, handed out under a mutex, a
slot being reused once the event behind its last consumer has completed). Twelve threads, more than
there are slots, update and evaluate their own tensors concurrently without synchronising between
calls; every thread's final weights, counters and outputs must be the oracle's (Alg. 2, Alg. 1's
inference step), as if the calls had been made one after the other.
"""
import threading

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

N_THREADS = 12
CALLS = 12


@pytest.fixture(scope="module")
def env(oracle):
    import torch
    import paper_2602_03120_amd as qes
    import gpu_util
    assert torch.cuda.is_available()
    return dict(torch=torch, qes=qes, u=gpu_util, oracle=oracle)


def _plan(oracle, tid):
    """Per thread: a tensor of its own and CALLS generations (members and window differ by thread)."""
    rng = np.random.default_rng(1000 + tid)
    bits = 4 if tid % 3 else 8
    out_f, in_f = 48 + 16 * (tid % 4), 128 + 64 * (tid % 3)
    group = 0 if bits == 8 else 32
    qw, sc, qmin, qmax = wl.random_tensor(500 + tid, out_f, in_f, bits, group)
    ot = oracle.Tensor(qw, sc, out_f, in_f, bits, group, qmin, qmax, 40 + tid)
    N = (4, 30, 64, 7)[tid % 4]
    K = (0, 3, 8)[tid % 3]
    seeds = rng.integers(0, 2 ** 63, size=(CALLS + K, N), dtype=np.uint64)
    fit = np.stack([oracle.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(CALLS + K)])
    T = 5 + tid
    x = wl.f32_to_bf16_bits(rng.standard_normal((N, T, in_f)).astype(np.float32))
    return dict(ot=ot, N=N, K=K, seeds=seeds, fit=fit, x=x, T=T)


def test_concurrent_callers_on_their_own_streams(env):
    torch, qes, u, oracle = env["torch"], env["qes"], env["u"], env["oracle"]
    plans = [_plan(oracle, tid) for tid in range(N_THREADS)]
    for p in plans:
        p["dt"] = u.device_tensor(p["ot"])
        p["stats"] = torch.zeros(2, dtype=torch.int64, device=u.DEV)
        p["xd"] = u.to_dev(p["x"]).view(torch.bfloat16)
        p["y"] = torch.zeros((p["N"], p["T"], p["ot"].out_features), dtype=torch.bfloat16, device=u.DEV)
        p["stream"] = torch.cuda.Stream()
    torch.cuda.synchronize()
    start = threading.Barrier(N_THREADS)
    errors = []

    def worker(p):
        try:
            s = p["stream"].cuda_stream
            K = p["K"]
            start.wait()
            for c in range(CALLS):
                g = c + K                      # generation of this call; its window: the K before it
                qes.update(p["dt"], p["seeds"][g], p["fit"][g], p["seeds"][g - K:g], p["fit"][g - K:g], 1.0, 1.5, 0.9,
                           stats=p["stats"], stream=s)
            # population evaluation on the updated weights, behind the updates on the same stream
            qes.perturbed_qgemm(p["dt"], p["seeds"][0], 1.0, p["xd"], p["y"], stream=s)
            p["stream"].synchronize()
        except Exception as e:              # reported by the main thread
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(p,)) for p in plans]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a caller did not return"
    assert not errors, errors
    torch.cuda.synchronize()

    for tid, p in enumerate(plans):
        ot, K = p["ot"], p["K"]
        ref_stats = np.zeros(2, dtype=np.uint64)
        for c in range(CALLS):
            g = c + K
            ref_stats = oracle.update(ot, p["seeds"][g], p["fit"][g], p["seeds"][g - K:g], p["fit"][g - K:g], 1.0, 1.5,
                                      0.9, stats=ref_stats)
        assert (p["dt"].qweight.cpu().numpy() == ot.qweight).all(), tid
        assert (p["stats"].cpu().numpy().view(np.uint64) == ref_stats).all(), tid
        ref_y = oracle.perturbed_qgemm(ot, p["seeds"][0], 1.0, p["x"])
        ok, worst = u.bf16_close(p["y"].view(torch.int16).cpu().numpy().view(np.uint16), ref_y)
        assert ok, (tid, worst)
    assert sum(int(p["stats"][0]) for p in plans) > 100      # weights did move
