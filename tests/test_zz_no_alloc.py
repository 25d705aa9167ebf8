"""GPU test of qes_update_noalloc, the entry point for callers that cannot allocate: same results
as qes_update (weights bit-exact, counters equal) on two calls in a row, the second with a smaller
input, so that whatever the first call left in the library's fixed device array is seen not to
leak into the second. Called through the C ABI like every other GPU test."""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2602_03120_amd as qes
    import gpu_util
    assert torch.cuda.is_available()
    return dict(torch=torch, qes=qes, u=gpu_util)


def _case(env, seed, out_f, in_f, bits, N, K):
    """One update through both entry points from identical inputs; returns what both produced."""
    torch, qes, u = env["torch"], env["qes"], env["u"]
    rng = np.random.default_rng(seed)
    qw, _, qmin, qmax = wl.random_tensor(seed, out_f, in_f, bits, 0)
    seeds = rng.integers(0, 2 ** 63, size=(K + 1, N), dtype=np.uint64)
    fit = np.stack([qes.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(K + 1)])
    out = []
    for noalloc in (False, True):
        t = qes.Tensor(u.to_dev(qw), None, out_f, in_f, bits, 0, qmin, qmax, 11)
        stats = torch.zeros(2, dtype=torch.int64, device=u.DEV)
        qes.update(t, seeds[K], fit[K], seeds[:K], fit[:K], 1.0, 1.5, 0.9, stats=stats, noalloc=noalloc)
        torch.cuda.synchronize()
        out.append((t.qweight.cpu().numpy().view(np.uint8), stats.cpu().numpy().copy()))
    return qw.view(np.uint8), out


def test_two_calls_in_a_row_second_smaller(env):
    # first call: 3 staging launches (600 records), ragged tensor; second: fewer records, smaller tensor
    for seed, out_f, in_f, bits, N, K in [(5, 96, 130, 4, 40, 14), (6, 17, 34, 8, 7, 2)]:
        before, (ref, got) = _case(env, seed, out_f, in_f, bits, N, K)
        assert (got[0] == ref[0]).all(), (out_f, in_f)
        assert (got[1] == ref[1]).all() and ref[1][0] > 0
        assert (ref[0] != before).any()


def test_no_history_and_limit(env):
    torch, qes, u = env["torch"], env["qes"], env["u"]
    before, (ref, got) = _case(env, 9, 8, 64, 4, 5, 0)
    assert (got[0] == ref[0]).all() and (got[1] == ref[1]).all()
    # one record more than the fixed array holds is refused, and nothing is written
    qw, _, qmin, qmax = wl.random_tensor(3, 8, 64, 4, 0)
    t = qes.Tensor(u.to_dev(qw), None, 8, 64, 4, 0, qmin, qmax, 1)
    N, K = 1024, 16          # 17 * 1024 = 17408 > 16384
    with pytest.raises(qes.QesError) as err:
        qes.update(t, np.zeros(N, np.uint64), np.zeros(N, np.float32), np.zeros((K, N), np.uint64),
                   np.zeros((K, N), np.float32), 1.0, 0.5, 0.9, noalloc=True)
    assert err.value.status == -5
    torch.cuda.synchronize()
    assert (t.qweight.cpu().numpy().view(np.uint8) == qw.view(np.uint8)).all()
    # exactly at the limit: 16 generations of 1024 members
    K = 15
    rng = np.random.default_rng(2)
    seeds = rng.integers(0, 2 ** 63, size=(K + 1, N), dtype=np.uint64)
    fit = np.stack([qes.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(K + 1)])
    t2 = qes.Tensor(u.to_dev(qw), None, 8, 64, 4, 0, qmin, qmax, 1)
    qes.update(t, seeds[K], fit[K], seeds[:K], fit[:K], 1.0, 4.0, 0.9, noalloc=True)
    qes.update(t2, seeds[K], fit[K], seeds[:K], fit[:K], 1.0, 4.0, 0.9)
    assert torch.equal(t.qweight, t2.qweight)


def test_captured_in_a_hip_graph_and_replayed(env):
    """The call enqueues kernel launches only, so it can be captured: the records travel in the
    captured kernels' arguments. Three replays, with eager work and synchronisations in between, must
    leave the weights where three eager calls of qes_update leave them (the update is in place, so
    replay k starts from the weights replay k-1 produced)."""
    torch, qes, u = env["torch"], env["qes"], env["u"]
    rng = np.random.default_rng(21)
    out_f, in_f, N, K = 64, 192, 12, 5
    qw, _, qmin, qmax = wl.random_tensor(21, out_f, in_f, 4, 0)
    seeds = rng.integers(0, 2 ** 63, size=(K + 1, N), dtype=np.uint64)
    fit = np.stack([qes.normalize_fitness(rng.standard_normal(N).astype(np.float32)) for _ in range(K + 1)])
    eager = qes.Tensor(u.to_dev(qw), None, out_f, in_f, 4, 0, qmin, qmax, 4)
    graphed = qes.Tensor(u.to_dev(qw), None, out_f, in_f, 4, 0, qmin, qmax, 4)
    warm = qes.Tensor(u.to_dev(qw), None, out_f, in_f, 4, 0, qmin, qmax, 4)
    # the first call on a device looks up the fixed array's address: outside the capture
    qes.update(warm, seeds[K], fit[K], seeds[:K], fit[:K], 1.0, 1.5, 0.9, noalloc=True)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph.capture_begin()
        qes.update(graphed, seeds[K], fit[K], seeds[:K], fit[:K], 1.0, 1.5, 0.9, noalloc=True, stream=side.cuda_stream)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert torch.equal(graphed.qweight.cpu(), torch.from_numpy(qw))        # capturing ran nothing
    for k in range(3):
        graph.replay()
        qes.update(eager, seeds[K], fit[K], seeds[:K], fit[:K], 1.0, 1.5, 0.9)
        # another call through the same fixed array between the replays: the graph carries its own records
        other = qes.Tensor(u.to_dev(qw), None, out_f, in_f, 4, 0, qmin, qmax, 9)
        qes.update(other, seeds[0], fit[0], None, None, 1.0, 1.5, 0.9, noalloc=True)
        torch.cuda.synchronize()
        assert torch.equal(graphed.qweight, eager.qweight), k
    assert not torch.equal(graphed.qweight.cpu(), torch.from_numpy(qw))
