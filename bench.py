#!/usr/bin/env python3
"""Benchmark of the QES hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input for one configuration
of workloads.CONFIGS: the perturbed quantised GEMM of every linear layer for every member
(population evaluation), then the seeded update with a full replay window for every tensor.
Inputs are resident in HBM before the timed region starts. Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--no-cpu-baseline] [--no-extras]
    python bench.py --split-phase        (replay on a side stream during evaluation; its own JSON line)

The headline workload is config 5 (the 8B-shaped stack of App. C: 32 layers, 6.98 G parameters,
N=32, T=128, K=32), the largest configuration that runs on one GPU. After the timed steps the same
run measures, outside the timed region: the machine ceilings with the library's own probes, the
replay-only and Full-Residual entry points, and two steps of the smaller configurations.
"""
import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

# ---- roofline constants ---------------------------------------------------------------------------
# Vector ALU peak: MI355X's published fp32 vector rate is 157.3 TFLOP/s = 256 CUs x 4 SIMDs x
# 32 lanes x 2.4 GHz fused multiply-adds (2 flops each), i.e. 78.6e12 lane-operations per second.
VALU_PEAK_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12
# Algorithmic lane-operations, counted from docs/NOISE_SPEC.md as native 32-bit operations
# (tensor kernels: counter words 1 and 3 are zero, tensor id and key are wave-uniform):
#   Philox 18 wide multiplies + 34 xors = 52; uniforms 12; ln 16; sqrt (approximation + correction
#   to the correctly rounded value) and -2L 10; sin/cos 10; quadrant and the two products 11;
#   two stochastic roundings with clamp 14.
OPS_PER_PAIR_DRAW = 125.0
OPS_PER_MEMBER_ELEMENT_UPDATE = 2.0    # Eq. 5: int -> float and one fma per member and element
OPS_PER_EF_STEP = 11.0                 # Eq. 6-8 + gate, per element and generation
OPS_PER_MEMBER_ELEMENT_GEMM = 6.0      # Eq. 4 gate and the exact small-integer operand packing
MFMA_PEAK = {"bf16": 2.5e15, "i8": 5.0e15}
HBM_PEAK_GBPS = 8000.0
# Counter figures of the dominant kernel's launch (qes_update_batch over one layer's linears), from
# the rocprofv3 --pmc runs of this file summarised under profiles/. They hold for exactly the
# (config, N, K) they were measured on and are omitted for anything else.
#   traffic_bytes: FETCH_SIZE + WRITE_SIZE per launch, scaled by the same counters on the plain
#                  copy issued below;  valu_insts: SQ_INSTS_VALU (wave instructions) per launch.
MEASURED_PER_LAUNCH = {
    (5, 32, 32): {"traffic_bytes": (53443.0 * 2 + 1307.05) * 1024, "valu_insts": 1.96147e11},
    (4, 64, 32): {"traffic_bytes": (23175.7 * 2 + 0.09) * 1024, "valu_insts": 8.37747e10},
    (3, 30, 16): {"traffic_bytes": (11559.9 * 2 + 382.56) * 1024, "valu_insts": 2.03498e10},
    (2, 30, 8): {"traffic_bytes": (3296.94 * 2 + 44.30) * 1024, "valu_insts": 3.01387e9},
}
HEADLINE_CONFIG = 5


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=HEADLINE_CONFIG, choices=sorted(wl.CONFIGS))
    ap.add_argument("--layers", type=int, default=None, help="limit the number of layers (debug)")
    ap.add_argument("--K", type=int, default=None, help="override the replay window of the configuration")
    ap.add_argument("--N", type=int, default=None, help="override the population of the configuration")
    ap.add_argument("--per-tensor-gemm", action="store_true",
                    help="one qes_perturbed_qgemm call per tensor instead of one qes_perturbed_qgemm_batch call per layer")
    ap.add_argument("--per-tensor-update", action="store_true",
                    help="one qes_update call per tensor instead of one qes_update_batch call per layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip what runs after the timed steps: ceilings, replay-only and Full-Residual timings, "
                         "the two-step runs of the smaller configurations")
    ap.add_argument("--antithetic", action="store_true",
                    help="members come in +δ/-δ pairs sharing a seed (App. A.1); not the headline setting")
    ap.add_argument("--split-phase", action="store_true",
                    help="time one layer with the replay on a side stream next to the evaluation, then one Alg. 1 "
                         "step, against the single-call step (§4.6, App. E.2); prints its own JSON line")
    return ap.parse_args()


def update_ops_per_element(N, generations):
    return generations * (N * (OPS_PER_PAIR_DRAW / 2 + OPS_PER_MEMBER_ELEMENT_UPDATE) + OPS_PER_EF_STEP)


class Workload:
    """A configuration's tensors, activations and output buffers, resident in device memory."""

    def __init__(self, torch, qes, cfg, n_layers, dev):
        self.cfg, self.n_layers = cfg, n_layers
        self.layer_tensors = []
        for layer in range(n_layers):
            row = []
            for li, spec in enumerate(cfg.linears):
                qw = torch.from_numpy(wl.make_qweight(cfg, layer, li)).to(dev)
                sc = torch.from_numpy(wl.make_scales(cfg, layer, li).view(np.float16)).to(dev)
                row.append(qes.Tensor(qw, sc, spec.out_features, spec.in_features, cfg.bits, cfg.group_size,
                                      cfg.qmin, cfg.qmax, cfg.tensor_id(layer, li)))
            self.layer_tensors.append(row)
        xs = {}
        for spec in cfg.linears:
            if spec.x_key not in xs:
                xb = wl.make_activations(cfg, spec.x_key, spec.in_features)
                xs[spec.x_key] = torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16)
        self.layer_xs = [xs[spec.x_key] for spec in cfg.linears]
        # a batched launch writes all outputs of a layer at once: one buffer per linear, reused by every layer
        self.layer_ys = [torch.empty((cfg.N, cfg.T, spec.out_features), dtype=torch.bfloat16, device=dev)
                         for spec in cfg.linears]
        ws_bytes = max(max(qes.gemm_workspace_bytes(t, cfg.N, cfg.T, cfg.act_mode) for t in self.layer_tensors[0]),
                       qes.gemm_batch_workspace_bytes(self.layer_tensors[0], self.layer_xs, cfg.N, cfg.T, cfg.act_mode))
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
        self.stats = torch.zeros(2, dtype=torch.int64, device=dev)
        self.params = n_layers * sum(l.out_features * l.in_features for l in cfg.linears)


def run_steps(torch, qes, work, steps, warmup, anti=False, per_tensor_gemm=False, per_tensor_update=False,
              progress_lines=True):
    """warmup untimed steps, then `steps` timed ones bracketed by synchronisations. Returns the wall
    time per step and the HIP-event times (recorded on the launch stream) of the evaluation pass
    and of every update launch."""
    cfg, n_layers = work.cfg, work.n_layers
    total_steps = steps + warmup
    seeds = wl.make_seeds(cfg, cfg.K + total_steps, cfg.N // 2 if anti else cfg.N)
    fits = np.stack([qes.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + total_steps)])
    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
    gemm_events, upd_events = [], []

    def step(s, timed):
        # population evaluation: every linear, every member
        g0, g1 = ev(), ev()
        g0.record()
        for layer in range(n_layers):
            if per_tensor_gemm:
                for li, t in enumerate(work.layer_tensors[layer]):
                    qes.perturbed_qgemm(t, seeds[cfg.K + s], cfg.sigma, work.layer_xs[li], work.layer_ys[li],
                                        act_mode=cfg.act_mode, workspace=work.ws, antithetic=anti)
            else:
                # the linears of a layer share members and token count: one launch per layer
                qes.perturbed_qgemm_batch(work.layer_tensors[layer], seeds[cfg.K + s], cfg.sigma, work.layer_xs,
                                          work.layer_ys, act_mode=cfg.act_mode, workspace=work.ws, antithetic=anti)
        g1.record()
        # seeded update with a full replay window (steady state: K generations of history): all
        # linears of a layer share the generation's records and go in one call
        h0 = s
        for layer in range(n_layers):
            if per_tensor_update:
                for li, t in enumerate(work.layer_tensors[layer]):
                    u0, u1 = ev(), ev()
                    u0.record()
                    qes.update(t, seeds[cfg.K + s], fits[cfg.K + s], seeds[h0:h0 + cfg.K], fits[h0:h0 + cfg.K],
                               cfg.sigma, cfg.alpha, cfg.gamma, stats=work.stats, antithetic=anti)
                    u1.record()
                    if timed:
                        upd_events.append((li, u0, u1))
            else:
                u0, u1 = ev(), ev()
                u0.record()
                qes.update_batch(work.layer_tensors[layer], seeds[cfg.K + s], fits[cfg.K + s], seeds[h0:h0 + cfg.K],
                                 fits[h0:h0 + cfg.K], cfg.sigma, cfg.alpha, cfg.gamma, stats=work.stats, antithetic=anti)
                u1.record()
                if timed:
                    upd_events.append((-1, u0, u1))
        if timed:
            gemm_events.append((g0, g1))

    # progress goes to stderr (the host runs at most a few launches ahead of the device, so the
    # lines follow the real progress): a run of minutes must not look hung
    last_line = [time.perf_counter()]

    def progress(what, s):
        # about one line a minute, long runs only
        if progress_lines and time.perf_counter() - last_line[0] > 45.0:
            last_line[0] = time.perf_counter()
            print("bench.py: config %d %s step %d of %d enqueued" % (cfg.index, what, s + 1, total_steps), file=sys.stderr,
                  flush=True)

    for s in range(warmup):
        step(s, False)
        progress("warm-up", s)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for s in range(warmup, total_steps):
        step(s, True)
        progress("timed", s)
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    upd_ms_by_li = {}
    for li, a, b in upd_events:
        upd_ms_by_li.setdefault(li, []).append(a.elapsed_time(b))
    return {"ms_per_step": (t_end - t_begin) * 1e3 / steps,
            "gemm_ms": float(np.mean([a.elapsed_time(b) for a, b in gemm_events])),
            "upd_ms_by_li": {k: float(np.mean(v)) for k, v in upd_ms_by_li.items()}}


def part_figures(cfg, work, r, anti, per_tensor_update):
    """GEMM-only and update-only rates of a run, with the fractions of the MFMA, HBM and VALU peaks."""
    member_tokens = cfg.N * cfg.T
    mfma_dtype = "i8" if cfg.act_mode == 1 else "bf16"
    params = work.params
    draws_n = cfg.N // 2 if anti else cfg.N
    if per_tensor_update:
        upd_ms_total = float(sum(r["upd_ms_by_li"].values())) * work.n_layers
    else:
        upd_ms_total = r["upd_ms_by_li"][-1] * work.n_layers
    upd_gbps = params * (cfg.bits / 8.0 * 2.0) / (upd_ms_total * 1e-3) / 1e9      # packed W read + written
    upd_draws = params * (cfg.K + 1) * draws_n
    upd_ops = params * update_ops_per_element(draws_n, cfg.K + 1)
    gemm_s = r["gemm_ms"] * 1e-3
    return {
        "gemm_ms_per_pass": r["gemm_ms"],
        "gemm_member_tokens_per_s": member_tokens / gemm_s,
        "gemm_mfma_frac": 2.0 * params * member_tokens / gemm_s / MFMA_PEAK[mfma_dtype],
        "gemm_mfma_dtype": mfma_dtype,
        "gemm_draws_per_s": params * draws_n / gemm_s,
        "gemm_alu_frac": params * draws_n * (OPS_PER_PAIR_DRAW / 2 + OPS_PER_MEMBER_ELEMENT_GEMM) / gemm_s / 1e12
        / VALU_PEAK_TOPS,
        "update_ms_per_step": upd_ms_total,
        "update_gb_per_s": upd_gbps,
        "update_hbm_frac": upd_gbps / HBM_PEAK_GBPS,
        "update_draws_per_s": upd_draws / (upd_ms_total * 1e-3),
        "update_alu_frac": upd_ops / (upd_ms_total * 1e-3) / 1e12 / VALU_PEAK_TOPS,
    }


def time_call(torch, fn, reps, warm=1):
    """Mean HIP-event time in ms of fn() over reps calls on the current stream."""
    for _ in range(warm):
        fn()
    pairs = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    return float(np.mean([a.elapsed_time(b) for a, b in pairs]))


def measure_ceilings(torch, qes, dev):
    """What the machine sustains on each resource, measured with the library's own probe kernels in
    this run: Philox words/s and full pair draws/s (four chains per thread, eight waves per SIMD, no
    memory), bf16 and int8 matrix instructions on register operands, a plain streaming copy."""
    out = {}
    # the update kernel's launch shape: many short waves (256 rounds of 8 waves per SIMD, 64 pair draws
    # per thread), about 16 ms per launch. Two rounds of long-running waves measure 7 % less: whole
    # SIMDs idle while the last waves finish.
    n_threads = 256 * 4 * 8 * 64 * 256
    sink = torch.empty(n_threads, dtype=torch.int32, device=dev)
    iters = 64
    ms = time_call(torch, lambda: qes.bench_noise(0, n_threads, iters, 1.0, sink), 3, warm=2)
    out["philox_words_per_s"] = 4.0 * n_threads * iters / (ms * 1e-3)
    ms = time_call(torch, lambda: qes.bench_noise(1, n_threads, iters, 1.0, sink), 3, warm=2)
    out["pair_draws_per_s"] = n_threads * iters / (ms * 1e-3)
    out["draws_per_s"] = 2.0 * out["pair_draws_per_s"]
    del sink
    n_blocks, m_iters, tiles = 256 * 8, 16384, 8
    msink = torch.empty(n_blocks * 256, dtype=torch.int32, device=dev)
    ms = time_call(torch, lambda: qes.bench_mfma(0, n_blocks, m_iters, msink), 5)
    out["mfma_bf16_flop_per_s"] = n_blocks * 4.0 * m_iters * tiles * 16384.0 / (ms * 1e-3)
    ms = time_call(torch, lambda: qes.bench_mfma(1, n_blocks, m_iters, msink), 5)
    out["mfma_i8_op_per_s"] = n_blocks * 4.0 * m_iters * tiles * 32768.0 / (ms * 1e-3)
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    ms = time_call(torch, lambda: qes.bench_copy(src, dst, nbytes), 10, warm=2)
    out["copy_gb_per_s"] = 2.0 * nbytes / (ms * 1e-3) / 1e9          # read + written
    return out


def measure_update_variants(torch, qes, work, dev):
    """Entry points of the update family that the timed step does not call: the replay loop alone
    (qes_replay_residual, every tensor of layer 0) and single Alg. 1 steps on a stored residual
    (qes_update_full_residual, fp32 and binary16, the largest tensor; at the configured population and
    at N=2, where the step is closest to memory-bound)."""
    cfg = work.cfg
    seeds = wl.make_seeds(cfg, cfg.K + 1)
    fits = np.stack([qes.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + 1)])
    tensors = work.layer_tensors[0]
    big = max(tensors, key=lambda t: t.out_features * t.in_features)
    res = torch.zeros((big.out_features, big.in_features), dtype=torch.float32, device=dev)
    out = {}
    replay_ms = 0.0
    for t in tensors:
        view = res.view(-1)[: t.out_features * t.in_features].view(t.out_features, t.in_features)
        replay_ms += time_call(torch, lambda: qes.replay_residual(t, seeds[:cfg.K], fits[:cfg.K], cfg.N, cfg.sigma,
                                                                  cfg.alpha, cfg.gamma, view), 2)
    layer_elems = sum(t.out_features * t.in_features for t in tensors)
    out["replay_residual_ms_per_layer"] = replay_ms
    out["replay_residual_ms_per_step_est"] = replay_ms * cfg.n_layers
    out["replay_residual_draws_per_s"] = layer_elems * cfg.K * cfg.N / (replay_ms * 1e-3)
    # fp32 residual written: 4 bytes per element next to half a byte (INT4) or one byte (INT8) read
    out["replay_residual_gb_per_s"] = layer_elems * (cfg.bits / 8.0 + 4.0) / (replay_ms * 1e-3) / 1e9
    elems = big.out_features * big.in_features
    res16 = torch.zeros((big.out_features, big.in_features), dtype=torch.float16, device=dev)
    for name, state, half, e_bytes in (("f32", res, False, 8.0), ("f16", res16, True, 4.0)):
        for n_pop in sorted({cfg.N, 2}):
            state.zero_()
            ms = time_call(torch, lambda: qes.update_full_residual(big, seeds[cfg.K][:n_pop], fits[cfg.K][:n_pop],
                                                                   cfg.sigma, cfg.alpha, cfg.gamma, state, half=half), 10,
                           warm=2)
            gbps = elems * (cfg.bits / 8.0 * 2.0 + e_bytes) / (ms * 1e-3) / 1e9
            out["full_residual_%s_N%d" % (name, n_pop)] = {
                "tensor": "%dx%d" % (big.out_features, big.in_features), "ms": ms,
                "draws_per_s": elems * n_pop / (ms * 1e-3), "gb_per_s": gbps, "hbm_frac": gbps / HBM_PEAK_GBPS}
    return out


def split_phase(torch, qes, dev, cfg_index=3, reps=5):
    """One layer, two ways (§4.6, App. E.2: replay off the critical path). Single call: evaluation,
    then qes_update_batch (replay + step). Split: qes_replay_residual of every tensor on a side
    stream while the evaluation runs on the main stream, then one Alg. 1 step per tensor
    (qes_update_full_residual) on the replayed residual. Both produce the same weights."""
    cfg = wl.CONFIGS[cfg_index]
    work = Workload(torch, qes, cfg, 1, dev)
    seeds = wl.make_seeds(cfg, cfg.K + 1)
    fits = np.stack([qes.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + 1)])
    tensors = work.layer_tensors[0]
    residuals = [torch.empty((t.out_features, t.in_features), dtype=torch.float32, device=dev) for t in tensors]
    side = torch.cuda.Stream()

    def evaluate():
        qes.perturbed_qgemm_batch(tensors, seeds[cfg.K], cfg.sigma, work.layer_xs, work.layer_ys, act_mode=cfg.act_mode,
                                  workspace=work.ws)

    def single():
        evaluate()
        qes.update_batch(tensors, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha, cfg.gamma)

    def split():
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for t, r in zip(tensors, residuals):
                qes.replay_residual(t, seeds[:cfg.K], fits[:cfg.K], cfg.N, cfg.sigma, cfg.alpha, cfg.gamma, r)
        evaluate()
        torch.cuda.current_stream().wait_stream(side)
        for t, r in zip(tensors, residuals):
            qes.update_full_residual(t, seeds[cfg.K], fits[cfg.K], cfg.sigma, cfg.alpha, cfg.gamma, r)

    def after_rollout():
        for t, r in zip(tensors, residuals):
            qes.update_full_residual(t, seeds[cfg.K], fits[cfg.K], cfg.sigma, cfg.alpha, cfg.gamma, r)

    def wall(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps

    out = {"workload": "config %d, one layer (%s), N=%d, T=%d, K=%d" % (cfg.index, "/".join(l.name for l in cfg.linears),
                                                                      cfg.N, cfg.T, cfg.K),
           "evaluation_ms": wall(evaluate), "single_call_step_ms": wall(single), "split_phase_step_ms": wall(split),
           "work_after_last_rollout_single_ms": None, "work_after_last_rollout_split_ms": wall(after_rollout)}
    out["work_after_last_rollout_single_ms"] = out["single_call_step_ms"] - out["evaluation_ms"]
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no sharding, no collectives).", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2602_03120_amd as qes

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    if args.split_phase:
        print(json.dumps({"metric": "split-phase step time", "unit": "ms", "n_gpus": 1, **split_phase(torch, qes, dev)}))
        return
    cfg = wl.CONFIGS[args.config]
    overridden = args.K is not None or args.N is not None or args.layers is not None
    if args.K is not None or args.N is not None:
        # the replay window is a cost knob (§4.6, App. E.2: cost linear in K); not the headline setting
        cfg = dataclasses.replace(cfg, K=cfg.K if args.K is None else args.K, N=cfg.N if args.N is None else args.N)
        if not (0 <= cfg.K <= 256 and 1 <= cfg.N <= 1024):
            print("bench.py: --K must be in 0..256 and --N in 1..1024", file=sys.stderr)
            sys.exit(2)
    n_layers = cfg.n_layers if args.layers is None else min(args.layers, cfg.n_layers)
    big = cfg.params > 100_000_000
    steps = args.steps if args.steps is not None else (3 if big else 20)
    warmup = args.warmup if args.warmup is not None else (1 if big else 3)
    anti = args.antithetic
    if anti and cfg.N % 2:
        print("bench.py: --antithetic needs an even population", file=sys.stderr)
        sys.exit(2)

    work = Workload(torch, qes, cfg, n_layers, dev)
    # one plain copy of known size before the timed region: the reference dispatch that scales the
    # rocprofv3 FETCH_SIZE / WRITE_SIZE counters of the same run
    copy_bytes = 256 << 20
    copy_src = torch.empty(copy_bytes, dtype=torch.uint8, device=dev)
    copy_dst = torch.empty(copy_bytes, dtype=torch.uint8, device=dev)
    qes.bench_copy(copy_src, copy_dst, copy_bytes)
    torch.cuda.synchronize()
    del copy_src, copy_dst

    r = run_steps(torch, qes, work, steps, warmup, anti, args.per_tensor_gemm, args.per_tensor_update)
    ms_per_step = r["ms_per_step"]
    member_tokens = cfg.N * cfg.T
    value = member_tokens / (ms_per_step * 1e-3)
    parts = part_figures(cfg, work, r, anti, args.per_tensor_update)
    parts["weights_changed_total"] = int(work.stats[0].item())
    parts["gated_total"] = int(work.stats[1].item())

    # dominant kernel: the update. One launch = one layer's linears (qes_update_batch), or, with
    # --per-tensor-update, the largest tensor shape (most launches x longest)
    draws_n = cfg.N // 2 if anti else cfg.N
    if args.per_tensor_update:
        dom_li = max(range(len(cfg.linears)), key=lambda i: cfg.linears[i].out_features * cfg.linears[i].in_features)
        dom = cfg.linears[dom_li]
        dom_ms = r["upd_ms_by_li"][dom_li]
        dom_elems = dom.out_features * dom.in_features
        dom_name = "update_kernel (qes_update, %s %dx%d)" % (dom.name, dom.out_features, dom.in_features)
        counters = None
    else:
        dom_ms = r["upd_ms_by_li"][-1]
        dom_elems = sum(l.out_features * l.in_features for l in cfg.linears)
        dom_name = "update_kernel (qes_update_batch, one layer: %s)" % "+".join(l.name for l in cfg.linears)
        counters = None if anti else MEASURED_PER_LAUNCH.get((cfg.index, cfg.N, cfg.K))
    ops = dom_elems * update_ops_per_element(draws_n, cfg.K + 1)
    achieved_tops = ops / (dom_ms * 1e-3) / 1e12
    roofline = {
        "kernel": dom_name,
        "bound": "alu", "achieved": achieved_tops, "peak": VALU_PEAK_TOPS, "unit": "Tlane-op/s",
        "frac": achieved_tops / VALU_PEAK_TOPS,
        "traffic": counters["traffic_bytes"] if counters else None,
        "traffic_source": "static: rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE summary under profiles/ for this config, N and K"
        if counters else None,
        "avg_launch_ms": dom_ms,
        "algorithmic_ops_per_launch": ops,
        "algorithmic_ops_per_pair_draw": OPS_PER_PAIR_DRAW,
        "algorithmic_bytes_per_launch": dom_elems * cfg.bits / 8.0 * 2.0,
        # issued vector instructions (SQ_INSTS_VALU, 64 lanes each) against the same peak: what the
        # compiled kernel actually occupies the VALUs with, as opposed to the hand count above
        "issue_frac": counters["valu_insts"] * 64.0 / (dom_ms * 1e-3) / 1e12 / VALU_PEAK_TOPS if counters else None,
        # wave instructions per wave-wide pair draw (64 lanes draw 64 pairs at a time)
        "valu_insts_per_pair_draw": counters["valu_insts"] / (dom_elems / 2.0 * (cfg.K + 1) * draws_n / 64.0)
        if counters else None,
        "draws_per_s": dom_elems * (cfg.K + 1) * draws_n / (dom_ms * 1e-3),
    }

    out = {
        "metric": "member-tokens/s",
        "value": value,
        "unit": "member-tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32+f32 noise/update; %s MFMA" % parts["gemm_mfma_dtype"],
        "data": "synthetic",
        "config": {"workload": "config %d: %s (%d layers of %s), N=%d, T=%d, K=%d, sigma=%g, alpha=%g, gamma=%g"
                   % (cfg.index, cfg.name, n_layers, "/".join(l.name for l in cfg.linears), cfg.N, cfg.T, cfg.K,
                      cfg.sigma, cfg.alpha, cfg.gamma),
                   "parameters": work.params, "step": "perturbed qGEMM of every linear + update with full replay window; %s"
                   % ("GEMM: one call per %s, update: one call per %s"
                      % ("tensor" if args.per_tensor_gemm else "layer", "tensor" if args.per_tensor_update else "layer")),
                   "antithetic_pairs": bool(anti), "overridden": bool(overridden)},
        # the two figures the stated metric names literally, for this workload (details in parts)
        "baseline_metrics": {
            "qgemm_member_tokens_per_s": parts["gemm_member_tokens_per_s"],
            "qgemm_mfma_frac": parts["gemm_mfma_frac"],
            "update_replay_gb_per_s": parts["update_gb_per_s"],
            "update_replay_hbm_frac": parts["update_hbm_frac"],
        },
        "roofline": roofline,
        "parts": parts,
    }

    if not args.no_extras:
        print("bench.py: timed steps done (%.1f ms per step); measuring ceilings and the other entry points" % ms_per_step,
              file=sys.stderr, flush=True)
        ceilings = measure_ceilings(torch, qes, dev)
        out["ceilings"] = ceilings
        # the binding resource, against what the same generator sustains with nothing else to do
        roofline["frac_of_measured_noise_ceiling"] = roofline["draws_per_s"] / ceilings["draws_per_s"]
        parts["gemm_frac_of_measured_noise_ceiling"] = parts["gemm_draws_per_s"] / ceilings["draws_per_s"]
        parts.update(measure_update_variants(torch, qes, work, dev))
        if not overridden and not anti and cfg.index == HEADLINE_CONFIG:
            # the same workload with antithetic perturbation pairs (App. A.1: N/2 seeds, members 2j and
            # 2j+1 on +δ and -δ): half the noise work; reported beside the headline, not as it
            ra = run_steps(torch, qes, work, 2, 1, anti=True)
            pa = part_figures(cfg, work, ra, True, False)
            parts["antithetic_pairs"] = {"ms_per_step": ra["ms_per_step"],
                                         "member_tokens_per_s": member_tokens / (ra["ms_per_step"] * 1e-3),
                                         "gemm_ms_per_pass": pa["gemm_ms_per_pass"],
                                         "update_ms_per_step": pa["update_ms_per_step"],
                                         "note": "2 steps after 1 warm-up, same tensors and inputs"}
            del work
            torch.cuda.empty_cache()
            others = {}
            for index in (2, 3, 4):
                c = wl.CONFIGS[index]
                w2 = Workload(torch, qes, c, c.n_layers, dev)
                r2 = run_steps(torch, qes, w2, 2, 1)
                p2 = part_figures(c, w2, r2, False, False)
                p2["ms_per_step"] = r2["ms_per_step"]
                p2["member_tokens_per_s"] = c.N * c.T / (r2["ms_per_step"] * 1e-3)
                p2["workload"] = "config %d: %s, %d layers, N=%d, T=%d, K=%d; 2 steps after 1 warm-up" % (
                    c.index, c.name, c.n_layers, c.N, c.T, c.K)
                others[str(index)] = p2
                del w2
                torch.cuda.empty_cache()
            parts["configs"] = others

    if not args.no_cpu_baseline and not anti:
        print("bench.py: timing the CPU oracle on a sample of the workload", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(cfg, member_tokens)
    print(json.dumps(out))


def cpu_baseline(cfg, member_tokens):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the same
    workload: evenly spaced output rows of every tensor of layer 0 (the same share of each tensor),
    all members, tokens and generations. Reported in the metric's unit by scaling the sample's time
    to the whole step."""
    import oracle
    cores = len(os.sched_getaffinity(0))
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    # aim at roughly 8e9 draws of work in the sample (10-20 s on 16 cores)
    layer_params = sum(l.out_features * l.in_features for l in cfg.linears)
    step_draws = float(layer_params) * cfg.n_layers * cfg.N * (cfg.K + 2)
    share = min(1.0, 8.0e9 / step_draws * cfg.n_layers)          # of layer 0's rows
    seeds = wl.make_seeds(cfg, cfg.K + 1)
    fits = np.stack([oracle.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + 1)])
    xs = {}
    sample_elems = 0
    t0 = time.perf_counter()
    t_prep = 0.0
    for li, spec in enumerate(cfg.linears):
        p0 = time.perf_counter()
        n_rows = max(1, int(round(spec.out_features * share)))
        rows = np.unique(np.linspace(0, spec.out_features - 1, n_rows).astype(np.int32))
        w = oracle.Tensor(wl.make_qweight(cfg, 0, li), wl.make_scales(cfg, 0, li), spec.out_features,
                          spec.in_features, cfg.bits, cfg.group_size, cfg.qmin, cfg.qmax, cfg.tensor_id(0, li))
        if spec.x_key not in xs:
            xs[spec.x_key] = wl.make_activations(cfg, spec.x_key, spec.in_features)
        t_prep += time.perf_counter() - p0
        oracle.perturbed_qgemm(w, seeds[cfg.K], cfg.sigma, xs[spec.x_key], act_mode=cfg.act_mode, rows=rows)
        oracle.update(w, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha, cfg.gamma,
                      rows=rows)
        sample_elems += rows.size * spec.in_features
    elapsed = time.perf_counter() - t0 - t_prep
    frac = sample_elems / float(layer_params * cfg.n_layers)
    est_step_s = elapsed / frac
    return {"value": member_tokens / est_step_s, "unit": "member-tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%.3g of the output rows of each tensor of layer 0, evenly spaced (%.3g of the step's elements), "
                      "all members, tokens and generations: GEMM and update; %.1f s of oracle time scaled to the whole step"
                      % (share, frac, elapsed)}


if __name__ == "__main__":
    main()
