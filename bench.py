#!/usr/bin/env python3
"""Benchmark of the QES hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input for one configuration
of workloads.CONFIGS: the perturbed quantised GEMM of every linear layer for every member
(population evaluation), then the seeded update with a full replay window for every tensor.
Inputs are resident in HBM before the timed region starts. Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-cpu-baseline]
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
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this file, scaled by the same counters on the plain copy issued below (see profiles/):
# {(config, what one launch covers): bytes}: one layer's linears (qes_update_batch), or one tensor
# with --per-tensor-update. A launch covers that much whatever --layers says.
MEASURED_TRAFFIC_BYTES = {(2, "layer"): 6.79e6, (3, "layer"): 24.06e6, (4, "layer"): 47.46e6, (5, "layer"): 110.8e6,
                          (2, "gate"): 2.374e6, (3, "gate"): 7.223e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=2, choices=sorted(wl.CONFIGS))
    ap.add_argument("--layers", type=int, default=None, help="limit the number of layers (debug)")
    ap.add_argument("--K", type=int, default=None, help="override the replay window of the configuration")
    ap.add_argument("--N", type=int, default=None, help="override the population of the configuration")
    ap.add_argument("--per-tensor-gemm", action="store_true",
                    help="one qes_perturbed_qgemm call per tensor instead of one qes_perturbed_qgemm_batch call per layer")
    ap.add_argument("--per-tensor-update", action="store_true",
                    help="one qes_update call per tensor instead of one qes_update_batch call per layer")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--antithetic", action="store_true",
                    help="members come in +δ/-δ pairs sharing a seed (App. A.1); not the headline setting")
    return ap.parse_args()


def update_ops_per_element(N, generations):
    return generations * (N * (OPS_PER_PAIR_DRAW / 2 + OPS_PER_MEMBER_ELEMENT_UPDATE) + OPS_PER_EF_STEP)


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
    cfg = wl.CONFIGS[args.config]
    if args.K is not None or args.N is not None:
        # the replay window is a cost knob (§4.6, App. E.2: cost linear in K); not the headline setting
        cfg = dataclasses.replace(cfg, K=cfg.K if args.K is None else args.K, N=cfg.N if args.N is None else args.N)
        if not (0 <= cfg.K <= 256 and 1 <= cfg.N <= 1024):
            print("bench.py: --K must be in 0..256 and --N in 1..1024", file=sys.stderr)
            sys.exit(2)
    n_layers = cfg.n_layers if args.layers is None else min(args.layers, cfg.n_layers)
    big = cfg.params > 100_000_000
    steps = args.steps if args.steps is not None else (2 if big else 20)
    warmup = args.warmup if args.warmup is not None else (1 if big else 3)

    # ---------------- inputs, resident in HBM
    tensors = []   # (layer, li, qes.Tensor)
    for layer in range(n_layers):
        for li, spec in enumerate(cfg.linears):
            qw = torch.from_numpy(wl.make_qweight(cfg, layer, li)).to(dev)
            sc = torch.from_numpy(wl.make_scales(cfg, layer, li).view(np.float16)).to(dev)
            tensors.append((layer, li, qes.Tensor(qw, sc, spec.out_features, spec.in_features, cfg.bits,
                                                  cfg.group_size, cfg.qmin, cfg.qmax, cfg.tensor_id(layer, li))))
    xs = {}
    for spec in cfg.linears:
        if spec.x_key not in xs:
            xb = wl.make_activations(cfg, spec.x_key, spec.in_features)
            xs[spec.x_key] = torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16)
    layer_tensors = [[t for la, _, t in tensors if la == layer] for layer in range(n_layers)]
    layer_xs = [xs[spec.x_key] for spec in cfg.linears]
    # a batched launch writes all outputs of a layer at once: one buffer per linear
    layer_ys = [torch.empty((cfg.N, cfg.T, spec.out_features), dtype=torch.bfloat16, device=dev) for spec in cfg.linears]
    ws_bytes = max(max(qes.gemm_workspace_bytes(t, cfg.N, cfg.T, cfg.act_mode) for _, _, t in tensors),
                   qes.gemm_batch_workspace_bytes(layer_tensors[0], layer_xs, cfg.N, cfg.T, cfg.act_mode))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
    stats = torch.zeros(2, dtype=torch.int64, device=dev)
    # one plain copy of known size before the timed region: the reference dispatch that scales the
    # rocprofv3 FETCH_SIZE / WRITE_SIZE counters of the same run
    copy_bytes = 256 << 20
    copy_src = torch.empty(copy_bytes, dtype=torch.uint8, device=dev)
    copy_dst = torch.empty(copy_bytes, dtype=torch.uint8, device=dev)
    qes.bench_copy(copy_src, copy_dst, copy_bytes)
    torch.cuda.synchronize()
    del copy_src, copy_dst

    total_steps = steps + warmup
    anti = args.antithetic
    if anti and cfg.N % 2:
        print("bench.py: --antithetic needs an even population", file=sys.stderr)
        sys.exit(2)
    seeds = wl.make_seeds(cfg, cfg.K + total_steps, cfg.N // 2 if anti else cfg.N)
    rewards = wl.make_rewards(cfg, cfg.K + total_steps)
    fits = np.stack([qes.normalize_fitness(r) for r in rewards])

    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
    gemm_events, upd_events = [], []

    def step(s, timed):
        # population evaluation: every linear, every member
        g0, g1 = ev(), ev()
        g0.record()
        if args.per_tensor_gemm:
            for layer, li, t in tensors:
                spec = cfg.linears[li]
                qes.perturbed_qgemm(t, seeds[cfg.K + s], cfg.sigma, xs[spec.x_key], layer_ys[li],
                                    act_mode=cfg.act_mode, workspace=ws, antithetic=anti)
        else:
            # the linears of a layer share members and token count: one launch per layer
            for layer in range(n_layers):
                qes.perturbed_qgemm_batch(layer_tensors[layer], seeds[cfg.K + s], cfg.sigma, layer_xs, layer_ys,
                                          act_mode=cfg.act_mode, workspace=ws, antithetic=anti)
        g1.record()
        # seeded update with a full replay window (steady state: K generations of history): all
        # linears of a layer share the generation's records and go in one call
        h0 = s
        if args.per_tensor_update:
            for layer, li, t in tensors:
                u0, u1 = ev(), ev()
                u0.record()
                qes.update(t, seeds[cfg.K + s], fits[cfg.K + s], seeds[h0:h0 + cfg.K], fits[h0:h0 + cfg.K],
                           cfg.sigma, cfg.alpha, cfg.gamma, stats=stats, antithetic=anti)
                u1.record()
                if timed:
                    upd_events.append((li, u0, u1))
        else:
            for layer in range(n_layers):
                u0, u1 = ev(), ev()
                u0.record()
                qes.update_batch(layer_tensors[layer], seeds[cfg.K + s], fits[cfg.K + s], seeds[h0:h0 + cfg.K],
                                 fits[h0:h0 + cfg.K], cfg.sigma, cfg.alpha, cfg.gamma, stats=stats, antithetic=anti)
                u1.record()
                if timed:
                    upd_events.append((-1, u0, u1))
        if timed:
            gemm_events.append((g0, g1))

    for s in range(warmup):
        step(s, False)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for s in range(warmup, total_steps):
        step(s, True)
    torch.cuda.synchronize()
    t_end = time.perf_counter()

    ms_per_step = (t_end - t_begin) * 1e3 / steps
    member_tokens = cfg.N * cfg.T
    value = member_tokens / (ms_per_step * 1e-3)

    # ---------------- per-part figures from HIP events recorded on the launch stream
    gemm_ms = float(np.mean([a.elapsed_time(b) for a, b in gemm_events]))
    params = n_layers * sum(l.out_features * l.in_features for l in cfg.linears)
    mfma_dtype = "i8" if cfg.act_mode == 1 else "bf16"
    gemm_flops = 2.0 * params * member_tokens
    upd_ms_by_li = {}
    for li, a, b in upd_events:
        upd_ms_by_li.setdefault(li, []).append(a.elapsed_time(b))
    # dominant kernel: the update. One launch = one layer's linears (qes_update_batch), or, with
    # --per-tensor-update, the largest tensor shape (most launches x longest)
    if args.per_tensor_update:
        dom_li = max(range(len(cfg.linears)), key=lambda i: cfg.linears[i].out_features * cfg.linears[i].in_features)
        dom = cfg.linears[dom_li]
        dom_ms = float(np.mean(upd_ms_by_li[dom_li]))
        dom_elems = dom.out_features * dom.in_features
        dom_name = "update_kernel (qes_update, %s %dx%d)" % (dom.name, dom.out_features, dom.in_features)
        traffic_key = (cfg.index, dom.name)
        upd_ms_total = float(sum(np.mean(v) for v in upd_ms_by_li.values())) * n_layers
    else:
        dom_ms = float(np.mean(upd_ms_by_li[-1]))
        dom_elems = sum(l.out_features * l.in_features for l in cfg.linears)
        dom_name = "update_kernel (qes_update_batch, one layer: %s)" % "+".join(l.name for l in cfg.linears)
        traffic_key = (cfg.index, "layer")
        upd_ms_total = dom_ms * n_layers
    ops = dom_elems * update_ops_per_element(cfg.N // 2 if anti else cfg.N, cfg.K + 1)
    achieved_tops = ops / (dom_ms * 1e-3) / 1e12
    bytes_per_param = cfg.bits / 8.0 * 2.0          # packed W read + written
    upd_gbps = params * bytes_per_param / (upd_ms_total * 1e-3) / 1e9
    upd_draws = params * (cfg.K + 1) * (cfg.N // 2 if anti else cfg.N)

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
        "dtype": "int32+f32 noise/update; %s MFMA" % mfma_dtype,
        "data": "synthetic",
        "config": {"workload": "config %d: %s (%d layers of %s), N=%d, T=%d, K=%d, sigma=%g, alpha=%g, gamma=%g"
                   % (cfg.index, cfg.name, n_layers, "/".join(l.name for l in cfg.linears), cfg.N, cfg.T, cfg.K,
                      cfg.sigma, cfg.alpha, cfg.gamma),
                   "parameters": params, "step": "perturbed qGEMM of every linear + update with full replay window; %s"
                   % ("GEMM: one call per %s, update: one call per %s"
                      % ("tensor" if args.per_tensor_gemm else "layer", "tensor" if args.per_tensor_update else "layer")),
                   "antithetic_pairs": bool(anti)},
        "roofline": {
            "kernel": dom_name,
            "bound": "alu", "achieved": achieved_tops, "peak": VALU_PEAK_TOPS, "unit": "Tlane-op/s",
            "frac": achieved_tops / VALU_PEAK_TOPS,
            "traffic": None if anti else MEASURED_TRAFFIC_BYTES.get(traffic_key),
            "avg_launch_ms": dom_ms,
            "algorithmic_ops_per_launch": ops,
            "algorithmic_bytes_per_launch": dom_elems * cfg.bits / 8.0 * 2.0,
        },
        "parts": {
            "gemm_ms_per_pass": gemm_ms,
            "gemm_member_tokens_per_s": member_tokens / (gemm_ms * 1e-3),
            "gemm_mfma_frac": gemm_flops / (gemm_ms * 1e-3) / MFMA_PEAK[mfma_dtype],
            "gemm_draws_per_s": params * cfg.N / (gemm_ms * 1e-3),
            "gemm_alu_frac": params * cfg.N * (OPS_PER_PAIR_DRAW / 2 + OPS_PER_MEMBER_ELEMENT_GEMM)
            / (gemm_ms * 1e-3) / 1e12 / VALU_PEAK_TOPS,
            "update_ms_per_step": upd_ms_total,
            "update_gb_per_s": upd_gbps,
            "update_hbm_frac": upd_gbps / HBM_PEAK_GBPS,
            "update_draws_per_s": upd_draws / (upd_ms_total * 1e-3),
            "weights_changed_total": int(stats[0].item()), "gated_total": int(stats[1].item()),
        },
    }

    if not args.no_cpu_baseline and not anti:
        out["cpu_baseline"] = cpu_baseline(cfg, member_tokens)
    print(json.dumps(out))


def cpu_baseline(cfg, member_tokens):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the same
    workload: a fixed stride of output rows of every tensor of layer 0, all members, tokens and
    generations. Reported in the metric's unit by scaling the sample's time to the whole step."""
    import oracle
    cores = len(os.sched_getaffinity(0))
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    # aim at roughly 8e9 draws of work in the sample (10-20 s on 16 cores)
    layer_params = sum(l.out_features * l.in_features for l in cfg.linears)
    step_draws = layer_params * cfg.n_layers * cfg.N * (cfg.K + 2)
    stride = max(1, int(round(step_draws / 8.0e9)))
    seeds = wl.make_seeds(cfg, cfg.K + 1)
    fits = np.stack([oracle.normalize_fitness(r) for r in wl.make_rewards(cfg, cfg.K + 1)])
    xs = {}
    sample_rows_total = 0
    t0 = time.perf_counter()
    t_prep = 0.0
    for li, spec in enumerate(cfg.linears):
        p0 = time.perf_counter()
        rows = np.arange(0, spec.out_features, stride * cfg.n_layers, dtype=np.int32)
        w = oracle.Tensor(wl.make_qweight(cfg, 0, li), wl.make_scales(cfg, 0, li), spec.out_features,
                          spec.in_features, cfg.bits, cfg.group_size, cfg.qmin, cfg.qmax, cfg.tensor_id(0, li))
        if spec.x_key not in xs:
            xs[spec.x_key] = wl.make_activations(cfg, spec.x_key, spec.in_features)
        t_prep += time.perf_counter() - p0
        oracle.perturbed_qgemm(w, seeds[cfg.K], cfg.sigma, xs[spec.x_key], act_mode=cfg.act_mode, rows=rows)
        oracle.update(w, seeds[cfg.K], fits[cfg.K], seeds[:cfg.K], fits[:cfg.K], cfg.sigma, cfg.alpha, cfg.gamma,
                      rows=rows)
        sample_rows_total += rows.size * spec.in_features
    elapsed = time.perf_counter() - t0 - t_prep
    frac = sample_rows_total / float(layer_params * cfg.n_layers)
    est_step_s = elapsed / frac
    return {"value": member_tokens / est_step_s, "unit": "member-tokens/s", "cores": cores, "kind": "oracle",
            "sample": "every %d-th output row of each tensor of layer 0 (%.4g of the step's elements), all members, "
                      "tokens and generations; %.1f s of oracle time scaled to the whole step"
                      % (stride * cfg.n_layers, frac, elapsed)}


if __name__ == "__main__":
    main()
