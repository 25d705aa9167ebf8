"""Seeded synthetic inputs shaped like the QES workloads.

This module serves both the CPU oracle's tests and the GPU path's tests and benchmark. It holds
none of the method's arithmetic: only shapes, formats and random fills (numpy PCG64 streams), plus
the bfloat16/float16 bit conversions needed to lay the data out.

The tensors stand in for GPTQ / LLM-Compressor quantised Qwen2.5 and Llama-3.1 linear layers
(paper §4.1, App. A.3, App. C), which need model weights that are not available here: shapes and
formats follow those models, values are uniform over the integer range.

Every array is generated from its own stream `SeedSequence([BASE_SEED + config, layer, slot])`, so
any tensor of any layer can be regenerated alone (the large configs are checked on slices).
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

BASE_SEED = 20260203

# slots of the per-array streams
_SLOT_W, _SLOT_S, _SLOT_X, _SLOT_TARGET, _SLOT_SEEDS, _SLOT_REWARD = 0, 1, 2, 3, 4, 5


@dataclass(frozen=True)
class LinearSpec:
    name: str
    out_features: int
    in_features: int
    x_key: str  # layers with the same key read the same activation tensor


@dataclass(frozen=True)
class Config:
    index: int
    name: str
    linears: Tuple[LinearSpec, ...]
    n_layers: int
    bits: int
    group_size: int  # 0 = one scale per output row
    qmin: int
    qmax: int
    N: int          # population
    T: int          # tokens per member
    K: int          # replay window
    sigma: float
    alpha: float
    gamma: float
    iters: int
    act_mode: int   # 0 = bf16 activations, 1 = per-token int8 activations (W8A8)
    fitness: str    # "mse" (from GEMM outputs) or "normal" (seeded scalar per member)

    @property
    def params(self) -> int:
        return self.n_layers * sum(l.out_features * l.in_features for l in self.linears)

    def tensor_id(self, layer: int, li: int) -> int:
        return layer * len(self.linears) + li + 1


def _mlp(h, inter):
    return (LinearSpec("gate", inter, h, "h"), LinearSpec("up", inter, h, "h"),
            LinearSpec("down", h, inter, "i"))


def _block(h, kv, inter):
    return (LinearSpec("q", h, h, "h"), LinearSpec("k", kv, h, "h"), LinearSpec("v", kv, h, "h"),
            LinearSpec("o", h, h, "a")) + _mlp(h, inter)


CONFIGS: Dict[int, Config] = {
    1: Config(1, "tiny-int4-g32", (LinearSpec("lin", 256, 256, "h"),), 1, 4, 32, -8, 7,
              N=8, T=16, K=4, sigma=1.0, alpha=0.5, gamma=0.9, iters=4, act_mode=0, fitness="mse"),
    2: Config(2, "mlp-0.5b-int4-g128", _mlp(896, 4864), 1, 4, 128, -8, 7,
              N=30, T=64, K=8, sigma=1.0, alpha=0.3, gamma=0.9, iters=10, act_mode=0, fitness="mse"),
    3: Config(3, "stack-1.5b-int4-g128", _block(1536, 256, 8960), 28, 4, 128, -8, 7,
              N=30, T=256, K=16, sigma=1.0, alpha=0.3, gamma=0.9, iters=1, act_mode=0, fitness="normal"),
    4: Config(4, "stack-1.5b-w8a8", _block(1536, 256, 8960), 28, 8, 0, -127, 127,
              N=64, T=512, K=32, sigma=1.0, alpha=0.3, gamma=0.9, iters=1, act_mode=1, fitness="normal"),
    5: Config(5, "stack-8b-int4-g128", _block(4096, 1024, 14336), 32, 4, 128, -8, 7,
              N=32, T=128, K=32, sigma=1.0, alpha=0.3, gamma=0.9, iters=1, act_mode=0, fitness="normal"),
}


def _rng(cfg_index: int, layer: int, slot: int, extra: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([BASE_SEED + cfg_index, layer, slot, extra])
    return np.random.Generator(np.random.PCG64(ss))


# ---------------------------------------------------------------- bit-level format helpers

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even. Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f16_bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(b, dtype=np.uint16).view(np.float16).astype(np.float32)


def pack_int4(q: np.ndarray) -> np.ndarray:
    """int array [out,in] in [-8,7] -> uint8 [out,in/2]; even column in the low nibble."""
    q = np.asarray(q)
    assert q.shape[-1] % 2 == 0
    lo = (q[..., 0::2] & 0xF).astype(np.uint8)
    hi = (q[..., 1::2] & 0xF).astype(np.uint8)
    return (lo | (hi << 4)).astype(np.uint8)


# ---------------------------------------------------------------- generators

def make_qweight(cfg: Config, layer: int, li: int, rows: slice = None) -> np.ndarray:
    """Packed integer weights of one linear: uint8 [out,in/2] (bits=4) or int8 [out,in] (bits=8).

    Uniform over the full range: int4 bytes uniform in 0..255 (each nibble uniform in [-8,7]);
    int8 uniform in [-127,127]. Uniform weights put 1/16 of INT4 elements on each range edge, far
    more than GPTQ weights do: a deliberate stress of the gate.
    """
    spec = cfg.linears[li]
    rng = _rng(cfg.index, layer, _SLOT_W, li)
    if cfg.bits == 4:
        w = rng.integers(0, 256, size=(spec.out_features, spec.in_features // 2), dtype=np.uint8)
        if cfg.qmin > -8:  # symmetric 4-bit range: fold -8 onto qmin
            lo, hi = w & 0xF, w >> 4
            lo = np.where(lo == 8, (cfg.qmin & 0xF), lo)
            hi = np.where(hi == 8, (cfg.qmin & 0xF), hi)
            w = (lo | (hi << 4)).astype(np.uint8)
    else:
        w = rng.integers(cfg.qmin, cfg.qmax + 1, size=(spec.out_features, spec.in_features), dtype=np.int8)
    return w if rows is None else w[rows]


def make_scales(cfg: Config, layer: int, li: int) -> np.ndarray:
    """fp16 scale bit patterns ~U(0.005, 0.02): [out,in/group] or [out]."""
    spec = cfg.linears[li]
    rng = _rng(cfg.index, layer, _SLOT_S, li)
    shape = (spec.out_features, spec.in_features // cfg.group_size) if cfg.group_size else (spec.out_features,)
    return f16_bits(rng.uniform(0.005, 0.02, size=shape).astype(np.float32))


def make_activations(cfg: Config, x_key: str, in_features: int, N: int = None, T: int = None) -> np.ndarray:
    """bf16 bit patterns [N,T,in] ~ N(0,1); one tensor per distinct x_key, shared by all layers."""
    N = cfg.N if N is None else N
    T = cfg.T if T is None else T
    rng = _rng(cfg.index, 0, _SLOT_X, sum(ord(c) for c in x_key))
    return f32_to_bf16_bits(rng.standard_normal(size=(N, T, in_features), dtype=np.float32))


def make_target(cfg: Config, li: int, N: int = None, T: int = None) -> np.ndarray:
    """Fixed random bf16 target [T,out] for the -MSE fitness of the small configs."""
    spec = cfg.linears[li]
    T = cfg.T if T is None else T
    rng = _rng(cfg.index, 0, _SLOT_TARGET, li)
    return f32_to_bf16_bits(rng.standard_normal(size=(T, spec.out_features), dtype=np.float32))


def make_seeds(cfg: Config, steps: int, N: int = None) -> np.ndarray:
    """uint64 member seeds [steps,N], uniform in [0, 2^63)."""
    N = cfg.N if N is None else N
    rng = _rng(cfg.index, 0, _SLOT_SEEDS)
    return rng.integers(0, 2 ** 63, size=(steps, N), dtype=np.uint64)


def make_rewards(cfg: Config, steps: int, N: int = None) -> np.ndarray:
    """Synthetic scalar reward per member ~N(0,1), float32 [steps,N] (normalised by the caller)."""
    N = cfg.N if N is None else N
    rng = _rng(cfg.index, 0, _SLOT_REWARD)
    return rng.standard_normal(size=(steps, N)).astype(np.float32)


def sample_rows(cfg: Config, layer: int, li: int, n_random: int = 64) -> np.ndarray:
    """First, last and n_random seeded-random distinct rows of a tensor, sorted (slice checks)."""
    out = cfg.linears[li].out_features
    rng = _rng(cfg.index, layer, 99, li)
    pick = set([0, out - 1])
    if out > 2:
        pick.update(int(v) for v in rng.choice(out, size=min(n_random, out), replace=False))
    return np.array(sorted(pick), dtype=np.int32)


def random_tensor(seed: int, out_features: int, in_features: int, bits: int, group_size: int,
                  qmin: int = None, qmax: int = None):
    """Free-form random quantised tensor for unit tests: (qweight, scale_bits, qmin, qmax)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if qmin is None:
        qmin, qmax = (-8, 7) if bits == 4 else (-127, 127)
    q = rng.integers(qmin, qmax + 1, size=(out_features, in_features), dtype=np.int64)
    qw = pack_int4(q) if bits == 4 else q.astype(np.int8)
    shape = (out_features, in_features // group_size) if group_size else (out_features,)
    sc = f16_bits(rng.uniform(0.005, 0.02, size=shape).astype(np.float32))
    return qw, sc, qmin, qmax
