"""ctypes front end of the CPU oracle (oracle/qes_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg. The GPU package never imports this module and this module never imports it.
All arrays are numpy, all pointers are host pointers. bf16 and fp16 travel as uint16 bit patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


class OracleTensor(ctypes.Structure):
    _fields_ = [
        ("qweight", ctypes.c_void_p),
        ("scales", ctypes.c_void_p),
        ("out_features", ctypes.c_int32),
        ("in_features", ctypes.c_int32),
        ("bits", ctypes.c_int32),
        ("group_size", ctypes.c_int32),
        ("qmin", ctypes.c_int32),
        ("qmax", ctypes.c_int32),
        ("tensor_id", ctypes.c_uint32),
    ]


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        u64, u32, i32, f32, vp, sz = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int32,
                                      ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t)
        tp = ctypes.POINTER(OracleTensor)
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_philox4x32_10.restype = None
        L.oracle_ln_u1.argtypes = [u32]
        L.oracle_ln_u1.restype = f32
        L.oracle_sincos_quarter.argtypes = [f32, vp, vp]
        L.oracle_sincos_quarter.restype = None
        L.oracle_noise_words.argtypes = [u64, u32, u64, u64, vp]
        L.oracle_noise_words.restype = None
        L.oracle_noise_gauss.argtypes = [u64, u32, u64, u64, vp]
        L.oracle_noise_gauss.restype = None
        L.oracle_noise_delta.argtypes = [u64, u32, u64, u64, f32, vp]
        L.oracle_noise_delta.restype = None
        L.oracle_noise_from_words.argtypes = [vp, u64, f32, vp, vp]
        L.oracle_noise_from_words.restype = None
        L.oracle_delta_from_gauss.argtypes = [f32, u32, f32]
        L.oracle_delta_from_gauss.restype = i32
        L.oracle_perturbed_qgemm.argtypes = [tp, vp, vp, i32, f32, vp, i32, vp, i32, vp, i32, i32]
        L.oracle_perturbed_qgemm.restype = i32
        L.oracle_normalize_fitness.argtypes = [vp, i32, vp]
        L.oracle_normalize_fitness.restype = i32
        L.oracle_replay_residual.argtypes = [tp, vp, vp, i32, i32, f32, f32, f32, vp, vp, i32, i32]
        L.oracle_replay_residual.restype = i32
        L.oracle_update.argtypes = [tp, vp, vp, vp, vp, i32, i32, f32, f32, f32, vp, vp, i32, i32]
        L.oracle_update.restype = i32
        L.oracle_update_full_residual.argtypes = [tp, vp, vp, i32, f32, f32, f32, vp, vp, vp]
        L.oracle_update_full_residual.restype = i32
        L.oracle_update_stochastic_rounding.argtypes = [tp, vp, vp, i32, f32, f32, u64, vp, vp, i32]
        L.oracle_update_stochastic_rounding.restype = i32
        L.oracle_update_full_residual_f16.argtypes = [tp, vp, vp, i32, f32, f32, f32, vp, vp]
        L.oracle_update_full_residual_f16.restype = i32
        L.oracle_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.oracle_f16_to_f32.restype = f32
        L.oracle_f32_to_f16_sat.argtypes = [f32]
        L.oracle_f32_to_f16_sat.restype = ctypes.c_uint16
        L.oracle_aggregate.argtypes = [tp, vp, vp, i32, f32, vp, i32]
        L.oracle_aggregate.restype = i32
        _LIB = L
    return _LIB


def _ptr(a):
    return None if a is None else a.ctypes.data


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


class Tensor:
    """Host-side quantised linear weight: packed qweight (uint8 or int8) + fp16 scale bits."""

    def __init__(self, qweight, scales, out_features, in_features, bits, group_size, qmin, qmax,
                 tensor_id):
        self.qweight = np.ascontiguousarray(qweight)
        self.scales = None if scales is None else _c(scales, np.uint16)
        self.out_features, self.in_features = int(out_features), int(in_features)
        self.bits, self.group_size = int(bits), int(group_size)
        self.qmin, self.qmax, self.tensor_id = int(qmin), int(qmax), int(tensor_id)
        nbytes = self.out_features * self.in_features * self.bits // 8
        assert self.qweight.nbytes == nbytes, (self.qweight.nbytes, nbytes)

    def desc(self):
        return OracleTensor(_ptr(self.qweight), _ptr(self.scales), self.out_features,
                            self.in_features, self.bits, self.group_size, self.qmin, self.qmax,
                            self.tensor_id)

    def copy(self):
        return Tensor(self.qweight.copy(), self.scales, self.out_features, self.in_features,
                      self.bits, self.group_size, self.qmin, self.qmax, self.tensor_id)

    def unpacked(self):
        """int32 [out,in] view of the integer weights (a copy)."""
        if self.bits == 8:
            return self.qweight.view(np.int8).reshape(self.out_features, self.in_features).astype(np.int32)
        b = self.qweight.view(np.uint8).reshape(self.out_features, self.in_features // 2)
        lo = (b & 0xF).astype(np.int32)
        hi = (b >> 4).astype(np.int32)
        lo = np.where(lo >= 8, lo - 16, lo)
        hi = np.where(hi >= 8, hi - 16, hi)
        out = np.empty((self.out_features, self.in_features), dtype=np.int32)
        out[:, 0::2] = lo
        out[:, 1::2] = hi
        return out


def _check(rc):
    if rc != 0:
        raise ValueError(f"oracle returned {rc}")


def philox4x32_10(ctr, key):
    ctr = _c(ctr, np.uint32)
    key = _c(key, np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_ptr(ctr), _ptr(key), _ptr(out))
    return out


def ln_u1(m):
    return float(lib().oracle_ln_u1(int(m)))


def sincos_quarter(f):
    s = ctypes.c_float()
    c = ctypes.c_float()
    lib().oracle_sincos_quarter(float(f), ctypes.addressof(s), ctypes.addressof(c))
    return s.value, c.value


def noise_words(seed, tensor_id, pair_begin, n_pairs):
    out = np.empty((n_pairs, 4), dtype=np.uint32)
    lib().oracle_noise_words(seed, tensor_id, pair_begin, n_pairs, _ptr(out))
    return out


def noise_gauss(seed, tensor_id, elem_begin, n_elems):
    out = np.empty(n_elems, dtype=np.float32)
    lib().oracle_noise_gauss(seed, tensor_id, elem_begin, n_elems, _ptr(out))
    return out


def noise_delta(seed, tensor_id, elem_begin, n_elems, sigma):
    out = np.empty(n_elems, dtype=np.int8)
    lib().oracle_noise_delta(seed, tensor_id, elem_begin, n_elems, sigma, _ptr(out))
    return out


def noise_from_words(words, sigma):
    """words: uint32 [n,4] -> (eps float32 [n,2], delta int8 [n,2])."""
    words = _c(words, np.uint32).reshape(-1, 4)
    n = words.shape[0]
    eps = np.empty((n, 2), dtype=np.float32)
    delta = np.empty((n, 2), dtype=np.int8)
    lib().oracle_noise_from_words(_ptr(words), n, sigma, _ptr(eps), _ptr(delta))
    return eps, delta


def delta_from_gauss(eps, wround, sigma):
    return int(lib().oracle_delta_from_gauss(float(eps), int(wround), float(sigma)))


def _rows(rows):
    if rows is None:
        return None, 0
    r = _c(rows, np.int32)
    return r, int(r.size)


def perturbed_qgemm(w, seeds, sigma, x, act_mode=0, perturb_mask=None, rows=None, y=None, antithetic=False):
    """x: uint16 bf16 bits [N,T,in] -> y: uint16 bf16 bits [N,T,out] (only `rows` columns written).
    antithetic: seeds has N/2 entries; members 2j, 2j+1 use +δ_j, -δ_j."""
    seeds = _c(seeds, np.uint64)
    x = _c(x, np.uint16)
    N, T, K = x.shape
    assert K == w.in_features and seeds.size == (N // 2 if antithetic else N)
    if y is None:
        y = np.zeros((N, T, w.out_features), dtype=np.uint16)
    mask = None if perturb_mask is None else _c(perturb_mask, np.uint8)
    r, nr = _rows(rows)
    d = w.desc()
    _check(lib().oracle_perturbed_qgemm(ctypes.byref(d), _ptr(seeds), _ptr(mask), N, sigma, _ptr(x),
                                        T, _ptr(y), act_mode, _ptr(r), nr, int(antithetic)))
    return y


def normalize_fitness(reward):
    reward = _c(reward, np.float32)
    fit = np.empty_like(reward)
    _check(lib().oracle_normalize_fitness(_ptr(reward), reward.size, _ptr(fit)))
    return fit


def _hist(hist_seeds, hist_fit, N, antithetic=False):
    if hist_seeds is None or len(hist_seeds) == 0:
        return None, None, 0
    hs = _c(hist_seeds, np.uint64).reshape(-1, N // 2 if antithetic else N)
    hf = _c(hist_fit, np.float32).reshape(-1, N)
    assert hs.shape[0] == hf.shape[0]
    return hs, hf, hs.shape[0]


def replay_residual(w, hist_seeds, hist_fit, N, sigma, alpha, gamma, rows=None, residual=None, antithetic=False):
    hs, hf, hl = _hist(hist_seeds, hist_fit, N, antithetic)
    if residual is None:
        residual = np.zeros((w.out_features, w.in_features), dtype=np.float32)
    r, nr = _rows(rows)
    d = w.desc()
    _check(lib().oracle_replay_residual(ctypes.byref(d), _ptr(hs), _ptr(hf), hl, N, sigma, alpha,
                                        gamma, _ptr(residual), _ptr(r), nr, int(antithetic)))
    return residual


def update(w, seeds_t, fit_t, hist_seeds, hist_fit, sigma, alpha, gamma, rows=None, stats=None, antithetic=False):
    """In-place Alg. 2 on w.qweight. Returns stats (uint64[2]: changed, gated) accumulated.
    antithetic: seeds arrays hold one seed per pair (N/2 per generation), fitnesses one per member."""
    seeds_t = _c(seeds_t, np.uint64)
    fit_t = _c(fit_t, np.float32)
    N = fit_t.size
    assert seeds_t.size == (N // 2 if antithetic else N)
    hs, hf, hl = _hist(hist_seeds, hist_fit, N, antithetic)
    if stats is None:
        stats = np.zeros(2, dtype=np.uint64)
    r, nr = _rows(rows)
    d = w.desc()
    _check(lib().oracle_update(ctypes.byref(d), _ptr(seeds_t), _ptr(fit_t), _ptr(hs), _ptr(hf), hl, N,
                               sigma, alpha, gamma, _ptr(stats), _ptr(r), nr, int(antithetic)))
    return stats


def update_full_residual(w, seeds_t, fit_t, sigma, alpha, gamma, e_state, want_u=False, stats=None):
    """In-place Alg. 1 step on w.qweight and e_state (float32 [out,in])."""
    seeds_t = _c(seeds_t, np.uint64)
    fit_t = _c(fit_t, np.float32)
    N = seeds_t.size
    assert e_state.dtype == np.float32 and e_state.flags.c_contiguous
    u = np.empty_like(e_state) if want_u else None
    if stats is None:
        stats = np.zeros(2, dtype=np.uint64)
    d = w.desc()
    _check(lib().oracle_update_full_residual(ctypes.byref(d), _ptr(seeds_t), _ptr(fit_t), N, sigma,
                                             alpha, gamma, _ptr(e_state), _ptr(u), _ptr(stats)))
    return u, stats


def update_full_residual_f16(w, seeds_t, fit_t, sigma, alpha, gamma, e_state, stats=None):
    """In-place Alg. 1 step on w.qweight and e_state (binary16 bit patterns, uint16 [out,in])."""
    seeds_t = _c(seeds_t, np.uint64)
    fit_t = _c(fit_t, np.float32)
    assert e_state.dtype == np.uint16 and e_state.flags.c_contiguous
    if stats is None:
        stats = np.zeros(2, dtype=np.uint64)
    d = w.desc()
    _check(lib().oracle_update_full_residual_f16(ctypes.byref(d), _ptr(seeds_t), _ptr(fit_t), seeds_t.size, sigma,
                                                 alpha, gamma, _ptr(e_state), _ptr(stats)))
    return stats


def update_stochastic_rounding(w, seeds_t, fit_t, sigma, alpha, round_seed, stats=None, rows=None):
    """In-place stateless step with stochastic rounding of the update (baseline of the paper's §5)."""
    seeds_t = _c(seeds_t, np.uint64)
    fit_t = _c(fit_t, np.float32)
    if stats is None:
        stats = np.zeros(2, dtype=np.uint64)
    rows_a = None if rows is None else _c(rows, np.int32)
    d = w.desc()
    _check(lib().oracle_update_stochastic_rounding(ctypes.byref(d), _ptr(seeds_t), _ptr(fit_t), seeds_t.size, sigma,
                                                   alpha, int(round_seed), _ptr(stats), _ptr(rows_a),
                                                   0 if rows_a is None else rows_a.size))
    return stats


def f16_to_f32(h):
    return float(lib().oracle_f16_to_f32(int(h)))


def f32_to_f16_sat(f):
    return int(lib().oracle_f32_to_f16_sat(float(f)))


def aggregate(w, seeds, fit, sigma, antithetic=False):
    seeds = _c(seeds, np.uint64)
    fit = _c(fit, np.float32)
    assert seeds.size == (fit.size // 2 if antithetic else fit.size)
    g = np.empty((w.out_features, w.in_features), dtype=np.float32)
    d = w.desc()
    _check(lib().oracle_aggregate(ctypes.byref(d), _ptr(seeds), _ptr(fit), fit.size, sigma, _ptr(g), int(antithetic)))
    return g
