"""ctypes binding of the C ABI declared in include/qes.h. Same names, same arguments.

Device buffers are torch tensors on a ROCm device (used as plain memory: data_ptr()); the stream is
torch's current stream unless one is passed. Host arrays are numpy. Nothing here computes.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libqes.so")
_lib = None


class QesError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = status_string(status) if _lib is not None else str(status)
        extra = f" (hipError {_lib.qes_last_hip_error()})" if _lib is not None and status == -3 else ""
        super().__init__(f"{where}: {msg}{extra}")


class _QesTensor(ctypes.Structure):
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


def library_path():
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2602_03120_amd.build` "
                          "(there is no fallback path)")
    L = ctypes.CDLL(_LIB_PATH)
    u64, u32, i32, f32, vp, sz = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int32, ctypes.c_float,
                                  ctypes.c_void_p, ctypes.c_size_t)
    tp = ctypes.POINTER(_QesTensor)
    sigs = {
        "qes_noise_words": ([u64, u32, u64, u64, vp, vp], i32),
        "qes_noise_gauss": ([u64, u32, u64, u64, vp, vp], i32),
        "qes_noise_delta": ([u64, u32, u64, u64, f32, vp, vp], i32),
        "qes_noise_from_words": ([vp, u64, f32, vp, vp, vp], i32),
        "qes_perturbed_qgemm": ([tp, vp, vp, i32, f32, vp, i32, vp, i32, vp, sz, vp], i32),
        "qes_perturbed_qgemm_antithetic": ([tp, vp, vp, i32, f32, vp, i32, vp, i32, vp, sz, vp], i32),
        "qes_gemm_workspace_bytes": ([tp, i32, i32, i32], sz),
        "qes_update": ([tp, vp, vp, vp, vp, i32, i32, f32, f32, f32, vp, vp], i32),
        "qes_update_noalloc": ([tp, vp, vp, vp, vp, i32, i32, f32, f32, f32, vp, vp], i32),
        "qes_perturbed_qgemm_batch": ([vp, i32, vp, vp, i32, f32, vp, i32, vp, i32, vp, sz, vp], i32),
        "qes_perturbed_qgemm_batch_antithetic": ([vp, i32, vp, vp, i32, f32, vp, i32, vp, i32, vp, sz, vp], i32),
        "qes_gemm_batch_workspace_bytes": ([vp, i32, vp, i32, i32, i32], sz),
        "qes_update_batch": ([vp, i32, vp, vp, vp, vp, i32, i32, f32, f32, f32, vp, vp], i32),
        "qes_update_batch_antithetic": ([vp, i32, vp, vp, vp, vp, i32, i32, f32, f32, f32, vp, vp], i32),
        "qes_replay_residual": ([tp, vp, vp, i32, i32, f32, f32, f32, vp, vp], i32),
        "qes_update_antithetic": ([tp, vp, vp, vp, vp, i32, i32, f32, f32, f32, vp, vp], i32),
        "qes_replay_residual_antithetic": ([tp, vp, vp, i32, i32, f32, f32, f32, vp, vp], i32),
        "qes_update_full_residual": ([tp, vp, vp, i32, f32, f32, f32, vp, vp, vp], i32),
        "qes_update_full_residual_f16": ([tp, vp, vp, i32, f32, f32, f32, vp, vp, vp], i32),
        "qes_update_stochastic_rounding": ([tp, vp, vp, i32, f32, f32, u64, vp, vp], i32),
        "qes_normalize_fitness": ([vp, i32, vp], i32),
        "qes_bench_noise": ([i32, u64, i32, f32, vp, vp], i32),
        "qes_bench_mfma": ([i32, u32, i32, vp, vp], i32),
        "qes_bench_copy": ([vp, vp, sz, vp], i32),
        "qes_status_string": ([i32], ctypes.c_char_p),
        "qes_last_hip_error": ([], i32),
        "qes_abi_version": ([], i32),
    }
    for name, (args, res) in sigs.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = res
    _lib = L
    return L


EXPORTS = ["qes_noise_words", "qes_noise_gauss", "qes_noise_delta", "qes_noise_from_words", "qes_perturbed_qgemm",
           "qes_perturbed_qgemm_antithetic", "qes_gemm_workspace_bytes", "qes_perturbed_qgemm_batch",
           "qes_perturbed_qgemm_batch_antithetic", "qes_gemm_batch_workspace_bytes", "qes_update", "qes_update_noalloc", "qes_update_antithetic",
           "qes_update_batch", "qes_update_batch_antithetic",
           "qes_replay_residual", "qes_replay_residual_antithetic", "qes_update_full_residual", "qes_update_full_residual_f16",
           "qes_update_stochastic_rounding", "qes_normalize_fitness",
           "qes_bench_noise", "qes_bench_mfma", "qes_bench_copy", "qes_status_string", "qes_last_hip_error",
           "qes_abi_version"]


def status_string(status):
    return _load().qes_status_string(int(status)).decode()


def abi_version():
    return int(_load().qes_abi_version())


def _check(rc, where):
    if rc != 0:
        raise QesError(rc, where)


def _stream(stream):
    if stream is not None:
        return int(stream)
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _dev_ptr(t, name):
    """Device pointer of a torch tensor used as plain memory."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    return int(t.data_ptr())


def _host(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _hptr(a):
    return None if a is None else a.ctypes.data


class Tensor:
    """A quantised linear weight living in device memory (the qes_tensor of include/qes.h).

    qweight: torch uint8 [out,in/2] (bits=4) or int8 [out,in] (bits=8) on the device.
    scales : torch float16 [out,in/group] or [out] on the device, or None (update only).
    """

    def __init__(self, qweight, scales, out_features, in_features, bits, group_size, qmin, qmax, tensor_id):
        self.qweight, self.scales = qweight, scales
        self.out_features, self.in_features = int(out_features), int(in_features)
        self.bits, self.group_size = int(bits), int(group_size)
        self.qmin, self.qmax, self.tensor_id = int(qmin), int(qmax), int(tensor_id)
        nbytes = self.out_features * self.in_features * self.bits // 8
        if qweight.numel() * qweight.element_size() != nbytes:
            raise ValueError("qweight has the wrong size")

    def desc(self):
        return _QesTensor(_dev_ptr(self.qweight, "qweight"), _dev_ptr(self.scales, "scales"),
                          self.out_features, self.in_features, self.bits, self.group_size, self.qmin,
                          self.qmax, self.tensor_id)


def noise_words(seed, tensor_id, pair_begin, n_pairs, out, stream=None):
    """out: device uint32/int32 tensor with n_pairs*4 elements."""
    _check(_load().qes_noise_words(seed, tensor_id, pair_begin, n_pairs, _dev_ptr(out, "out"), _stream(stream)),
           "qes_noise_words")


def noise_gauss(seed, tensor_id, elem_begin, n_elems, out, stream=None):
    _check(_load().qes_noise_gauss(seed, tensor_id, elem_begin, n_elems, _dev_ptr(out, "out"), _stream(stream)),
           "qes_noise_gauss")


def noise_delta(seed, tensor_id, elem_begin, n_elems, sigma, out, stream=None):
    _check(_load().qes_noise_delta(seed, tensor_id, elem_begin, n_elems, sigma, _dev_ptr(out, "out"),
                                   _stream(stream)), "qes_noise_delta")


def noise_from_words(words, n, sigma, eps2=None, delta2=None, stream=None):
    """words: device int32/uint32 [n,4]; eps2: device float32 [n,2] or None; delta2: device int8 [n,2] or None."""
    _check(_load().qes_noise_from_words(_dev_ptr(words, "words"), n, sigma, _dev_ptr(eps2, "eps2"),
                                        _dev_ptr(delta2, "delta2"), _stream(stream)), "qes_noise_from_words")


def gemm_workspace_bytes(w, N, T, act_mode):
    d = w.desc()
    return int(_load().qes_gemm_workspace_bytes(ctypes.byref(d), N, T, act_mode))


def perturbed_qgemm(w, seeds, sigma, x, y, act_mode=0, perturb_mask=None, workspace=None, stream=None,
                    antithetic=False):
    """x: device bf16 [N,T,in]; y: device bf16 [N,T,out] (written). seeds: host uint64 [N], or [N/2]
    pair seeds with antithetic=True (qes_perturbed_qgemm_antithetic)."""
    seeds = _host(seeds, np.uint64)
    mask = _host(perturb_mask, np.uint8)
    N, T = int(x.shape[0]), int(x.shape[1])
    if seeds.size != (N // 2 if antithetic else N) or (mask is not None and mask.size != N) or (antithetic and N % 2):
        raise ValueError("seeds / perturb_mask do not match the population")
    if x.shape[2] != w.in_features or tuple(y.shape) != (N, T, w.out_features):
        raise ValueError("x / y shapes do not match the tensor")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    d = w.desc()
    fn = _load().qes_perturbed_qgemm_antithetic if antithetic else _load().qes_perturbed_qgemm
    _check(fn(ctypes.byref(d), _hptr(seeds), _hptr(mask), N, sigma, _dev_ptr(x, "x"), T, _dev_ptr(y, "y"), act_mode,
              _dev_ptr(workspace, "workspace"), ws_bytes, _stream(stream)),
           "qes_perturbed_qgemm_antithetic" if antithetic else "qes_perturbed_qgemm")


def _batch_arrays(tensors, xs, ys=None):
    descs = (_QesTensor * len(tensors))(*[t.desc() for t in tensors])
    xp = (ctypes.c_void_p * len(tensors))(*[_dev_ptr(x, "x") for x in xs])
    yp = None if ys is None else (ctypes.c_void_p * len(tensors))(*[_dev_ptr(y, "y") for y in ys])
    return descs, xp, yp


def gemm_batch_workspace_bytes(tensors, xs, N, T, act_mode):
    descs, xp, _ = _batch_arrays(tensors, xs)
    return int(_load().qes_gemm_batch_workspace_bytes(ctypes.cast(descs, ctypes.c_void_p), len(tensors),
                                                      ctypes.cast(xp, ctypes.c_void_p), N, T, act_mode))


def perturbed_qgemm_batch(tensors, seeds, sigma, xs, ys, act_mode=0, perturb_mask=None, workspace=None, stream=None,
                          antithetic=False):
    """perturbed_qgemm for a list of tensors in one call: xs[i] device bf16 [N,T,in_i] (tensors may share
    one), ys[i] device bf16 [N,T,out_i] (written)."""
    seeds = _host(seeds, np.uint64)
    mask = _host(perturb_mask, np.uint8)
    if len(tensors) == 0 or len(xs) != len(tensors) or len(ys) != len(tensors):
        raise ValueError("tensors, xs and ys differ in length")
    N, T = int(xs[0].shape[0]), int(xs[0].shape[1])
    if seeds.size != (N // 2 if antithetic else N) or (mask is not None and mask.size != N) or (antithetic and N % 2):
        raise ValueError("seeds / perturb_mask do not match the population")
    for w, x, y in zip(tensors, xs, ys):
        if tuple(x.shape) != (N, T, w.in_features) or tuple(y.shape) != (N, T, w.out_features):
            raise ValueError("x / y shapes do not match the tensor")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    descs, xp, yp = _batch_arrays(tensors, xs, ys)
    name = "qes_perturbed_qgemm_batch_antithetic" if antithetic else "qes_perturbed_qgemm_batch"
    _check(getattr(_load(), name)(ctypes.cast(descs, ctypes.c_void_p), len(tensors), _hptr(seeds), _hptr(mask), N, sigma,
                                  ctypes.cast(xp, ctypes.c_void_p), T, ctypes.cast(yp, ctypes.c_void_p), act_mode,
                                  _dev_ptr(workspace, "workspace"), ws_bytes, _stream(stream)), name)


def _hist(hist_seeds, hist_fit, N, antithetic=False):
    if hist_seeds is None or len(hist_seeds) == 0:
        return None, None, 0
    hs = _host(hist_seeds, np.uint64).reshape(-1, N // 2 if antithetic else N)
    hf = _host(hist_fit, np.float32).reshape(-1, N)
    if hs.shape[0] != hf.shape[0]:
        raise ValueError("history seeds and fitnesses differ in length")
    return hs, hf, int(hs.shape[0])


def update(w, seeds_t, fit_t, hist_seeds, hist_fit, sigma, alpha, gamma, stats=None, stream=None, antithetic=False,
           noalloc=False):
    """In-place Alg. 2 on w.qweight. stats: device int64/uint64 tensor [2] or None. antithetic=True:
    one seed per pair (N/2 per generation), one fitness per member (qes_update_antithetic).
    noalloc=True: qes_update_noalloc (records staged in the library's fixed device array)."""
    seeds_t = _host(seeds_t, np.uint64)
    fit_t = _host(fit_t, np.float32)
    N = int(fit_t.size)
    if seeds_t.size != (N // 2 if antithetic else N) or (antithetic and N % 2):
        raise ValueError("seeds_t and fit_t do not match")
    if noalloc and antithetic:
        raise ValueError("qes_update_noalloc has no antithetic form")
    hs, hf, hl = _hist(hist_seeds, hist_fit, N, antithetic)
    d = w.desc()
    name = "qes_update_noalloc" if noalloc else ("qes_update_antithetic" if antithetic else "qes_update")
    _check(getattr(_load(), name)(ctypes.byref(d), _hptr(seeds_t), _hptr(fit_t), _hptr(hs), _hptr(hf), hl, N, sigma,
                                  alpha, gamma, _dev_ptr(stats, "stats"), _stream(stream)), name)


def update_batch(tensors, seeds_t, fit_t, hist_seeds, hist_fit, sigma, alpha, gamma, stats=None, stream=None,
                 antithetic=False):
    """In-place Alg. 2 on every tensor of a list in one call (qes_update_batch): same arguments as update()."""
    seeds_t = _host(seeds_t, np.uint64)
    fit_t = _host(fit_t, np.float32)
    N = int(fit_t.size)
    if seeds_t.size != (N // 2 if antithetic else N) or (antithetic and N % 2):
        raise ValueError("seeds_t and fit_t do not match")
    hs, hf, hl = _hist(hist_seeds, hist_fit, N, antithetic)
    descs = (_QesTensor * len(tensors))(*[t.desc() for t in tensors])
    name = "qes_update_batch_antithetic" if antithetic else "qes_update_batch"
    _check(getattr(_load(), name)(ctypes.cast(descs, ctypes.c_void_p), len(tensors), _hptr(seeds_t), _hptr(fit_t),
                                  _hptr(hs), _hptr(hf), hl, N, sigma, alpha, gamma, _dev_ptr(stats, "stats"),
                                  _stream(stream)), name)


def replay_residual(w, hist_seeds, hist_fit, N, sigma, alpha, gamma, residual, stream=None, antithetic=False):
    """residual: device float32 [out,in] (written)."""
    hs, hf, hl = _hist(hist_seeds, hist_fit, N, antithetic)
    d = w.desc()
    fn = _load().qes_replay_residual_antithetic if antithetic else _load().qes_replay_residual
    _check(fn(ctypes.byref(d), _hptr(hs), _hptr(hf), hl, N, sigma, alpha, gamma, _dev_ptr(residual, "residual"),
              _stream(stream)), "qes_replay_residual_antithetic" if antithetic else "qes_replay_residual")


def update_full_residual(w, seeds_t, fit_t, sigma, alpha, gamma, e_state, stats=None, stream=None, half=False):
    """One Alg. 1 step in place on w.qweight and e_state (device [out,in]: float32, or float16 with half=True)."""
    seeds_t = _host(seeds_t, np.uint64)
    fit_t = _host(fit_t, np.float32)
    N = int(fit_t.size)
    if seeds_t.size != N:
        raise ValueError("seeds_t and fit_t differ in length")
    d = w.desc()
    name = "qes_update_full_residual_f16" if half else "qes_update_full_residual"
    _check(getattr(_load(), name)(ctypes.byref(d), _hptr(seeds_t), _hptr(fit_t), N, sigma, alpha, gamma,
                                  _dev_ptr(e_state, "e_state"), _dev_ptr(stats, "stats"), _stream(stream)), name)


def update_stochastic_rounding(w, seeds_t, fit_t, sigma, alpha, round_seed, stats=None, stream=None):
    """One stateless step with stochastic rounding of the update (baseline), in place on w.qweight."""
    seeds_t = _host(seeds_t, np.uint64)
    fit_t = _host(fit_t, np.float32)
    N = int(fit_t.size)
    if seeds_t.size != N:
        raise ValueError("seeds_t and fit_t differ in length")
    d = w.desc()
    _check(_load().qes_update_stochastic_rounding(ctypes.byref(d), _hptr(seeds_t), _hptr(fit_t), N, sigma, alpha,
                                                  int(round_seed), _dev_ptr(stats, "stats"), _stream(stream)),
           "qes_update_stochastic_rounding")


def normalize_fitness(reward):
    reward = _host(reward, np.float32)
    fit = np.empty_like(reward)
    _check(_load().qes_normalize_fitness(_hptr(reward), int(reward.size), _hptr(fit)), "qes_normalize_fitness")
    return fit


def bench_noise(mode, n_threads, iters, sigma, sink, stream=None):
    _check(_load().qes_bench_noise(mode, n_threads, iters, sigma, _dev_ptr(sink, "sink"), _stream(stream)),
           "qes_bench_noise")


def bench_mfma(mode, n_blocks, iters, sink, stream=None):
    _check(_load().qes_bench_mfma(mode, n_blocks, iters, _dev_ptr(sink, "sink"), _stream(stream)), "qes_bench_mfma")


def bench_copy(src, dst, n_bytes, stream=None):
    _check(_load().qes_bench_copy(_dev_ptr(src, "src"), _dev_ptr(dst, "dst"), n_bytes, _stream(stream)),
           "qes_bench_copy")
