"""Helpers for the GPU parity tests: move the seeded numpy inputs to device memory and back."""
import numpy as np
import torch

import paper_2602_03120_amd as qes
import workloads as wl

DEV = "cuda:0"


def to_dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(DEV)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def from_dev(t, dtype):
    return t.cpu().numpy().view(dtype)


def device_tensor(ot):
    """oracle.Tensor (host) -> qes.Tensor (device copy of the same bits)."""
    qw = to_dev(ot.qweight)
    sc = None if ot.scales is None else to_dev(ot.scales)
    return qes.Tensor(qw, sc, ot.out_features, ot.in_features, ot.bits, ot.group_size, ot.qmin, ot.qmax,
                      ot.tensor_id)


def bf16_close(y_bits, ref_bits, rtol=1e-2):
    """|y - ref| <= rtol*|ref| + rtol*rms(ref over the member); y, ref uint16 bf16 [N,T,out]."""
    y = wl.bf16_bits_to_f32(y_bits).astype(np.float64)
    r = wl.bf16_bits_to_f32(ref_bits).astype(np.float64)
    rms = np.sqrt((r ** 2).mean(axis=(1, 2), keepdims=True))
    err = np.abs(y - r)
    bound = rtol * np.abs(r) + rtol * rms
    return bool((err <= bound).all()), float((err / (bound + 1e-30)).max())
