"""Helpers for the GPU parity tests: device tensors in the library's layouts."""
import ctypes as C

import numpy as np
import torch

from paper_2406_06911_amd import binding as B

DEV = "cuda:0"


def tdtype(dtype):
    return torch.bfloat16 if dtype == B.AD_BF16 else torch.float32


def quantize(a, dtype):
    """Round a float array to the values the storage dtype can hold (so both sides see the same input)."""
    a = np.asarray(a, np.float32)
    if dtype == B.AD_BF16:
        return torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    return a


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV).to(tdtype(dtype)).contiguous()


def dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV)


def dev_bytes(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def nchw_to_nhwc(a):
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))


def nhwc_to_nchw(a):
    return np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2)))


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def p(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def stream_ptr(s=None):
    s = s or torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


TOL = {B.AD_F32: 1e-4, B.AD_BF16: 2e-2}      # per-component budget (whole unit ranges)
KTOL = {B.AD_F32: 2e-5, B.AD_BF16: 5e-3}     # one kernel: a single rounding of the result to the storage type
ULP = {B.AD_F32: 1e-5, B.AD_BF16: 2.0 ** -8}


def assert_kernel_close(got, ref, dtype, c=2.0, rel=None):
    """Single-kernel bar: relative L2 within KTOL and, element by element, |got - ref| <= c * ulp * (|ref| + rms(ref)).
    One rounding to bf16 is at most 2^-9 |ref|; the rms term covers results that cancel to near zero.  A single
    wrong element (a pad column read as data, a lost tap) is off by about rms(ref), i.e. a hundred times the bound."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all()
    scale = float(np.sqrt(np.mean(ref * ref)))
    bound = c * ULP[dtype] * (np.abs(ref) + scale)
    excess = np.abs(got - ref) - bound
    worst = int(np.argmax(excess))
    assert excess.flat[worst] <= 0, (f"element {np.unravel_index(worst, ref.shape)}: got {got.flat[worst]!r} ref {ref.flat[worst]!r} "
                                      f"bound {bound.flat[worst]:.3e}")
    err = rel_l2(got, ref)
    assert err < (KTOL[dtype] if rel is None else rel), err
