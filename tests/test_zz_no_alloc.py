"""The allocation-free GroupNorm entry point against the one that takes a caller scratch buffer."""
import numpy as np
import pytest
import torch

import synthetic_inputs as SI
from gpu_util import DEV, dev, dev_f32, host, nchw_to_nhwc, nhwc_to_nchw, p, quantize, stream_ptr, tdtype, assert_kernel_close
from oracle import primitives as P
from paper_2406_06911_amd import binding as B

pytestmark = pytest.mark.gpu
lib = B.lib


def _both(dtype, n, c0, c1, h, w, groups, silu, seed):
    x0 = quantize(SI.make_array((n, c0, h, w), seed) * 2 + 0.5, dtype)
    x1 = quantize(SI.make_array((n, c1, h, w), seed + 1) - 1.0, dtype) if c1 else None
    gam, bet = 1 + SI.make_array((c0 + c1,), seed + 2, 0.3), SI.make_array((c0 + c1,), seed + 3, 0.3)
    d0 = dev(nchw_to_nhwc(x0), dtype)
    d1 = dev(nchw_to_nhwc(x1), dtype) if c1 else None
    dg, dbt = dev_f32(gam), dev_f32(bet)
    out_a = torch.full((n, h, w, c0 + c1), float("nan"), device=DEV, dtype=tdtype(dtype))
    out_b = torch.full((n, h, w, c0 + c1), float("nan"), device=DEV, dtype=tdtype(dtype))
    scratch = torch.zeros(lib.ad_groupnorm_scratch_bytes(n, h * w, c0 + c1), dtype=torch.uint8, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]
    B.check(lib.ad_groupnorm_forward_static(dtype, p(d0), p(d1), c0, c1, n, h * w, groups, p(dg), p(dbt), 1e-5, silu, p(out_b), stream_ptr()))
    assert torch.cuda.memory_stats(DEV)["allocation.all.allocated"] == before        # nothing went through torch's allocator
    B.check(lib.ad_groupnorm_forward(dtype, p(d0), p(d1), c0, c1, n, h * w, groups, p(dg), p(dbt), 1e-5, silu, p(out_a), p(scratch), stream_ptr()))
    torch.cuda.synchronize()
    xin = x0 if x1 is None else np.concatenate([x0, x1], 1)
    ref = P.group_norm(xin, groups, gam, bet, 1e-5)
    if silu:
        ref = P.silu(ref)
    return host(out_a), host(out_b), ref


@pytest.mark.parametrize("dtype", [B.AD_F32, B.AD_BF16])
def test_static_scratch_groupnorm_two_calls_in_a_row(dtype):
    # both shapes take the two-pass path (partial sums in scratch); the second is smaller and has two sources,
    # so it reuses a part of the array that still holds the first call's sums
    for shape in [(2, 320, 0, 48, 48, 32, 1, 900), (1, 64, 32, 20, 20, 8, 0, 910)]:
        n, c0, c1, h, w, groups, silu, seed = shape
        a, b, ref = _both(dtype, n, c0, c1, h, w, groups, silu, seed)
        np.testing.assert_array_equal(a, b)                     # same kernels, same summation order: bit for bit
        assert_kernel_close(nhwc_to_nchw(b), ref, dtype, rel=1e-5 if dtype == B.AD_F32 else 5e-3)


def test_static_scratch_rejects_oversize():
    dtype, n, c, hw, groups = B.AD_F32, 16, 2048, 64 * 64, 256          # 2 * 16 * 64 * 256 * 8 bytes = 4 MiB > 512 KiB
    x = torch.zeros(64, device=DEV)          # rejected on the host before anything is launched: never read
    g = torch.ones(64, device=DEV)
    st = lib.ad_groupnorm_forward_static(dtype, p(x), None, c, 0, n, hw, groups, p(g), p(g), 1e-5, 0, p(x), stream_ptr())
    assert st == B.AD_ERR_NOMEM
    assert b"fixed buffer" in lib.ad_last_error()
