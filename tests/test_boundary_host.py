"""C-ABI library: it loads, exports every declared symbol, and its integer host logic (unit list,
partition, schedule table, timesteps) is bit-exact against the oracle.  No GPU needed."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2406_06911_amd as ad
from paper_2406_06911_amd import binding as B
from configs import CONFIGS
from oracle import sampler as SM
from oracle import schedule as SC
from oracle.partition import component_ranges, partition, segment_ranges_wrapped, unit_flops
from oracle.unet import UNetConfig, build_units, component_io, weight_manifest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "asyncdiff.h")).read()
    declared = set(re.findall(r"\b(ad_[a-z_0-9]+)\s*\(", header))
    declared -= {"ad_component_io()", "ad_device_bytes()"}
    assert declared, "no declarations found"
    lib = ctypes.CDLL(B.lib_path)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in asyncdiff.h but not exported"
    assert declared == set(B.EXPORTS)


@pytest.mark.parametrize("name", ["tiny", "sd_512", "sd21_768", "sdxl_1024", "sd21_narrow", "video_16f", "video_narrow", "video_tiny"])
def test_units_flops_partition_manifest_match_oracle(name):
    d = CONFIGS[name]
    dtype = B.AD_F32 if name.endswith("tiny") else B.AD_BF16
    ocfg = UNetConfig(**d)
    ounits = build_units(ocfg)
    for n in (1, 2, 3, 4):
        m = ad.AsyncDiff(d, n, 1, 1, dtype)
        units = m.units()
        assert len(units) == len(ounits)
        for u, o in zip(units, ounits):
            assert (u.name.decode(), B.UNIT_KINDS[u.kind], u.c_in, u.c_skip, u.c_out, u.h_in, u.w_in, u.h_out, u.w_out,
                    u.depth, u.skip_from) == (o.name, o.kind, o.c_in, o.c_skip, o.c_out, o.h_in, o.w_in, o.h_out, o.w_out,
                                              o.depth, o.skip_from)
            assert u.flops == unit_flops(ocfg, o)
        assert m.partition() == component_ranges(ocfg, n)
        for k, (a, b) in enumerate(m.partition(), start=1):
            assert m.component_io(k) == tuple(component_io(ounits, a, b))
        assert m.weight_manifest() == [(nm, tuple(s)) for nm, s in weight_manifest(ocfg)]
        m.close()


@pytest.mark.parametrize("T,N,w,S,shift", [(10, 2, 1, 1, False), (50, 4, 3, 1, False), (50, 4, 3, 2, False), (25, 4, 2, 1, False),
                                           (13, 3, 2, 3, False), (50, 3, 2, 1, True), (7, 1, 0, 1, False), (9, 2, 12, 2, False),
                                           (11, 3, 1, 2, True)])
def test_schedule_and_timesteps_bit_exact(T, N, w, S, shift):
    m = ad.AsyncDiff(CONFIGS["tiny"], N, w, S, B.AD_F32)
    m.reset(T, time_shift=shift)
    assert m.timesteps() == SM.timesteps(T)
    rows = SC.build_schedule(T, N, w, S, shift)
    assert m.schedule() == [(r.round, r.comp, r.tau_step, r.read_slot, r.write_slot, r.latent_step, r.eps_step, r.fresh_from) for r in rows]
    m.close()


@pytest.mark.parametrize("sampler,beta", [(B.AD_DDIM, B.AD_BETA_LINEAR), (B.AD_EULER, B.AD_BETA_SCALED_LINEAR)])
def test_sampler_coefficients(sampler, beta):
    T = 50
    m = ad.AsyncDiff(CONFIGS["tiny"], 2, 1, 1, B.AD_F32)
    m.reset(T, sampler=sampler, beta=beta)
    taus = SM.timesteps(T)
    acp = SM.alphas_cumprod(kind="linear" if beta == B.AD_BETA_LINEAR else "scaled_linear")
    x, e = 0.7, -1.3
    for i in (0, 1, 17, 48, 49):
        cx, ce, in_scale, init_scale = m.sampler_coeffs(i)
        if sampler == B.AD_DDIM:
            ref = SM.ddim_step(np.array(x), np.array(e), i, taus, acp)
            assert in_scale == 1.0 and init_scale == 1.0
        else:
            ref = SM.euler_step(np.array(x), np.array(e), i, taus, acp)
            assert abs(in_scale - SM.euler_input_scale(i, taus, acp)) < 1e-14
            assert abs(init_scale - SM.euler_init_scale(taus, acp)) < 1e-12
        assert abs(cx * x + ce * e - float(ref)) < 1e-12
    m.close()


def test_balance_cuts_matches_oracle_partition_rule():
    """ad_balance_cuts on arbitrary costs (the use: measured unit times) is the oracle's minimax / lexicographic rule."""
    rng = np.random.default_rng(7)
    for trial in range(60):
        nu = int(rng.integers(1, 40))
        n = int(rng.integers(1, min(nu, 6) + 1))
        costs = [int(c) for c in rng.integers(0 if trial % 3 else 1, 1000 if trial % 2 else 5, size=nu)]
        assert ad.balance_cuts(costs, n) == partition(costs, n), (costs, n)
    with pytest.raises(ad.AsyncDiffError):
        ad.balance_cuts([1, 2, 3], 4)
    with pytest.raises(ad.AsyncDiffError):
        ad.balance_cuts([1, -2, 3], 2)


def test_explicit_cuts():
    d = CONFIGS["tiny"]
    ocfg = UNetConfig(**d)
    ounits = build_units(ocfg)
    nu = len(ounits)
    for cuts in ([1], [nu - 1], [2, 5], [1, 2, 3], list(range(1, nu))):
        m = ad.AsyncDiff(d, len(cuts) + 1, 1, 1, B.AD_F32, cuts=cuts)
        edges = [0] + cuts + [nu]
        assert m.partition() == [(edges[k], edges[k + 1] - 1) for k in range(len(cuts) + 1)]
        for k, (a, b) in enumerate(m.partition(), start=1):
            assert m.component_io(k) == tuple(component_io(ounits, a, b))
        m.close()
    for cuts in ([0], [nu], [3, 3], [5, 2]):
        with pytest.raises(ad.AsyncDiffError) as e:
            ad.AsyncDiff(d, len(cuts) + 1, 1, 1, B.AD_F32, cuts=cuts)
        assert e.value.status == B.AD_ERR_INVALID


@pytest.mark.parametrize("name", ["tiny", "sdxl_narrow", "sdxl_1024", "sd21_768"])
def test_wrapped_segmentation_matches_oracle(name):
    """Segments, per-segment inputs / outputs and the schedule table of the wrapped segmentation, entry by entry."""
    d = CONFIGS[name]
    dtype = B.AD_F32 if name == "tiny" else B.AD_BF16
    ocfg = UNetConfig(**d)
    ounits = build_units(ocfg)
    for n in (2, 3, 4):
        m = ad.AsyncDiff(d, n, 2, 1, dtype, wrap=True)
        segs = segment_ranges_wrapped(ocfg, n)
        assert m.partition() == segs and len(segs) == n + 1
        for k, (a, b) in enumerate(segs, start=1):
            assert m.component_io(k) == tuple(component_io(ounits, a, b))
        for shift in (False, True):
            m.reset(9, time_shift=shift)
            rows = SC.build_schedule(9, n, 2, 1, shift, wrap=True)
            assert m.schedule() == [(r.round, r.comp, r.tau_step, r.read_slot, r.write_slot, r.latent_step, r.eps_step, r.fresh_from)
                                    for r in rows]
        m.close()
    cuts = [2, 5, len(ounits) - 2]
    m = ad.AsyncDiff(d, 3, 1, 1, dtype, wrap=True, cuts=cuts)
    assert m.partition() == segment_ranges_wrapped(ocfg, 3, cuts)
    m.close()
    for bad in ([0, 3, 5], [3, 3, 5], [2, 5, len(ounits)]):
        with pytest.raises(ad.AsyncDiffError):
            ad.AsyncDiff(d, 3, 1, 1, dtype, wrap=True, cuts=bad)
    with pytest.raises(ad.AsyncDiffError):
        ad.AsyncDiff(d, 1, 1, 1, dtype, wrap=True)


def test_invalid_arguments_are_reported():
    bad = [
        (dict(CONFIGS["tiny"]), 0, 1, 1), (dict(CONFIGS["tiny"]), 2, 0, 1), (dict(CONFIGS["tiny"]), 2, 1, 0),
        (dict(CONFIGS["tiny"]), 2, -1, 1), (dict(CONFIGS["tiny"]), 99, 1, 1),
        (dict(CONFIGS["tiny"], channels=[30, 64]), 1, 1, 1), (dict(CONFIGS["tiny"], height=15), 1, 1, 1),
        (dict(CONFIGS["tiny"], head_dim=24), 1, 1, 1), (dict(CONFIGS["tiny"], gn_groups=7), 1, 1, 1),
    ]
    for d, n, w, s in bad:
        with pytest.raises(ad.AsyncDiffError) as e:
            ad.AsyncDiff(d, n, w, s, B.AD_F32)
        assert e.value.status == B.AD_ERR_INVALID and len(str(e.value)) > 20
    m = ad.AsyncDiff(CONFIGS["tiny"], 1, 0, 1, B.AD_F32)          # N = 1 needs no warm-up
    with pytest.raises(ad.AsyncDiffError) as e:
        m.timesteps() if hasattr(m, "T") else B.check(B.lib.ad_get_timesteps(m._h, (ctypes.c_int * 4)(), 4))
    assert e.value.status == B.AD_ERR_STATE
    with pytest.raises(ad.AsyncDiffError):
        m.reset(0)
    with pytest.raises(ad.AsyncDiffError):
        m.reset(2000)
    m.close()
    B.lib.ad_destroy(None)


def test_weight_packing_layout():
    rng = np.random.default_rng(0)
    w = rng.standard_normal((5, 32, 3, 3)).astype(np.float32)
    p = B.pack_conv_weight(B.AD_F32, w).view(np.float32).reshape(128, 9 * 32)
    for o, c, u, v in [(0, 0, 0, 0), (4, 31, 2, 1), (2, 7, 1, 2)]:
        assert p[o, (u * 3 + v) * 32 + c] == w[o, c, u, v]
    assert not p[5:].any()
    # bf16 packing rounds to nearest even
    pb = B.pack_conv_weight(B.AD_BF16, w[:, :, 0, 0].repeat(2, axis=1)).view(np.uint16).reshape(128, 64)
    import synthetic_inputs as SI
    ref = (SI.round_to_bf16(w[:, :, 0, 0].repeat(2, axis=1)).view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(pb[:5], ref)
    # GEGLU packing interleaves 32 value rows with 32 gate rows
    g = rng.standard_normal((128, 32)).astype(np.float32)
    pg = B.pack_conv_weight(B.AD_F32, g, geglu=True).view(np.float32).reshape(128, 32)
    assert np.array_equal(pg[0:32], g[0:32]) and np.array_equal(pg[32:64], g[64:96])
    assert np.array_equal(pg[64:96], g[32:64]) and np.array_equal(pg[96:128], g[96:128])


def test_video_configuration_shapes_and_checks():
    d = CONFIGS["video_16f"]
    m = ad.AsyncDiff(d, 4, 2, 1, B.AD_BF16)
    nu = len(m.units())
    assert m.tensor_shape(-1)[0] == (16, 64, 64, 4) and m.tensor_shape(-1)[1] == 16 * 4 * 64 * 64 * 4      # one latent per frame
    assert m.tensor_shape(nu - 1)[0] == (16, 64, 64, 4)
    m.close()
    for bad in (dict(d, batch=2), dict(d, frames=17, batch=17), dict(d, frames=0), dict(d, temporal_heads=7),
                dict(d, pooled_dim=1280)):
        with pytest.raises(B.AsyncDiffError):
            ad.AsyncDiff(bad, 4, 2, 1, B.AD_BF16)


def test_kernel_entry_points_reject_bad_shapes_before_touching_the_gpu():
    """Shape checks sit on the host, in front of every launch: a bad call comes back with AD_ERR_INVALID."""
    import ctypes as C
    L = B.lib
    fake = C.c_void_p(256)                     # never dereferenced: every call below fails validation first
    none = C.c_void_p(0)
    bad = [
        L.ad_attention_frames_forward(B.AD_BF16, none, fake, fake, 16, 64, 320, 8, 320, 320, 320, 320, fake, none),   # null q
        L.ad_attention_frames_forward(B.AD_BF16, fake, fake, fake, 17, 64, 320, 8, 320, 320, 320, 320, fake, none),   # too many frames
        L.ad_attention_frames_forward(B.AD_BF16, fake, fake, fake, 16, 64, 320, 7, 320, 320, 320, 320, fake, none),   # heads do not divide c
        L.ad_attention_frames_forward(B.AD_BF16, fake, fake, fake, 16, 64, 320, 8, 319, 320, 320, 320, fake, none),   # leading dimension < c
        L.ad_attention_frames_forward(7, fake, fake, fake, 16, 64, 320, 8, 320, 320, 320, 320, fake, none),           # dtype
        L.ad_attention_forward(B.AD_BF16, fake, fake, fake, 1, 2, 128, 128, 320, 64, 320, 320, 100, 320, fake, none),  # V^T rows shorter than the keys
        L.ad_attention_forward(B.AD_BF16, fake, fake, fake, 0, 2, 128, 128, 320, 256, 320, 320, 320, 320, fake, none),  # head_dim > 128
    ]
    assert all(st == B.AD_ERR_INVALID for st in bad), bad
    assert b"frame attention" in L.ad_last_error() or b"attention" in L.ad_last_error()
