"""Kernel-level parity: every HIP kernel against the oracle's plain definition, through the C ABI."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

import synthetic_inputs as SI
from gpu_util import (DEV, KTOL, TOL, assert_kernel_close, dev, dev_bytes, dev_f32, host, nchw_to_nhwc, nhwc_to_nchw, p, quantize, rel_l2, stream_ptr, tdtype)
from oracle import primitives as P
from oracle import sampler as SM
from paper_2406_06911_amd import binding as B

pytestmark = pytest.mark.gpu
lib = B.lib
DT = [B.AD_F32, B.AD_BF16]


def sync():
    torch.cuda.synchronize()


# ---------------------------------------------------------------------------------------------------
def run_conv(dtype, x0, x1, w, bias, stride=1, up=0, rowvec=None, residual=None, mode=B.OUT_ROWMAJOR, geglu=False, splitk=False):
    """x0/x1 NCHW float arrays (already quantised); returns the device result as float64 array."""
    n, c0, hs, ws = x0.shape
    c1 = x1.shape[1] if x1 is not None else 0
    k = w.shape[2]
    n_out = w.shape[0]
    d0 = dev(nchw_to_nhwc(x0), dtype)
    d1 = dev(nchw_to_nhwc(x1), dtype) if x1 is not None else None
    wp = dev_bytes(B.pack_conv_weight(dtype, w, geglu))
    nb = (n_out + 127) // 128 * 128
    bpad = np.zeros(nb, np.float32)
    if bias is not None:
        bb = np.asarray(bias, np.float32)
        if geglu:
            half = n_out // 2
            idx = [(r // 64) * 32 + r % 64 if r % 64 < 32 else half + (r // 64) * 32 + r % 64 - 32 for r in range(n_out)]
            bb = bb[idx]
        bpad[:n_out] = bb
    db = dev_f32(bpad) if bias is not None else None
    hin, win = hs << up, ws << up
    pad = k // 2
    ho, wo = (hin + 2 * pad - k) // stride + 1, (win + 2 * pad - k) // stride + 1
    drow = dev_f32(rowvec) if rowvec is not None else None
    dres = dev(residual, dtype) if residual is not None else None
    if mode == B.OUT_ROWMAJOR:
        out = torch.full((n, ho, wo, n_out), float("nan"), device=DEV, dtype=tdtype(dtype))
        ld_t = 0
    elif mode == B.OUT_GEGLU:
        out = torch.full((n, ho, wo, n_out // 2), float("nan"), device=DEV, dtype=tdtype(dtype))
        ld_t = 0
    else:
        ld_t = (ho * wo + 63) // 64 * 64
        out = torch.full((n, n_out, ld_t), float("nan"), device=DEV, dtype=tdtype(dtype) if mode == B.OUT_TRANSPOSED else torch.float32)
    ws_bytes = lib.ad_conv_workspace_bytes(dtype, n, ho, wo, n_out, c0 + c1, k, mode) if splitk else 0
    wsb = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=DEV)
    B.check(lib.ad_conv_forward(dtype, p(d0), p(d1), c0, c1, n, hs, ws, up, k, stride, p(wp), n_out, p(db), p(drow), p(dres),
                                p(out), None, None, mode, ld_t, p(wsb) if ws_bytes else None, ws_bytes, stream_ptr()))
    run_conv.last_ws_bytes = ws_bytes
    sync()
    return host(out), (ho, wo)


CONV_CASES = [
    # name, batch, c0, c1, hs, ws, n_out, k, stride, up
    ("3x3_multi_tile_ragged", 2, 64, 0, 13, 11, 192, 3, 1, 0),
    ("3x3_stride2", 2, 64, 0, 12, 10, 64, 3, 2, 0),
    ("3x3_upsampled", 1, 64, 0, 7, 9, 128, 3, 1, 1),
    ("3x3_concat", 2, 64, 128, 9, 9, 64, 3, 1, 0),
    ("1x1_concat", 2, 128, 64, 10, 9, 320, 1, 1, 0),
    ("3x3_small_n", 2, 64, 0, 8, 8, 4, 3, 1, 0),
    ("3x3_big_tiles", 2, 64, 0, 96, 96, 320, 3, 1, 0),
]


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("case", CONV_CASES, ids=[c[0] for c in CONV_CASES])
def test_conv_matches_direct_summation(dtype, case):
    name, n, c0, c1, hs, ws, n_out, k, stride, up = case
    x0 = quantize(SI.make_array((n, c0, hs, ws), 11), dtype)
    x1 = quantize(SI.make_array((n, c1, hs, ws), 12), dtype) if c1 else None
    w = quantize(SI.make_array((n_out, c0 + c1, k, k), 13, 0.05), dtype)
    bias = SI.make_array((n_out,), 14, 0.1)
    got, (ho, wo) = run_conv(dtype, x0, x1, w, bias, stride, up)
    xin = x0 if x1 is None else np.concatenate([x0, x1], 1)
    if up:
        xin = P.upsample_nearest2x(xin)
    if name == "3x3_big_tiles":
        # full size of the first level of the 768px model: compare sampled outputs computed one by one
        rng = np.random.default_rng(5)
        xp = np.pad(xin.astype(np.float64), ((0, 0), (0, 0), (1, 1), (1, 1)))
        errs, refs = [], []
        for _ in range(400):
            b, o, i, j = int(rng.integers(n)), int(rng.integers(n_out)), int(rng.integers(ho)), int(rng.integers(wo))
            ref = bias[o] + float(np.sum(w[o].astype(np.float64) * xp[b, :, i:i + 3, j:j + 3]))
            errs.append(got[b, i, j, o] - ref); refs.append(ref)
        assert_kernel_close(np.asarray(refs) + np.asarray(errs), np.asarray(refs), dtype)
        assert np.isfinite(got).all()
        return
    ref = P.conv2d(xin, w, bias, stride=stride)
    assert got.shape == (n, ho, wo, n_out)
    assert_kernel_close(nhwc_to_nchw(got), ref, dtype)


@pytest.mark.parametrize("dtype", DT)
def test_conv_epilogues(dtype):
    n, c, h, wd, n_out = 2, 64, 9, 7, 192
    x = quantize(SI.make_array((n, c, h, wd), 21), dtype)
    w = quantize(SI.make_array((n_out, c, 3, 3), 22, 0.05), dtype)
    bias = SI.make_array((n_out,), 23, 0.1)
    rowvec = SI.make_array((n, n_out), 24)
    res = quantize(SI.make_array((n, h, wd, n_out), 25), dtype)
    got, _ = run_conv(dtype, x, None, w, bias, rowvec=rowvec, residual=res)
    ref = P.conv2d(x, w, bias) + rowvec[:, :, None, None] + nhwc_to_nchw(res)
    assert_kernel_close(nhwc_to_nchw(got), ref, dtype)
    # transposed outputs (storage dtype and fp32)
    for mode in (B.OUT_TRANSPOSED, B.OUT_TRANSPOSED_F32):
        got, (ho, wo) = run_conv(dtype, x, None, w, bias, mode=mode)
        ref = P.conv2d(x, w, bias).reshape(n, n_out, ho * wo)
        assert_kernel_close(got[:, :, :ho * wo], ref, dtype)


@pytest.fixture(params=[1, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12], ids=["reg128", "reg64", "dma2_128", "dma3_128", "dma3_256", "dma3_64", "halo_128", "halo_256", "dma3_256_w4", "dma3_128_w4", "dma3_256_w16"])
def force_big_tiles(request):
    """Forces one GEMM kernel family on every shape (the LDS-DMA ones apply to bf16 only; fp32 keeps the automatic choice)."""
    B.check(lib.ad_tune_conv_tile(request.param))
    yield
    B.check(lib.ad_tune_conv_tile(-1))


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("case", CONV_CASES[:5], ids=[c[0] for c in CONV_CASES[:5]])
def test_conv_big_tile_kernels(dtype, case, force_big_tiles):
    test_conv_matches_direct_summation(dtype, case)
    test_conv_epilogues(dtype)
    test_linear_and_geglu(dtype)
    test_conv_split_k(dtype)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("big", [0, 1, 4, 5, 6, 7, 10, 11, 12])
@pytest.mark.parametrize("vt", [False, True])
def test_fused_qkv_projection(dtype, big, vt):
    """One GEMM for q, k, v: thirds of the output columns go to three tensors, the last optionally transposed."""
    bsz, l, c = 2, 72, 64
    if big:
        B.check(lib.ad_tune_conv_tile(big))
    try:
        x = quantize(SI.make_array((bsz * l, c), 35), dtype)
        w = quantize(SI.make_array((3 * c, c), 36, 0.2), dtype)
        dx = dev(x, dtype)
        wp = dev_bytes(B.pack_conv_weight(dtype, w))
        ld_t = 128 if vt else 0
        q = torch.full((bsz * l, c), float("nan"), device=DEV, dtype=tdtype(dtype))
        k = torch.full((bsz * l, c), float("nan"), device=DEV, dtype=tdtype(dtype))
        v = torch.full((bsz, c, ld_t) if vt else (bsz * l, c), float("nan"), device=DEV, dtype=tdtype(dtype))
        B.check(lib.ad_conv_forward(dtype, p(dx), None, c, 0, bsz, l, 1, 0, 1, 1, p(wp), 3 * c, None, None, None, p(q), p(k), p(v),
                                    B.OUT_QKV, ld_t, None, 0, stream_ptr()))
        sync()
    finally:
        B.check(lib.ad_tune_conv_tile(-1))
    ref = P.linear(x, w)
    assert_kernel_close(host(q), ref[:, :c], dtype)
    assert_kernel_close(host(k), ref[:, c:2 * c], dtype)
    if vt:
        got = host(v)[:, :, :l]
        assert_kernel_close(got, ref[:, 2 * c:].reshape(bsz, l, c).transpose(0, 2, 1), dtype)
    else:
        assert_kernel_close(host(v), ref[:, 2 * c:], dtype)


@pytest.mark.parametrize("dtype", DT)
def test_conv_split_k(dtype):
    """Deep-level shapes (few output positions, long K) take the split-K path when scratch is supplied."""
    n, c, h, wd, n_out = 2, 640, 6, 6, 192
    x = quantize(SI.make_array((n, c, h, wd), 26), dtype)
    w = quantize(SI.make_array((n_out, c, 3, 3), 27, 0.02), dtype)
    bias = SI.make_array((n_out,), 28, 0.1)
    rowvec = SI.make_array((n, n_out), 29)
    res = quantize(SI.make_array((n, h, wd, n_out), 30), dtype)
    ref = P.conv2d(x, w, bias) + rowvec[:, :, None, None] + nhwc_to_nchw(res)
    got, _ = run_conv(dtype, x, None, w, bias, rowvec=rowvec, residual=res, splitk=True)
    assert run_conv.last_ws_bytes > 0, "shape was expected to split"
    assert_kernel_close(nhwc_to_nchw(got), ref, dtype)
    plain, _ = run_conv(dtype, x, None, w, bias, rowvec=rowvec, residual=res, splitk=False)
    assert_kernel_close(nhwc_to_nchw(plain), ref, dtype)
    got, (ho, wo) = run_conv(dtype, x, None, w, bias, mode=B.OUT_TRANSPOSED_F32, splitk=True)
    assert_kernel_close(got[:, :, :ho * wo], P.conv2d(x, w, bias).reshape(n, n_out, ho * wo), dtype)


@pytest.mark.parametrize("dtype", DT)
def test_linear_and_geglu(dtype):
    rows, cin, cff = 200, 64, 256                      # GEGLU: 64 -> 2*256, value * gelu(gate)
    x = quantize(SI.make_array((1, cin, rows, 1), 31), dtype)
    w1 = quantize(SI.make_array((2 * cff, cin), 32, 0.2), dtype)
    b1 = SI.make_array((2 * cff,), 33, 0.1)
    got, _ = run_conv(dtype, x, None, w1[:, :, None, None], b1, mode=B.OUT_GEGLU, geglu=True)
    tok = x[0, :, :, 0].T
    hcat = P.linear(tok, w1, b1)
    ref = hcat[:, :cff] * P.gelu(hcat[:, cff:])
    assert_kernel_close(got.reshape(rows, cff), ref, dtype)
    w2 = quantize(SI.make_array((96, cin), 34, 0.2), dtype)
    got, _ = run_conv(dtype, x, None, w2[:, :, None, None], None)
    assert_kernel_close(got.reshape(rows, 96), P.linear(tok, w2), dtype)


# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("shape", [(2, 64, 0, 16, 16, 8, 1), (2, 320, 0, 24, 24, 32, 1), (1, 64, 32, 9, 7, 8, 0),
                                   (2, 640, 320, 12, 12, 32, 1), (2, 2560, 0, 6, 6, 32, 1)])
def test_groupnorm_silu(dtype, shape):
    n, c0, c1, h, w, groups, silu = shape
    x0 = quantize(SI.make_array((n, c0, h, w), 41) * 2 + 0.5, dtype)
    x1 = quantize(SI.make_array((n, c1, h, w), 42) - 1.0, dtype) if c1 else None
    gam, bet = 1 + SI.make_array((c0 + c1,), 43, 0.3), SI.make_array((c0 + c1,), 44, 0.3)
    d0 = dev(nchw_to_nhwc(x0), dtype)
    d1 = dev(nchw_to_nhwc(x1), dtype) if c1 else None
    out = torch.full((n, h, w, c0 + c1), float("nan"), device=DEV, dtype=tdtype(dtype))
    scratch = torch.zeros(lib.ad_groupnorm_scratch_bytes(n, h * w, c0 + c1), dtype=torch.uint8, device=DEV)
    dg, dbt = dev_f32(gam), dev_f32(bet)
    B.check(lib.ad_groupnorm_forward(dtype, p(d0), p(d1), c0, c1, n, h * w, groups, p(dg), p(dbt), 1e-5, silu, p(out), p(scratch), stream_ptr()))
    sync()
    xin = x0 if x1 is None else np.concatenate([x0, x1], 1)
    ref = P.group_norm(xin, groups, gam, bet, 1e-5)
    if silu:
        ref = P.silu(ref)
    assert_kernel_close(nhwc_to_nchw(host(out)), ref, dtype, rel=1e-5 if dtype == B.AD_F32 else 5e-3)


@pytest.mark.parametrize("dtype", DT)
@pytest.mark.parametrize("rows,c", [(7, 64), (300, 320), (33, 1280)])
def test_layernorm(dtype, rows, c):
    x = quantize(SI.make_array((rows, c), 51) * 3 + 1, dtype)
    gam, bet = 1 + SI.make_array((c,), 52, 0.3), SI.make_array((c,), 53, 0.3)
    dx, out = dev(x, dtype), torch.full((rows, c), float("nan"), device=DEV, dtype=tdtype(dtype))
    dg, dbt = dev_f32(gam), dev_f32(bet)
    B.check(lib.ad_layernorm_forward(dtype, p(dx), rows, c, p(dg), p(dbt), 1e-5, p(out), stream_ptr()))
    sync()
    assert_kernel_close(host(out), P.layer_norm(x, gam, bet, 1e-5), dtype, rel=1e-5 if dtype == B.AD_F32 else 5e-3)


# ---------------------------------------------------------------------------------------------------
LOG2E_F32 = np.float32(1.4426950408889634)


def mfma2_contract(q, d, variant, dtype, transposed, lk):
    """The second-generation MFMA attention kernels feed the matrix cores q * (log2(e) / sqrt(d)) rounded to bf16 (one
    more rounding than the first kernel, which scales the fp32 scores).  That operand rounding is part of the kernel's
    contract like the bf16 storage of q itself, so the oracle is given the same operand: returns the q (fp64) whose
    plain softmax(q k^T / sqrt(d)) equals 2^(q' k^T) for the rounded q'.  Other kernels: q unchanged."""
    second = variant in (1, 2, 3) or (variant == -1 and lk > 256)
    if not (second and dtype == B.AD_BF16 and d == 64 and transposed):
        return q
    c32 = np.float32(1.0) / np.sqrt(np.float32(d)) * LOG2E_F32
    qp = SI.round_to_bf16(q.astype(np.float32) * c32)
    return qp.astype(np.float64) * (math.log(2.0) * math.sqrt(d))


def run_attention(dtype, q, k, v, heads, transposed):
    bsz, l, c = q.shape
    lk = k.shape[1]
    d = c // heads
    dq, dk = dev(q, dtype), dev(k, dtype)
    if transposed:
        ldv = (lk + 63) // 64 * 64
        vt = np.full((bsz, c, ldv), np.nan, np.float32)          # the pad must never be read as data
        vt[:, :, :lk] = np.transpose(v, (0, 2, 1))
        dv = dev(vt, dtype)
    else:
        ldv = c
        dv = dev(v, dtype)
    out = torch.full((bsz, l, c), float("nan"), device=DEV, dtype=tdtype(dtype))
    B.check(lib.ad_attention_forward(dtype, p(dq), p(dk), p(dv), int(transposed), bsz, l, lk, c, d, c, c, ldv, c, p(out), stream_ptr()))
    sync()
    return host(out)


ATT_CASES = [
    # dtype, batch, l, lk, heads, d, transposed
    (B.AD_F32, 1, 64, 64, 4, 16, False), (B.AD_F32, 2, 37, 8, 2, 16, False), (B.AD_F32, 1, 70, 130, 1, 64, False),
    (B.AD_BF16, 2, 37, 77, 2, 16, False), (B.AD_BF16, 1, 20, 77, 1, 128, True),
    (B.AD_BF16, 2, 200, 200, 3, 64, True), (B.AD_BF16, 2, 144, 77, 2, 64, True), (B.AD_BF16, 1, 576, 576, 5, 64, True),
    (B.AD_BF16, 1, 130, 1, 1, 64, True),
]


@pytest.fixture(params=[-1, 0, 1, 2, 3], ids=["auto", "gen1", "gen2_q32", "gen2_q64", "gen2_pipelined"])
def attn_variant(request):
    """Forces one of the MFMA attention kernels (applies to bf16, head width 64, transposed v; other calls are unaffected)."""
    B.check(lib.ad_tune_attention(request.param))
    yield request.param
    B.check(lib.ad_tune_attention(-1))


ATT_CASES += [
    # several 256-query blocks with a ragged tail, several key tiles with a ragged tail
    (B.AD_BF16, 2, 600, 333, 2, 64, True), (B.AD_BF16, 1, 257, 64, 1, 64, True), (B.AD_BF16, 1, 31, 65, 2, 64, True),
    (B.AD_BF16, 1, 1024, 1024, 1, 64, True), (B.AD_BF16, 2, 96, 128, 1, 64, True),
]


@pytest.mark.parametrize("case", ATT_CASES, ids=[f"{'bf16' if c[0] else 'f32'}_l{c[2]}_lk{c[3]}_h{c[4]}_d{c[5]}_{'vt' if c[6] else 'v'}" for c in ATT_CASES])
def test_attention(case, attn_variant):
    dtype, bsz, l, lk, heads, d, tr = case
    if attn_variant >= 0 and not (dtype == B.AD_BF16 and d == 64 and tr):
        pytest.skip("the knob only selects among the bf16 MFMA kernels")
    c = heads * d
    q, k, v = (quantize(SI.make_array(s, sd), dtype) for s, sd in (((bsz, l, c), 61), ((bsz, lk, c), 62), ((bsz, lk, c), 63)))
    got = run_attention(dtype, q, k, v, heads, tr)
    q = mfma2_contract(q, d, attn_variant, dtype, tr, lk)
    # the probabilities are rounded to bf16 and the result is an average of v rows: its rms is well below that of the
    # v entries the errors are proportional to
    assert_kernel_close(got, P.attention(q, k, v, heads), dtype, c=4.0)


@pytest.mark.parametrize("dtype,tr", [(B.AD_F32, False), (B.AD_BF16, True)])
def test_attention_peaky_softmax(dtype, tr, attn_variant):
    """Scores far from uniform (scaled q, k) so that a mistake in the running max / rescaling shows."""
    bsz, l, lk, heads, d = 1, 96, 200, 2, 64
    c = heads * d
    q = quantize(SI.make_array((bsz, l, c), 71) * 3, dtype)
    k = quantize(SI.make_array((bsz, lk, c), 72) * 3, dtype)
    v = quantize(SI.make_array((bsz, lk, c), 73), dtype)
    # put the dominant key of some queries in the last tile so that the maximum moves late
    k[0, lk - 1] = q[0, 5] * 0.5
    got = run_attention(dtype, q, k, v, heads, tr)
    ref = P.attention(mfma2_contract(q, d, attn_variant, dtype, tr, lk), k, v, heads)
    assert_kernel_close(got, ref, dtype, c=4.0)
    pmax = P.softmax_rows(q[0, :, :d] @ k[0, :, :d].T / math.sqrt(d)).max(axis=1)
    assert np.median(pmax) > 0.5


@pytest.mark.parametrize("lk", [640, 700])
def test_attention_rising_and_falling_maximum(lk, attn_variant):
    """Scores that keep growing from key tile to key tile (the reference maximum has to move again and again, by
    more and by less than the slack the lazy maximum allows), then collapse far below it; one query row is all zeros."""
    dtype, l, d = B.AD_BF16, 300, 64
    rng = np.random.default_rng(77)
    base = rng.standard_normal((l, d)).astype(np.float32)
    q = quantize(base[None] * 2.0, dtype)
    q[0, 7] = 0.0
    k = rng.standard_normal((1, lk, d)).astype(np.float32) * 0.3
    ramp = np.concatenate([np.linspace(0.0, 3.0, lk // 2), np.linspace(3.0, -3.0, lk - lk // 2)]).astype(np.float32)
    k[0] += ramp[:, None] * np.sign(base[rng.integers(0, l, lk)])          # every key lines up with some query, more and more
    k = quantize(k, dtype)
    v = quantize(SI.make_array((1, lk, d), 75), dtype)
    got = run_attention(dtype, q, k, v, 1, True)
    ref = P.attention(mfma2_contract(q, d, attn_variant, dtype, True, lk), k, v, 1)
    assert_kernel_close(got, ref, dtype, c=4.0)
    sc = q[0] @ k[0].T / math.sqrt(d) * math.log2(math.e)
    tile_max = np.stack([sc[:, t:t + 32].max(axis=1) for t in range(0, lk, 32)], 1)
    run_max = np.maximum.accumulate(tile_max, axis=1)
    jumps = np.diff(run_max, axis=1)
    assert (jumps > 8).any() and ((jumps > 0) & (jumps < 8)).any()          # both kinds of moves occur


# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("batch", [1, 2])
def test_sampler_update(batch):
    T, n = 50, 4 * 24 * 24
    taus, acp = SM.timesteps(T), SM.alphas_cumprod()
    x = SI.make_array((n,), 81)
    eps = SI.make_array((batch, n), 82)
    for i, sampler in [(0, B.AD_DDIM), (17, B.AD_DDIM), (49, B.AD_DDIM), (3, B.AD_EULER)]:
        e = SM.cfg_combine(eps.astype(np.float64), 7.5)
        if sampler == B.AD_DDIM:
            ref = SM.ddim_step(x, e, i, taus, acp)
            a, a2 = acp[taus[i]], (acp[taus[i + 1]] if i + 1 < T else 1.0)
            cx, ce = math.sqrt(a2 / a), math.sqrt(1 - a2) - math.sqrt(a2) * math.sqrt(1 - a) / math.sqrt(a)
        else:
            ref = SM.euler_step(x, e, i, taus, acp)
            cx, ce = 1.0, SM.sigma(i + 1, taus, acp) - SM.sigma(i, taus, acp)
        dx, de = dev_f32(x), dev_f32(eps)
        B.check(lib.ad_sampler_update_raw(p(dx), p(de), n, batch, cx, ce, 7.5, stream_ptr()))
        sync()
        assert rel_l2(host(dx), ref) < 1e-6


@pytest.mark.parametrize("dtype", [B.AD_F32, B.AD_BF16])
@pytest.mark.parametrize("frames,positions,c,heads", [(16, 37, 320, 8), (3, 64, 64, 4), (16, 5, 1280, 8), (1, 9, 64, 8), (7, 130, 96, 2), (16, 33, 640, 8),
                                                      (5, 21, 60, 4), (13, 4097, 64, 1)])
def test_attention_over_frames(dtype, frames, positions, c, heads):
    """Temporal layer kernel: the sequences are the frames of each spatial position (row = frame * positions + p)."""
    rows = frames * positions
    ld = c + 8                                               # padded leading dimension
    q, k, v = (quantize(SI.make_array((rows, ld), 700 + i), dtype) for i in range(3))
    out = torch.full((rows, ld), float("nan"), device=DEV, dtype=tdtype(dtype))
    dq, dk, dv = dev(q, dtype), dev(k, dtype), dev(v, dtype)
    B.check(B.lib.ad_attention_frames_forward(dtype, p(dq), p(dk), p(dv), frames, positions, c, heads,
                                              ld, ld, ld, ld, p(out), stream_ptr()))
    torch.cuda.synchronize()
    seq = lambda a: a[:, :c].reshape(frames, positions, c).transpose(1, 0, 2)        # [positions][frames][c]
    ref = P.attention(seq(q), seq(k), seq(v), heads).transpose(1, 0, 2).reshape(rows, c)
    got = host(out)
    assert np.isnan(got[:, c:]).all()                        # nothing written past the row
    assert_kernel_close(got[:, :c], ref, dtype)
