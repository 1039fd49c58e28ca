"""Parity of the branch convolution (F x F as F*F shifted binary 1x1 branches
with per-branch real scales; paper, Section 4.2.1, last paragraph) and of the
bias-then-sign packing with the CPU oracle, on a real MI355X.

The library evaluates z in float32 as one fused multiply-add per branch in a
fixed order, exactly the chain the oracle's float result follows, so z is
compared for equality (and, as a sanity check, against the oracle's double
result within the chain's rounding bound); the fused bits and the packed words
are compared bit for bit.
"""
import functools

import numpy as np
import pytest
import torch

import oracle
from paper_2010_00704_amd import binding as B
from paper_2010_00704_amd import workloads as W
from gpu_helpers import (GUARD, Guarded, gpu_device, i32, oracle_bits_of_sign, oracle_pack_nchw,
                         oracle_pack_vectors, run_variant, up)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    return gpu_device()


def pack_nchw(x):
    return oracle_pack_nchw(x)


def pack_padv(padv):
    return oracle_pack_vectors(padv)


# ------------------------------------------------------------ bias, sign, pack
PACK_BIAS_SHAPES = [
    # outer, channels, inner   (every kernel family: rows, small inner, columns, 4-pixel columns, generic)
    (5, 70, 1), (3, 64, 49), (2, 100, 9), (2, 33, 300), (2, 64, 784), (1, 32, 4), (3, 96, 17), (2, 256, 1024),
    (33, 70, 1000),
]


@pytest.mark.parametrize("outer,channels,inner", PACK_BIAS_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "f16", "i8"])
def test_pack_bias(dev, outer, channels, inner, dtype):
    seed = 7000 + outer * 131 + channels * 7 + inner
    signs = W.pm1(seed, (outer, channels, inner))
    if dtype == "i8":
        mag = (W.raw_u64(seed + 1, 0, signs.size) % np.uint64(4)).astype(np.int8).reshape(signs.shape)
        x = (signs * mag).astype(np.int8)                      # -3 .. 3, zeros included
        bias = W.uniform_f32(seed + 2, (channels,), -3.0, 3.0, steps=12)   # halves: ties with integers
        xt, code = torch.from_numpy(x), B.BCNN_I8
        x_f32 = x.astype(np.float32)
    else:
        x = W.real_with_sign(seed, signs)
        bias = W.uniform_f32(seed + 2, (channels,), -1.5, 1.5)
        if dtype == "f16":
            x = oracle.store_f16(x)
            xt, code = torch.from_numpy(x), B.BCNN_F16
        else:
            xt, code = torch.from_numpy(x), B.BCNN_F32
        x_f32 = x.astype(np.float32)
        # exact cancellations and near misses in a few places
        flat = x_f32.reshape(outer, channels, inner)
        for k in range(min(channels, 6)):
            a, i = k % outer, (3 * k) % inner
            bias[k] = -flat[a, k, i]
    want = oracle.pack_channels(oracle.sign_bias_f32(x_f32.reshape(outer, channels, inner), bias))
    cw = (channels + 31) // 32
    out = Guarded(outer * inner * cw, dev)
    B.check(B.bcnn_pack_bias(xt.to(dev), code, outer, channels, inner, up(bias, dev), out.ptr), "pack_bias")
    got = out.get().reshape(outer, inner, cw)
    assert np.array_equal(got, want)


REPLICATED_SHAPES = [
    # outer, source channels, inner, replication   (every kernel family; ragged and word-aligned channel counts)
    (12, 48, 2800, 3),
    (5, 35, 1, 2), (3, 32, 49, 4), (2, 50, 9, 3), (2, 33, 300, 2), (2, 32, 784, 8), (1, 16, 4, 2), (3, 64, 1, 3),
    (2, 64, 1024, 2),
]


@pytest.mark.parametrize("outer,src_channels,inner,rep", REPLICATED_SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_pack_bias_replicated(dev, outer, src_channels, inner, rep, dtype):
    """Section 4.2.2: channels replicated by bookkeeping, one bias per replicated
    channel; the oracle makes the copy for real."""
    seed = 7500 + outer * 131 + src_channels * 7 + inner + rep
    x = W.real_with_sign(seed, W.pm1(seed, (outer, src_channels, inner)))
    if dtype == "f16":
        x = oracle.store_f16(x)
    channels = src_channels * rep
    bias = W.uniform_f32(seed + 2, (channels,), -1.5, 1.5)
    x32 = x.astype(np.float32)
    for k in range(min(channels, 6)):
        bias[channels - 1 - k] = -x32[k % outer, (channels - 1 - k) % src_channels, (5 * k) % inner]
    want = oracle.pack_channels(oracle.sign_bias_f32(oracle.replicate_channels(x32, rep), bias))
    cw = (channels + 31) // 32
    out = Guarded(outer * inner * cw, dev)
    B.check(B.bcnn_pack_bias_replicated(torch.from_numpy(x).to(dev), B.BCNN_F16 if dtype == "f16" else B.BCNN_F32,
                                        outer, src_channels, inner, rep, up(bias, dev), out.ptr), "pack_rep")
    assert np.array_equal(out.get().reshape(outer, inner, cw), want)


def test_pack_bias_rejects_missing_bias(dev):
    x = torch.zeros((1, 32, 4), dtype=torch.float32, device=dev)
    out = torch.zeros((4,), dtype=torch.int32, device=dev)
    assert B.bcnn_pack_bias(x, B.BCNN_F32, 1, 32, 4, None, out) == B.BCNN_ERR_INVALID_ARG


# ------------------------------------------------------------ branch convolution
def make_case(seed, n, c, h, w, o, k, shared, grid):
    p = k * k
    xb = W.pm1(seed, (1 if shared else p, n, c, h, w), 0.4)
    wt = W.pm1(seed + 1, (o, c, k, k))
    padv = W.pm1(seed + 2, (p, c))
    if grid:   # scales and biases on a grid of quarters: exact float sums, exact zeros of z occur
        g = W.uniform_f32(seed + 3, (p, o), -2.0, 2.0, steps=16)
        hb = W.uniform_f32(seed + 4, (o,), -8.0, 8.0, steps=64)
    else:
        g = W.uniform_f32(seed + 3, (p, o), -1.5, 1.5)
        hb = W.uniform_f32(seed + 4, (o,), -float(c), float(c))
    return xb, wt, padv, g, hb


VARIANTS = [B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU, B.BCNN_VARIANT_MFMA_FP4]
VARIANT_IDS = ["auto", "valu", "mfma_fp4"]


def gpu_branches(dev, xb, wt, padv_words, mode, g, hb, stride, pad, fused, variant=B.BCNN_VARIANT_AUTO):
    bcount, n, c, h, w = xb.shape
    o, k = wt.shape[0], (wt.shape[2] if wt.ndim == 4 else 1)
    p = g.shape[0]
    desc = B.conv_desc(n, c, h, w, o, k, stride, pad)
    ho, wo = B.out_shape(desc)
    cw = (c + 31) // 32
    xp = up(i32(np.stack([pack_nchw(xb[t]) for t in range(bcount)])), dev)
    wp = up(i32(oracle.pack_channels(wt.reshape(o, c, -1))), dev)
    stride_words = 0 if bcount == 1 else n * h * w * cw
    pw = up(i32(padv_words), dev) if padv_words is not None else None
    gt, ht = up(g, dev), (up(hb, dev) if hb is not None else None)
    if fused:
        cwo = (o + 31) // 32
        out = Guarded(n * ho * wo * cwo, dev)
        run_variant(B.bcnn_conv2d_binary_branches_sign_pack(desc, p, xp, stride_words, wp, pw, mode, gt, ht, out.ptr,
                                                            variant), "branches_sign_pack", variant)
        return out.get(np.uint32).reshape(n, ho * wo, cwo)
    out = Guarded(n * ho * wo * o, dev)
    run_variant(B.bcnn_conv2d_binary_branches(desc, p, xp, stride_words, wp, pw, mode, gt, ht, out.ptr, variant),
                "branches", variant)
    return out.get(np.float32).reshape(n, ho, wo, o)


def oracle_bits(z32):
    return oracle_bits_of_sign(oracle.sign_f32(z32))


BRANCH_SHAPES = [
    # n, c_in, h, w, c_out, k, stride, pad
    (1, 64, 14, 14, 64, 3, 1, 1),
    (2, 128, 9, 7, 96, 3, 1, 1),
    (3, 33, 6, 5, 7, 3, 1, 1),       # ragged channels both ways, scalar word loads
    (2, 100, 8, 8, 40, 3, 2, 1),
    (2, 64, 7, 7, 33, 3, 1, 0),      # no padding
    (1, 256, 20, 20, 64, 3, 2, 1),
    (4, 192, 5, 5, 130, 1, 1, 0),    # F = 1: one branch
    (1, 70, 17, 3, 31, 3, 2, 0),
    (40, 64, 14, 14, 64, 3, 1, 1),   # enough waves for two pixels per lane
    (2, 1, 4, 4, 1, 3, 1, 1),
    (6, 256, 14, 14, 128, 3, 1, 1),  # c_in a multiple of 256: the matrix-core kernel covers these
    (3, 512, 20, 19, 100, 3, 2, 1),
    (9, 256, 13, 11, 200, 3, 1, 0),
    (2, 768, 25, 25, 64, 3, 1, 1),
]
MODES = ["minus", "words", "zero"]


@pytest.mark.parametrize("shape", BRANCH_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("shared", [True, False], ids=["shared", "per_branch"])
@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
def test_branches_match_oracle(dev, shape, mode, shared, variant):
    n, c, h, w, o, k, stride, pad = shape
    seed = 8000 + sum(v * q for v, q in zip(shape, (3, 5, 7, 11, 13, 17, 19, 23))) + MODES.index(mode) + 2 * shared
    p = k * k
    for grid in (False, True):
        xb, wt, padv, g, hb = make_case(seed + 50 * grid, n, c, h, w, o, k, shared, grid)
        if mode == "minus":
            padv_o, words, code = -np.ones((p, c), dtype=np.int8), None, B.BCNN_PAD_WORDS
        elif mode == "words":
            padv_o, words, code = padv, pack_padv(padv), B.BCNN_PAD_WORDS
        else:
            padv_o, words, code = np.zeros((p, c), dtype=np.int8), pack_padv(padv), B.BCNN_PAD_ZERO
        z64, z32, yt = oracle.branches_pm1(xb, padv_o, wt, g, hb, stride, pad, taps=True)
        got = gpu_branches(dev, xb, wt, words, code, g, hb, stride, pad, fused=False, variant=variant)
        assert np.array_equal(got, z32)
        mag = np.abs(hb.astype(np.float64)) + (np.abs(g.astype(np.float64)).T[None, None, None] * np.abs(yt)).sum(-1)
        assert np.all(np.abs(got.astype(np.float64) - z64) <= p * 2.0**-24 * mag + 1e-30)
        bits = gpu_branches(dev, xb, wt, words, code, g, hb, stride, pad, fused=True, variant=variant)
        assert np.array_equal(bits, oracle_bits(z32))
        if grid:
            assert np.any(z32 == 0) or z32.size < 20000, "grid case should produce exact zeros of z"


PARALLEL_SHAPES = [
    # n, c_in, h, w, c_out, P, stride   (1x1 branches on the unshifted map: Figure 2, bottom)
    (2, 64, 14, 14, 64, 2, 1),
    (1, 100, 9, 9, 70, 3, 1),
    (3, 256, 7, 7, 96, 2, 2),
    (2, 32, 28, 28, 32, 4, 1),
    (1, 33, 5, 6, 5, 1, 1),
    (2, 256, 28, 28, 128, 2, 1),     # matrix-core kernel
    (5, 512, 15, 15, 70, 3, 2),
    (8, 256, 12, 12, 256, 5, 1),
]


@pytest.mark.parametrize("shape", PARALLEL_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("shared", [True, False], ids=["shared", "per_branch"])
@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
def test_parallel_branches_match_oracle(dev, shape, shared, variant):
    n, c, h, w, o, p, stride = shape
    seed = 8800 + sum(v * q for v, q in zip(shape, (3, 5, 7, 11, 13, 17, 19))) + shared
    for grid in (False, True):
        xb = W.pm1(seed + 50 * grid, (1 if shared else p, n, c, h, w), 0.45)
        wt = W.pm1(seed + 1, (o, c, p))
        if grid:
            g = W.uniform_f32(seed + 3, (p, o), -2.0, 2.0, steps=16)
            hb = W.uniform_f32(seed + 4, (o,), -8.0, 8.0, steps=64)
        else:
            g = W.uniform_f32(seed + 3, (p, o), -1.5, 1.5)
            hb = W.uniform_f32(seed + 4, (o,), -float(c), float(c))
        padv = -np.ones((p, c), dtype=np.int8)
        _, z32 = oracle.branches_pm1(xb, padv, wt, g, hb, stride, 0)
        got = gpu_branches(dev, xb, wt, None, B.BCNN_PAD_WORDS, g, hb, stride, 0, fused=False, variant=variant)
        assert np.array_equal(got, z32)
        bits = gpu_branches(dev, xb, wt, None, B.BCNN_PAD_WORDS, g, hb, stride, 0, fused=True, variant=variant)
        assert np.array_equal(bits, oracle_bits(z32))


def test_null_bias_is_zero_and_unit_scales_give_the_integer_convolution(dev):
    n, c, h, w, o, k = 2, 96, 10, 9, 64, 3
    xb = W.pm1(9100, (1, n, c, h, w))
    wt = W.pm1(9101, (o, c, k, k))
    g = np.ones((9, o), dtype=np.float32)
    got = gpu_branches(dev, xb, wt, None, B.BCNN_PAD_WORDS, g, None, 1, 1, fused=False)
    y = oracle.conv2d_pm1(xb[0], wt, 1, 1)
    assert np.array_equal(got, y.astype(np.float32))


def test_branch_argument_checks(dev):
    desc = B.conv_desc(1, 64, 8, 8, 32, 3, 1, 1)
    x = torch.zeros((64 * 2,), dtype=torch.int32, device=dev)
    w = torch.zeros((32 * 9 * 2,), dtype=torch.int32, device=dev)
    g = torch.zeros((9 * 32,), dtype=torch.float32, device=dev)
    z = torch.zeros((64 * 32,), dtype=torch.float32, device=dev)
    assert B.bcnn_conv2d_binary_branches(desc, 9, x, 0, w, None, 7, g, None, z) == B.BCNN_ERR_INVALID_ARG
    assert B.bcnn_conv2d_binary_branches(desc, 9, x, 5, w, None, 0, g, None, z) == B.BCNN_ERR_INVALID_ARG
    assert B.bcnn_conv2d_binary_branches(desc, 9, x, 0, w, None, 0, None, None, z) == B.BCNN_ERR_INVALID_ARG
    assert B.bcnn_conv2d_binary_branches(desc, 9, x, 0, w, None, 0, g, None, None) == B.BCNN_ERR_INVALID_ARG
    assert B.bcnn_conv2d_binary_branches(desc, 9, x, 0, w, None, 0, g.data_ptr() + 2, None, z) == B.BCNN_ERR_ALIGNMENT
    assert B.bcnn_conv2d_binary_branches(desc, 8, x, 0, w, None, 0, g, None, z) == B.BCNN_ERR_INVALID_ARG
    assert B.bcnn_conv2d_binary_branches(desc, 0, x, 0, w, None, 0, g, None, z) == B.BCNN_ERR_INVALID_ARG
    assert B.bcnn_conv2d_binary_branches(desc, 9, x, 0, w, None, 0, g, None, z) == B.BCNN_OK
    torch.cuda.synchronize()


# ------------------------------------------------------------ full-size shapes
def _branch_params(index):
    cfg = W.CONFIGS[index - 1]
    p = cfg.k * cfg.k
    padv = W.pm1(9200 + index, (p, cfg.c_in))
    g = W.uniform_f32(9300 + index, (p, cfg.c_out), -1.5, 1.5)
    hb = W.uniform_f32(9400 + index, (cfg.c_out,), -40.0, 40.0)
    return padv, g, hb


@functools.lru_cache(maxsize=None)
def _full_size_branch_oracle(index):
    """The oracle's float chain on the whole batch, once per session for all variants."""
    cfg, x_all, ws, _ = W.make_inputs(index)
    padv, g, hb = _branch_params(index)
    _, z32 = oracle.branches_pm1(x_all[None], padv, ws[0], g, hb, cfg.stride, cfg.pad)
    return z32, oracle_bits(z32)


@pytest.mark.parametrize("index", [3, 4, 5])
@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
def test_branches_full_size(dev, index, variant):
    """The launch is the full benchmark shape (3x3, whole batch, one tensor
    shared by the branches, per-branch pad words); the oracle evaluates every
    image and the whole output is compared (shape 5: its first layer)."""
    cfg, x_all, ws, _ = W.make_inputs(index)
    wt = ws[0]
    p = cfg.k * cfg.k
    padv, g, hb = _branch_params(index)
    z32, want_bits = _full_size_branch_oracle(index)
    desc = B.conv_desc(cfg.n, cfg.c_in, cfg.h, cfg.w, cfg.c_out, cfg.k, cfg.stride, cfg.pad)
    ho, wo = B.out_shape(desc)
    xp = B.pack_nchw(up(x_all, dev))
    wp = B.pack_nchw(up(wt, dev))
    pw = up(i32(pack_padv(padv)), dev)
    gt, ht = up(g, dev), up(hb, dev)
    z = torch.empty((cfg.n, ho, wo, cfg.c_out), dtype=torch.float32, device=dev)
    zp = torch.empty((cfg.n, ho * wo, cfg.c_out // 32), dtype=torch.int32, device=dev)
    run_variant(B.bcnn_conv2d_binary_branches(desc, p, xp, 0, wp, pw, B.BCNN_PAD_WORDS, gt, ht, z, variant),
                "branches", variant)
    run_variant(B.bcnn_conv2d_binary_branches_sign_pack(desc, p, xp, 0, wp, pw, B.BCNN_PAD_WORDS, gt, ht, zp,
                                                        variant), "fused", variant)
    torch.cuda.synchronize()
    assert np.array_equal(z.cpu().numpy(), z32)
    assert np.array_equal(zp.cpu().numpy().view(np.uint32), want_bits)


# ------------------------------------------------------------ branches inside a module
TAIL_SHAPES = [
    # n, c_in, h, w, c_out, k or P (negative: -P parallel 1x1 branches), stride, pad
    (2, 256, 14, 14, 128, -2, 1, 0),     # the paper's P = 2 module, matrix-core kernel
    (3, 512, 9, 9, 100, -2, 1, 0),
    (2, 256, 12, 12, 96, 3, 1, 1),       # F x F construction inside a module
    (2, 64, 14, 14, 64, -2, 1, 0),       # vector-ALU kernel
    (3, 96, 7, 9, 70, 3, 2, 1),
    (40, 64, 14, 14, 64, -3, 1, 0),
]


@pytest.mark.parametrize("shape", TAIL_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("half", [False, True], ids=["f32", "f16"])
@pytest.mark.parametrize("mode", ["minus", "words", "zero"])
def test_branches_module_matches_oracle(dev, shape, variant, half, mode):
    """Parallel branches (or the nine shifted ones) followed by identity
    addition, PReLU, real stream out and the next module's bias + sign."""
    n, c, h, w, o, kp, stride, pad = shape
    k, p = (1, -kp) if kp < 0 else (kp, kp * kp)
    if k == 1 and mode != "minus":
        pytest.skip("no padding with 1x1 branches")
    seed = 9900 + sum(v * q for v, q in zip(shape, (3, 5, 7, 11, 13, 17, 19, 23))) + half + 2 * MODES.index(mode)
    xb = W.pm1(seed, (p, n, c, h, w), 0.45)
    wt = W.pm1(seed + 1, (o, c, p) if k == 1 else (o, c, k, k))
    padv = W.pm1(seed + 2, (p, c))
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    m = n * ho * wo
    for grid in (False, True):
        if grid:
            g = W.uniform_f32(seed + 3, (p, o), -2.0, 2.0, steps=16)
            hb = W.uniform_f32(seed + 4, (o,), -8.0, 8.0, steps=64)
            ident = W.uniform_f32(seed + 5, (m, o), -16.0, 16.0, steps=128)
            alpha = W.uniform_f32(seed + 6, (o,), 0.0, 1.0, steps=4)
            cn = W.uniform_f32(seed + 7, (o,), -4.0, 4.0, steps=32)
        else:
            g = W.uniform_f32(seed + 3, (p, o), -1.5, 1.5)
            hb = W.uniform_f32(seed + 4, (o,), -30.0, 30.0)
            ident = W.uniform_f32(seed + 5, (m, o), -40.0, 40.0)
            alpha = W.uniform_f32(seed + 6, (o,), 0.05, 0.5)
            cn = W.uniform_f32(seed + 7, (o,), -10.0, 10.0)
        if half:
            ident = oracle.store_f16(ident)
        if mode == "minus":
            padv_o, words, code = -np.ones((p, c), dtype=np.int8), None, B.BCNN_PAD_WORDS
        elif mode == "words":
            padv_o, words, code = padv, pack_padv(padv), B.BCNN_PAD_WORDS
        else:
            padv_o, words, code = np.zeros((p, c), dtype=np.int8), None, B.BCNN_PAD_ZERO
        z64, z32 = oracle.branches_pm1(xb, padv_o, wt, g, hb, stride, pad)
        _, r32 = oracle.module_tail(z64, z32, ident.astype(np.float32).reshape(z32.shape), alpha)
        stored = oracle.store_f16(r32) if half else r32
        sgn = oracle.sign_bias_f32(stored.astype(np.float32).reshape(m, o, 1), cn)
        want_bits = oracle.pack_channels(sgn.reshape(n, ho * wo, o).transpose(0, 2, 1))

        desc = B.conv_desc(n, c, h, w, o, k, stride, pad)
        cw = (c + 31) // 32
        xp = up(i32(np.stack([pack_nchw(xb[t]) for t in range(p)])), dev)
        wp = up(i32(oracle.pack_channels(wt.reshape(o, c, -1))), dev)
        esz = 2 if half else 4
        rbuf = Guarded((m * o * esz + 3) // 4, dev)
        rbuf.buf.view(torch.uint8)[4 * GUARD:4 * GUARD + m * o * esz] = \
            torch.from_numpy(np.ascontiguousarray(ident).view(np.uint8).reshape(-1)).to(dev)
        cwo = (o + 31) // 32
        bits = Guarded(m * cwo, dev)
        rc = B.bcnn_conv2d_binary_branches_module(
            desc, p, xp, n * h * w * cw, wp, up(i32(words), dev) if words is not None else None, code, up(g, dev),
            up(hb, dev), rbuf.ptr, up(alpha, dev), up(cn, dev), B.BCNN_F16 if half else B.BCNN_F32, rbuf.ptr,
            bits.ptr, variant)
        run_variant(rc, "branches_module", variant)
        got_r = rbuf.get(np.uint8)[:m * o * esz].view(np.float16 if half else np.float32).reshape(m, o)
        assert np.array_equal(got_r, stored.reshape(m, o))
        assert np.array_equal(bits.get(np.uint32).reshape(n, ho * wo, cwo), want_bits)
