"""Seeded random shapes through every convolution entry point (plain, fused,
module, branch, branch + module tail), each compared bit for bit with the CPU
oracle.  The fixed shape lists of the other GPU tests aim at known tile edges;
this one looks for the edges nobody thought of.  Shapes stay inside what the
header documents as supported; a variant that does not cover a shape skips.
"""
import os

import numpy as np
import pytest

import oracle
from paper_2010_00704_amd import binding as B
from paper_2010_00704_amd import workloads as W
from gpu_helpers import (COVER_ALL, Guarded, gpu_device, i32, oracle_bits_of_sign, oracle_pack_nchw,
                         oracle_pack_vectors, up)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    return gpu_device()


def draw_shape(rng, mfma_friendly):
    k = int(rng.choice([1, 3]))
    stride = int(rng.choice([1, 2]))
    pad = int(rng.integers(0, 2)) if k == 3 else 0
    if mfma_friendly:
        c_in = int(rng.choice([128, 256, 384, 512]))
        c_out = int(rng.choice([64, 96, 100, 128, 130, 192, 257]))
        n = int(rng.integers(1, 5))
        h, w = int(rng.integers(12, 30)), int(rng.integers(12, 30))
    else:
        c_in = int(rng.integers(1, 200))
        c_out = int(rng.integers(1, 150))
        n = int(rng.integers(1, 4))
        h, w = int(rng.integers(k, 16)), int(rng.integers(k, 16))
    return n, c_in, h, w, c_out, k, stride, pad


# BCNN_TEST_EXTRA_SEEDS=N adds N more seeds to every test below (a longer run for a changed kernel)
EXTRA = int(os.environ.get("BCNN_TEST_EXTRA_SEEDS", "0"))
CASES = [(seed, seed % 2 == 0) for seed in range(40 + EXTRA)]


@pytest.mark.parametrize("seed,mfma_friendly", CASES)
def test_random_plain_and_fused(dev, seed, mfma_friendly):
    rng = np.random.default_rng(12000 + seed)
    n, c, h, w, o, k, stride, pad = draw_shape(rng, mfma_friendly)
    x = W.pm1(12100 + seed, (n, c, h, w), float(rng.choice([0.3, 0.5, 0.7])))
    wt = W.pm1(12200 + seed, (o, c, k, k))
    y = oracle.conv2d_pm1(x, wt, stride, pad)
    kk = c * k * k
    thr = W.thresholds(12300 + seed, o, max(1, int(2 * np.sqrt(kk))))
    want_bits = oracle_bits_of_sign(oracle.threshold_sign(y, thr))
    desc = B.conv_desc(n, c, h, w, o, k, stride, pad)
    xp = up(i32(oracle_pack_nchw(x)), dev)
    wp = up(i32(oracle_pack_nchw(wt)), dev)
    variants = [B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU]
    if mfma_friendly:
        variants += [B.BCNN_VARIANT_MFMA_FP4_T4, B.BCNN_VARIANT_MFMA_FP4_T7, B.BCNN_VARIANT_MFMA_I8]
    ran = 0
    for v in variants:
        out = Guarded(y.size, dev)
        rc = B.bcnn_conv2d_binary_variant(desc, xp, wp, None, out.ptr, v)
        if rc != B.BCNN_ERR_UNSUPPORTED or v in COVER_ALL:
            B.check(rc, "conv")
            assert np.array_equal(out.get(np.int32).reshape(y.shape), y), "variant %d sums" % v
            ran += 1
        bits = Guarded(want_bits.size, dev)
        rc = B.bcnn_conv2d_binary_variant(desc, xp, wp, up(thr, dev), bits.ptr, v)
        if rc != B.BCNN_ERR_UNSUPPORTED or v in COVER_ALL:
            B.check(rc, "fused")
            assert np.array_equal(bits.get(np.uint32).reshape(want_bits.shape), want_bits), "variant %d bits" % v
            ran += 1
    assert ran >= 4


@pytest.mark.parametrize("seed", range(16 + EXTRA))
def test_random_position_major(dev, seed):
    """Shapes the position-major tilings cover (3 x 3 filter, whole groups of 32 images, c_in a multiple of 256
    give or take tail bits): every such tiling and the default choice against the oracle."""
    rng = np.random.default_rng(17000 + seed)
    n = 32 * int(rng.integers(1, 4))
    c = int(rng.choice([256, 512, 768, 1024])) - int(rng.choice([0, 0, 5, 31]))
    h, w = int(rng.integers(2, 13)), int(rng.integers(2, 13))
    o = int(rng.choice([32, 64, 100, 128, 130, 257]))
    stride, pad = int(rng.choice([1, 2])), int(rng.integers(0, 2))
    if (h + 2 * pad - 3) // stride + 1 < 1 or (w + 2 * pad - 3) // stride + 1 < 1:
        pad = 1
    x = W.pm1(17100 + seed, (n, c, h, w), float(rng.choice([0.3, 0.5, 0.7])))
    wt = W.pm1(17200 + seed, (o, c, 3, 3))
    y = oracle.conv2d_pm1(x, wt, stride, pad)
    thr = (int(np.median(y)) + W.thresholds(17300 + seed, o, max(1, int(2 * np.sqrt(9 * c))))).astype(np.int32)
    want_bits = oracle_bits_of_sign(oracle.threshold_sign(y, thr))
    desc = B.conv_desc(n, c, h, w, o, 3, stride, pad)
    xp = up(i32(oracle_pack_nchw(x)), dev)
    wp = up(i32(oracle_pack_nchw(wt)), dev)
    ran = 0
    for v in (B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_MFMA_FP4_P5, B.BCNN_VARIANT_MFMA_FP4_P68, B.BCNN_VARIANT_MFMA_FP4_P6,
              B.BCNN_VARIANT_MFMA_FP4_P7):
        bits = Guarded(want_bits.size, dev)
        rc = B.bcnn_conv2d_binary_variant(desc, xp, wp, up(thr, dev), bits.ptr, v)
        B.check(rc, "fused")       # (maps of two or more rows and columns: no window misses the image on both sides)
        assert np.array_equal(bits.get(np.uint32).reshape(want_bits.shape), want_bits), "variant %d bits" % v
        ran += 1
    assert ran == 5


@pytest.mark.parametrize("seed,mfma_friendly", CASES[:24 + EXTRA])
@pytest.mark.parametrize("half", [False, True], ids=["f32", "f16"])
def test_random_module(dev, seed, mfma_friendly, half):
    rng = np.random.default_rng(13000 + seed)
    n, c, h, w, o, k, stride, pad = draw_shape(rng, mfma_friendly)
    x = W.pm1(13100 + seed, (n, c, h, w))
    wt = W.pm1(13200 + seed, (o, c, k, k))
    y = oracle.conv2d_pm1(x, wt, stride, pad)
    _, ho, wo, _ = y.shape
    m = n * ho * wo
    g = W.uniform_f32(13300 + seed, (o,), -1.5, 1.5)
    b = W.uniform_f32(13400 + seed, (o,), -20.0, 20.0)
    idc = o if seed % 3 else max(1, o // 2)                      # sometimes a narrower, replicated identity
    ident = W.uniform_f32(13500 + seed, (m, idc), -30.0, 30.0)
    alpha = W.uniform_f32(13600 + seed, (o,), 0.0, 0.5)
    cn = W.uniform_f32(13700 + seed, (o,), -5.0, 5.0)
    if half:
        ident = oracle.store_f16(ident)
    ident_full = oracle.replicate_channels(ident.astype(np.float32), -(-o // idc), axis=1)[:, :o]
    _, r32 = oracle.module_epilogue(y, g, b, ident_full.reshape(y.shape), alpha)
    stored = (oracle.store_f16(r32) if half else r32).reshape(m, o)
    sgn = oracle.sign_bias_f32(stored.astype(np.float32).reshape(m, o, 1), cn)
    want_bits = oracle_bits_of_sign(sgn.reshape(n, ho, wo, o))
    desc = B.conv_desc(n, c, h, w, o, k, stride, pad)
    xp = up(i32(oracle_pack_nchw(x)), dev)
    wp = up(i32(oracle_pack_nchw(wt)), dev)
    for v in (B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU, B.BCNN_VARIANT_MFMA_FP4):
        rbuf = Guarded.of_bytes(m * o * (2 if half else 4), dev)
        bits = Guarded(want_bits.size, dev)
        rc = B.bcnn_conv2d_binary_module(desc, xp, wp, up(g, dev), up(b, dev), up(ident, dev), up(alpha, dev),
                                         up(cn, dev), B.BCNN_F16 if half else B.BCNN_F32, rbuf.ptr, bits.ptr, v,
                                         identity_channels=idc)
        if rc == B.BCNN_ERR_UNSUPPORTED and v not in COVER_ALL:
            continue
        B.check(rc, "module")
        assert np.array_equal(rbuf.get(np.float16 if half else np.float32, m * o).reshape(m, o), stored)
        assert np.array_equal(bits.get(np.uint32).reshape(want_bits.shape), want_bits)


@pytest.mark.parametrize("seed", range(24 + EXTRA))
def test_random_branches(dev, seed):
    rng = np.random.default_rng(14000 + seed)
    mfma_friendly = seed % 2 == 0
    k = 3 if seed % 3 else 1
    p = 9 if k == 3 else int(rng.integers(1, 5))
    stride = int(rng.choice([1, 2]))
    pad = int(rng.integers(0, 2)) if k == 3 else 0
    if mfma_friendly:
        c, o = int(rng.choice([256, 512])), int(rng.choice([64, 100, 128, 160]))
        n, h, w = int(rng.integers(2, 5)), int(rng.integers(10, 20)), int(rng.integers(10, 20))
    else:
        c, o = int(rng.integers(1, 150)), int(rng.integers(1, 120))
        n, h, w = int(rng.integers(1, 3)), int(rng.integers(k, 12)), int(rng.integers(k, 12))
    shared = bool(seed % 4 < 2)
    xb = W.pm1(14100 + seed, (1 if shared else p, n, c, h, w), 0.45)
    wt = W.pm1(14200 + seed, (o, c, p) if k == 1 else (o, c, k, k))
    padv = W.pm1(14300 + seed, (p, c))
    g = W.uniform_f32(14400 + seed, (p, o), -1.5, 1.5)
    hb = W.uniform_f32(14500 + seed, (o,), -20.0, 20.0)
    mode = ["minus", "words", "zero"][seed % 3] if k == 3 else "minus"
    if mode == "minus":
        padv_o, words, code = -np.ones((p, c), dtype=np.int8), None, B.BCNN_PAD_WORDS
    elif mode == "words":
        padv_o, words, code = padv, oracle_pack_vectors(padv), B.BCNN_PAD_WORDS
    else:
        padv_o, words, code = np.zeros((p, c), dtype=np.int8), None, B.BCNN_PAD_ZERO
    z64, z32 = oracle.branches_pm1(xb, padv_o, wt, g, hb, stride, pad)
    want_bits = oracle_bits_of_sign(oracle.sign_f32(z32))
    _, ho, wo, _ = z32.shape
    m = n * ho * wo
    ident = W.uniform_f32(14600 + seed, (m, o), -30.0, 30.0)
    alpha = W.uniform_f32(14700 + seed, (o,), 0.0, 0.5)
    cn = W.uniform_f32(14800 + seed, (o,), -5.0, 5.0)
    _, r32 = oracle.module_tail(z64, z32, ident.reshape(z32.shape), alpha)
    tail_bits = oracle_bits_of_sign(oracle.sign_bias_f32(r32.reshape(m, o, 1), cn).reshape(n, ho, wo, o))
    desc = B.conv_desc(n, c, h, w, o, k, stride, pad)
    cw = (c + 31) // 32
    xp = up(i32(np.stack([oracle_pack_nchw(xb[t]) for t in range(xb.shape[0])])), dev)
    wp = up(i32(oracle.pack_channels(wt.reshape(o, c, -1))), dev)
    xs = 0 if shared else n * h * w * cw
    pw = up(i32(words), dev) if words is not None else None
    for v in (B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU, B.BCNN_VARIANT_MFMA_FP4):
        out = Guarded(z32.size, dev)
        rc = B.bcnn_conv2d_binary_branches(desc, p, xp, xs, wp, pw, code, up(g, dev), up(hb, dev), out.ptr, v)
        if rc == B.BCNN_ERR_UNSUPPORTED and v not in COVER_ALL:
            continue
        B.check(rc, "branches")
        assert np.array_equal(out.get(np.float32).reshape(z32.shape), z32)
        bits = Guarded(want_bits.size, dev)
        B.check(B.bcnn_conv2d_binary_branches_sign_pack(desc, p, xp, xs, wp, pw, code, up(g, dev), up(hb, dev),
                                                        bits.ptr, v), "branches_sign_pack")
        assert np.array_equal(bits.get(np.uint32).reshape(want_bits.shape), want_bits)
        if o >= 32:
            rbuf = Guarded(m * o, dev)
            tb = Guarded(tail_bits.size, dev)
            B.check(B.bcnn_conv2d_binary_branches_module(desc, p, xp, xs, wp, pw, code, up(g, dev), up(hb, dev),
                                                         up(ident, dev), up(alpha, dev), up(cn, dev), B.BCNN_F32,
                                                         rbuf.ptr, tb.ptr, v), "branches_module")
            assert np.array_equal(rbuf.get(np.float32).reshape(m, o), r32.reshape(m, o))
            assert np.array_equal(tb.get(np.uint32).reshape(tail_bits.shape), tail_bits)


TINY = [
    # n, c_in, h, w, c_out, k, stride, pad: problems far smaller than one matrix-core tile, which AUTO
    # still sends to the matrix-core kernel whenever the channel count allows it
    (1, 128, 1, 1, 1, 1, 1, 0),
    (1, 128, 1, 1, 32, 1, 1, 0),
    (1, 256, 1, 2, 100, 1, 1, 0),
    (1, 128, 3, 3, 7, 3, 1, 1),
    (1, 256, 3, 3, 64, 3, 1, 0),        # a single output pixel from a 3x3 window
    (2, 128, 4, 4, 33, 3, 2, 1),
    (1, 384, 5, 7, 130, 3, 1, 1),       # c_in a multiple of 128 but not of 256
    (1, 512, 7, 7, 512, 3, 1, 1),
    (3, 256, 2, 5, 40, 1, 2, 0),
]


@pytest.mark.parametrize("shape", TINY, ids=lambda s: "x".join(map(str, s)))
def test_tiny_problems_on_every_path(dev, shape):
    n, c, h, w, o, k, stride, pad = shape
    seed = 15000 + 31 * c + 7 * o + h
    x = W.pm1(seed, (n, c, h, w))
    wt = W.pm1(seed + 1, (o, c, k, k))
    y = oracle.conv2d_pm1(x, wt, stride, pad)
    thr = W.thresholds(seed + 2, o, max(1, int(2 * np.sqrt(c * k * k))))
    want_bits = oracle_bits_of_sign(oracle.threshold_sign(y, thr))
    desc = B.conv_desc(n, c, h, w, o, k, stride, pad)
    xp = up(i32(oracle_pack_nchw(x)), dev)
    wp = up(i32(oracle_pack_nchw(wt)), dev)
    for v in (B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU, B.BCNN_VARIANT_MFMA_FP4_T4, B.BCNN_VARIANT_MFMA_FP4_T7,
              B.BCNN_VARIANT_MFMA_I8):
        out = Guarded(y.size, dev)
        rc = B.bcnn_conv2d_binary_variant(desc, xp, wp, None, out.ptr, v)
        if rc != B.BCNN_ERR_UNSUPPORTED or v in COVER_ALL:
            B.check(rc, "conv")
            assert np.array_equal(out.get(np.int32).reshape(y.shape), y), "variant %d sums" % v
        bits = Guarded(want_bits.size, dev)
        rc = B.bcnn_conv2d_binary_variant(desc, xp, wp, up(thr, dev), bits.ptr, v)
        if rc != B.BCNN_ERR_UNSUPPORTED or v in COVER_ALL:
            B.check(rc, "fused")
            assert np.array_equal(bits.get(np.uint32).reshape(want_bits.shape), want_bits), "variant %d bits" % v
    # the module call on the same tiny problem (AUTO stays on the vector ALUs here, the matrix cores are forced)
    _, ho, wo, _ = y.shape
    m = n * ho * wo
    g = W.uniform_f32(seed + 3, (o,), -1.5, 1.5)
    b = W.uniform_f32(seed + 4, (o,), -20.0, 20.0)
    ident = W.uniform_f32(seed + 5, (m, o), -30.0, 30.0)
    alpha = W.uniform_f32(seed + 6, (o,), 0.0, 0.5)
    cn = W.uniform_f32(seed + 7, (o,), -5.0, 5.0)
    _, r32 = oracle.module_epilogue(y, g, b, ident.reshape(y.shape), alpha)
    mod_bits = oracle_bits_of_sign(oracle.sign_bias_f32(r32.reshape(m, o, 1), cn).reshape(n, ho, wo, o))
    for v in (B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU, B.BCNN_VARIANT_MFMA_FP4):
        rbuf = Guarded(m * o, dev)
        nb = Guarded(mod_bits.size, dev)
        rc = B.bcnn_conv2d_binary_module(desc, xp, wp, up(g, dev), up(b, dev), up(ident, dev), up(alpha, dev),
                                         up(cn, dev), B.BCNN_F32, rbuf.ptr, nb.ptr, v)
        if rc == B.BCNN_ERR_UNSUPPORTED and v not in COVER_ALL:
            continue
        B.check(rc, "module")
        assert np.array_equal(rbuf.get(np.float32, m * o).reshape(m, o), r32.reshape(m, o)), "variant %d stream" % v
        assert np.array_equal(nb.get(np.uint32).reshape(mod_bits.shape), mod_bits), "variant %d next bits" % v


@pytest.mark.parametrize("shape", [(1, 256, 1, 1, 32, 1, 1, 0, 3), (1, 256, 3, 3, 64, 3, 1, 1, 9), (2, 512, 4, 5, 100, 3, 2, 1, 9),
                                   (1, 256, 3, 3, 40, 3, 1, 0, 9), (3, 256, 2, 2, 1, 1, 1, 0, 2)],
                         ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("mode", ["minus", "words", "zero"])
def test_tiny_branch_problems_on_every_path(dev, shape, mode):
    n, c, h, w, o, k, stride, pad, p = shape
    if k == 1 and mode != "minus":
        pytest.skip("unshifted branches have no padding")
    seed = 16000 + 13 * o + h + 100 * ["minus", "words", "zero"].index(mode)
    xb = W.pm1(seed, (p, n, c, h, w), 0.45)
    wt = W.pm1(seed + 1, (o, c, p) if k == 1 else (o, c, k, k))
    padv = W.pm1(seed + 2, (p, c))
    g = W.uniform_f32(seed + 3, (p, o), -1.5, 1.5)
    hb = W.uniform_f32(seed + 4, (o,), -20.0, 20.0)
    if mode == "minus":
        padv_o, words, code = -np.ones((p, c), dtype=np.int8), None, B.BCNN_PAD_WORDS
    elif mode == "words":
        padv_o, words, code = padv, oracle_pack_vectors(padv), B.BCNN_PAD_WORDS
    else:
        padv_o, words, code = np.zeros((p, c), dtype=np.int8), None, B.BCNN_PAD_ZERO
    _, z32 = oracle.branches_pm1(xb, padv_o, wt, g, hb, stride, pad)
    want_bits = oracle_bits_of_sign(oracle.sign_f32(z32))
    desc = B.conv_desc(n, c, h, w, o, k, stride, pad)
    cw = (c + 31) // 32
    xp = up(i32(np.stack([oracle_pack_nchw(xb[t]) for t in range(p)])), dev)
    wp = up(i32(oracle.pack_channels(wt.reshape(o, c, -1))), dev)
    pw = up(i32(words), dev) if words is not None else None
    for v in (B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU, B.BCNN_VARIANT_MFMA_FP4):
        out = Guarded(z32.size, dev)
        rc = B.bcnn_conv2d_binary_branches(desc, p, xp, n * h * w * cw, wp, pw, code, up(g, dev), up(hb, dev), out.ptr, v)
        if rc == B.BCNN_ERR_UNSUPPORTED and v not in COVER_ALL:
            continue
        B.check(rc, "branches")
        assert np.array_equal(out.get(np.float32).reshape(z32.shape), z32), "variant %d" % v
        bits = Guarded(want_bits.size, dev)
        B.check(B.bcnn_conv2d_binary_branches_sign_pack(desc, p, xp, n * h * w * cw, wp, pw, code, up(g, dev),
                                                        up(hb, dev), bits.ptr, v), "branches_sign_pack")
        assert np.array_equal(bits.get(np.uint32).reshape(want_bits.shape), want_bits), "variant %d bits" % v
