"""Parity of the HIP library with the CPU oracle on a real MI355X (bit-exact).

Every comparison is element by element on int32 sums or packed words; both
sides receive the same seeded host tensors.  Outputs are written between
sentinel guard bands that must stay untouched.
"""
import functools
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2010_00704_amd import binding as B
from paper_2010_00704_amd import workloads as W
from gpu_helpers import COVER_ALL, Guarded, gpu_device, i32, oracle_pack_nchw, run_variant, up

pytestmark = pytest.mark.gpu

VARIANTS = [B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU, B.BCNN_VARIANT_MFMA_FP4_T4, B.BCNN_VARIANT_MFMA_FP4_T7,
            B.BCNN_VARIANT_MFMA_I8, B.BCNN_VARIANT_MFMA_FP4_P6, B.BCNN_VARIANT_MFMA_FP4_P7, B.BCNN_VARIANT_MFMA_FP4_P5,
            B.BCNN_VARIANT_MFMA_FP4_P68]
VARIANT_IDS = ["auto", "valu", "mfma_fp4_t4", "mfma_fp4_t7", "mfma_i8", "mfma_fp4_p6", "mfma_fp4_p7", "mfma_fp4_p5", "mfma_fp4_p68"]


@pytest.fixture(scope="module")
def dev():
    return gpu_device()


def packed_view(a):
    return i32(a)


def oracle_pack_weights(w):
    return oracle_pack_nchw(w)   # [o, kh*kw, cw]


def rand_pm1(rng, shape, p=0.5):
    return np.where(rng.random(shape) < p, 1, -1).astype(np.int8)


def gpu_conv(dev, x, w, stride, pad, thr=None, variant=B.BCNN_VARIANT_AUTO, entry="variant", must_cover=False):
    """x, w logical +-1 tensors (packed on the host by the oracle's packer).  must_cover: a refusal
    of the shape by the variant is a failure, not a skip."""
    n, c, h, wd = x.shape
    o, _, k, _ = w.shape
    desc = B.conv_desc(n, c, h, wd, o, k, stride, pad)
    ho, wo = B.out_shape(desc)
    xp = up(packed_view(oracle_pack_nchw(x)), dev)
    wp = up(packed_view(oracle_pack_weights(w)), dev)
    if thr is None:
        out = Guarded(n * ho * wo * o, dev)
        if entry == "variant":
            rc = B.bcnn_conv2d_binary_variant(desc, xp, wp, None, out.ptr, variant)
        else:
            rc = B.bcnn_conv2d_binary(desc, xp, wp, out.ptr)
        run_variant(rc, "conv", variant if entry == "variant" else B.BCNN_VARIANT_AUTO)
        return out.get(np.int32).reshape(n, ho, wo, o)
    cwo = (o + 31) // 32
    t = up(np.asarray(thr, dtype=np.int32), dev)
    out = Guarded(n * ho * wo * cwo, dev)
    if entry == "variant":
        rc = B.bcnn_conv2d_binary_variant(desc, xp, wp, t, out.ptr, variant)
    else:
        rc = B.bcnn_conv2d_binary_sign_pack(desc, xp, wp, t, out.ptr)
    run_variant(rc, "conv_sign_pack", variant if entry == "variant" and not must_cover else B.BCNN_VARIANT_AUTO)
    return out.get(np.uint32).reshape(n, ho * wo, cwo)


def oracle_fused(x, w, stride, pad, thr):
    y = oracle.conv2d_pm1(x, w, stride, pad)
    n, ho, wo, o = y.shape
    s = oracle.threshold_sign(y, thr)                       # [n, ho, wo, o]
    s_ncp = s.reshape(n, ho * wo, o).transpose(0, 2, 1)     # [n, o, ho*wo]
    return y, oracle.pack_channels(s_ncp)                   # [n, ho*wo, cwo]


# ------------------------------------------------------------------ packing
PACK_SHAPES = [
    # outer, channels, inner
    (2, 64, 196), (3, 33, 300), (1, 256, 784), (2, 1, 70), (5, 31, 64), (2, 65, 129),
    (7, 64, 9), (64, 64, 9), (3, 40, 1), (100, 256, 1), (9, 65, 1), (1, 32, 1), (2, 300, 5),
    (13, 96, 63), (1, 1, 1), (4, 1024, 49), (3, 70, 17), (2, 96, 33), (6, 33, 8), (3, 64, 4),
    (40, 256, 196), (2, 512, 3136),
    (11, 65, 3000), (9, 1030, 3644), (170, 96, 196),      # four pixels per thread, whole rows per block
]


@pytest.mark.parametrize("shape", PACK_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f32", "f16", "i8", "bf16"])
def test_pack_matches_oracle(dev, shape, dtype):
    outer, c, inner = shape
    rng = np.random.default_rng(outer * 1000 + c * 10 + inner)
    vals = rng.standard_normal(shape).astype(np.float32)
    vals[rng.random(shape) < 0.05] = 0.0
    vals[rng.random(shape) < 0.02] = -0.0
    if dtype == "i8":
        src = np.clip(np.round(vals * 40), -128, 127).astype(np.int8)
        as_f32 = src.astype(np.float32)
        code = B.BCNN_I8
    elif dtype == "f16":
        vals[rng.random(shape) < 0.02] = np.nan
        vals[rng.random(shape) < 0.01] = -np.inf
        src = oracle.store_f16(vals)
        as_f32 = src.astype(np.float32)
        code = B.BCNN_F16
    elif dtype == "bf16":
        vals[rng.random(shape) < 0.02] = np.nan
        vals[rng.random(shape) < 0.01] = -np.inf
        vals[rng.random(shape) < 0.01] = -1e-40  # negative bfloat16 denormal
        src, as_f32 = oracle.store_bf16(vals)
        code = B.BCNN_BF16
    else:
        vals[rng.random(shape) < 0.02] = np.nan
        vals[rng.random(shape) < 0.01] = np.inf
        vals[rng.random(shape) < 0.01] = -1e-42  # negative denormal
        src = vals
        as_f32 = src
        code = B.BCNN_F32
    want = oracle.pack_channels(oracle.sign_f32(as_f32))
    out = Guarded(want.size, dev)
    B.check(B.bcnn_pack(up(src, dev), code, outer, c, inner, out.ptr), "pack")
    np.testing.assert_array_equal(out.get().reshape(want.shape), want)


# ------------------------------------------------------- convolution, int32
CONV_SHAPES = [
    # n, c, h, w, o, k, stride, pad
    (1, 64, 14, 14, 64, 3, 1, 1),      # config 1
    (2, 32, 5, 5, 32, 3, 1, 1), (1, 7, 6, 5, 5, 3, 1, 1), (3, 33, 9, 7, 40, 3, 2, 1),
    (2, 96, 8, 8, 33, 1, 1, 0), (1, 256, 13, 13, 64, 1, 2, 0), (2, 128, 15, 17, 96, 3, 2, 1),
    (1, 64, 3, 3, 32, 3, 1, 0), (1, 1, 4, 4, 1, 3, 1, 1), (5, 64, 1, 1, 70, 1, 1, 0),
    (1, 100, 2, 2, 31, 3, 1, 1), (4, 256, 7, 7, 128, 3, 1, 1), (2, 512, 6, 6, 64, 3, 2, 0),
    (1, 192, 20, 20, 160, 3, 1, 1), (3, 1024, 4, 4, 96, 1, 1, 0), (2, 160, 11, 11, 48, 3, 1, 0),
    (2, 64, 30, 31, 64, 3, 2, 1), (1, 320, 9, 9, 257, 3, 1, 1),
    (3, 128, 19, 17, 130, 3, 1, 1), (2, 128, 9, 9, 64, 1, 1, 0), (1, 384, 33, 20, 200, 3, 2, 1),
    (2, 256, 16, 16, 128, 3, 1, 1), (1, 100, 12, 12, 48, 3, 1, 1), (5, 128, 3, 3, 384, 1, 2, 0),
]


@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_int32_matches_oracle(dev, shape, variant):
    n, c, h, wd, o, k, s, p = shape
    rng = np.random.default_rng(sum(shape) * 31 + k)
    x = rand_pm1(rng, (n, c, h, wd), 0.4)
    w = rand_pm1(rng, (o, c, k, k))
    want = oracle.conv2d_pm1(x, w, s, p)
    got = gpu_conv(dev, x, w, s, p, variant=variant)
    np.testing.assert_array_equal(got, want)


def test_config1_through_the_named_entry_points(dev):
    cfg, x, ws, _ = W.make_inputs(1)
    want = oracle.conv2d_pm1(x, ws[0], cfg.stride, cfg.pad)
    got = gpu_conv(dev, x, ws[0], cfg.stride, cfg.pad, entry="named")
    np.testing.assert_array_equal(got, want)
    thr = W.thresholds(77, cfg.c_out, W.k_total(cfg) // 8)
    _, want_bits = oracle_fused(x, ws[0], cfg.stride, cfg.pad, thr)
    got_bits = gpu_conv(dev, x, ws[0], cfg.stride, cfg.pad, thr=thr, entry="named")
    np.testing.assert_array_equal(got_bits, want_bits)


def test_conv_extreme_inputs(dev):
    """All +1 / all -1 operands reach |y| = K at interior pixels and exercise
    full and empty popcounts; -1 padding shows at the border."""
    n, c, h, wd, o, k = 1, 96, 6, 6, 32, 3
    for xs, wsgn in [(1, 1), (1, -1), (-1, 1), (-1, -1)]:
        x = np.full((n, c, h, wd), xs, dtype=np.int8)
        w = np.full((o, c, k, k), wsgn, dtype=np.int8)
        got = gpu_conv(dev, x, w, 1, 1)
        np.testing.assert_array_equal(got, oracle.conv2d_pm1(x, w, 1, 1))
        assert abs(int(got[0, 2, 2, 0])) == c * 9


# ------------------------------------------------ fused threshold/sign/repack
FUSED_SHAPES = [
    (2, 64, 9, 9, 64, 3, 1, 1), (1, 96, 7, 6, 33, 3, 2, 1), (3, 128, 5, 5, 100, 1, 1, 0),
    (2, 256, 10, 10, 256, 3, 1, 1), (1, 40, 8, 8, 31, 3, 1, 0), (2, 64, 12, 12, 65, 3, 2, 1),
    (1, 512, 7, 7, 64, 3, 1, 1), (3, 128, 17, 15, 130, 3, 1, 1), (2, 384, 20, 20, 100, 3, 2, 1),
    (6, 128, 8, 8, 257, 1, 1, 0),
]


@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("tight", [False, True], ids=["k8", "tight"])
@pytest.mark.parametrize("shape", FUSED_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_fused_epilogue_matches_oracle(dev, shape, tight, variant):
    n, c, h, wd, o, k, s, p = shape
    rng = np.random.default_rng(sum(shape) * 17 + int(tight))
    x = rand_pm1(rng, (n, c, h, wd), 0.3)
    w = rand_pm1(rng, (o, c, k, k))
    kk = c * k * k
    bound = int(2 * math.sqrt(kk)) if tight else kk // 8
    thr = rng.integers(-bound, bound + 1, size=o).astype(np.int32)
    y, want = oracle_fused(x, w, s, p, thr)
    got = gpu_conv(dev, x, w, s, p, thr=thr, variant=variant)
    np.testing.assert_array_equal(got, want)
    if tight:
        # the case is only meaningful if ties and both outcomes occur
        assert (y == thr[None, None, None, :]).any() or (np.abs(y - thr) <= 2).any()
        on = oracle.threshold_sign(y, thr) > 0
        assert on.any() and (~on).any()
    # fused == unfused on the GPU: int32 sums, then the stand-alone epilogue
    y_gpu = gpu_conv(dev, x, w, s, p, variant=variant)
    rows = y_gpu.size // o
    out = Guarded(rows * ((o + 31) // 32), dev)
    B.check(B.bcnn_threshold_sign_pack(up(y_gpu, dev), up(thr, dev), rows, o, out.ptr), "thr")
    np.testing.assert_array_equal(out.get().reshape(want.shape), want)


# Position-major tiles (a block of 32 GEMM rows = one output position in 32 images; taps outside
# the image are not walked but accounted for per channel).  Shapes the scheme covers: a refusal is a
# failure here.  They span: no interior (2 x 2), no edges (pad 0), edges on two sides only (stride 2),
# ragged last tiles of every class, several groups of 32 images, a ragged channel tile, channel counts
# that leave tail bits in the last word of every tap, thresholds out of reach.
POS_SHAPES = [
    (32, 256, 7, 7, 128, 3, 1, 1), (64, 256, 5, 6, 130, 3, 1, 1), (32, 512, 9, 8, 64, 3, 2, 1),
    (96, 256, 3, 3, 96, 3, 1, 1), (32, 256, 4, 5, 32, 3, 1, 0), (32, 256, 2, 2, 40, 3, 1, 1),
    (32, 250, 6, 6, 40, 3, 1, 1), (64, 225, 8, 8, 257, 3, 2, 1), (32, 256, 15, 13, 64, 3, 1, 1),
    (128, 256, 2, 3, 33, 3, 1, 1), (32, 768, 3, 4, 256, 3, 1, 1),
    # wide channel counts: the skipped taps' weight words are counted in one pass (1024 channels) or two (2048, 2540)
    (32, 1024, 4, 5, 130, 3, 1, 1), (32, 2048, 3, 3, 64, 3, 1, 1), (32, 2540, 2, 3, 40, 3, 1, 1),
]


POS_VARIANTS = [B.BCNN_VARIANT_MFMA_FP4_P6, B.BCNN_VARIANT_MFMA_FP4_P7, B.BCNN_VARIANT_MFMA_FP4_P5, B.BCNN_VARIANT_MFMA_FP4_P68]


@pytest.mark.parametrize("variant", POS_VARIANTS, ids=["p6", "p7", "p5", "p68"])
@pytest.mark.parametrize("shape", POS_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_position_major_tiles_match_oracle(dev, shape, variant):
    n, c, h, wd, o, k, s, p = shape
    rng = np.random.default_rng(sum(shape) * 13 + variant)
    x = rand_pm1(rng, (n, c, h, wd), 0.35)
    w = rand_pm1(rng, (o, c, k, k), 0.45)
    kk = c * k * k
    bound = int(2 * math.sqrt(kk))
    # thresholds around the sums' median (the operands are biased, so the sums are not centred on 0)
    centre = int(np.median(oracle.conv2d_pm1(x, w, s, p)))
    thr = (centre + rng.integers(-bound, bound + 1, size=o)).astype(np.int32)
    thr[0] = np.iinfo(np.int32).min
    thr[-1] = np.iinfo(np.int32).max
    y, want = oracle_fused(x, w, s, p, thr)
    assert (np.abs(y - thr) <= 1).any()
    on = oracle.threshold_sign(y, thr) > 0
    assert on[..., 1:-1].any() and (~on[..., 1:-1]).any()
    got = gpu_conv(dev, x, w, s, p, thr=thr, variant=variant, must_cover=True)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("variant", POS_VARIANTS, ids=["p6", "p7", "p5", "p68"])
def test_position_major_closed_form(dev, variant):
    """All-(+1) inputs and weights on a 3 x 3 map with -1 padding: the sums are C * [[-1, 3, -1], [3, 9, 3],
    [-1, 3, -1]] (a corner has 4 taps inside and 5 outside, an edge 6 and 3), whatever the oracle says.  With
    all-(-1) weights the signs flip.  Thresholds just below, at and above each value show every class of
    position taking the right side, which fixes sign and size of the term that stands for the taps the
    position-major tiles do not walk."""
    n, c, o = 32, 256, 64
    x = up(np.full((n, 9, c // 32), -1, dtype=np.int32), dev)                     # every bit set: +1
    pattern = np.array([-1, 3, -1, 3, 9, 3, -1, 3, -1]) * c
    desc = B.conv_desc(n, c, 3, 3, o, 3, 1, 1)
    for wsign in (1, -1):
        w = up(np.full((o, 9, c // 32), -1 if wsign > 0 else 0, dtype=np.int32), dev)
        values = sorted(set((wsign * pattern).tolist()))
        thr = np.array([v + d for v in values for d in (-1, 0, 1)] * 8, dtype=np.int32)[:o]
        out = Guarded(n * 9 * (o // 32), dev)
        B.check(B.bcnn_conv2d_binary_variant(desc, x, w, up(thr, dev), out.ptr, variant), "position-major conv")
        got = out.get().reshape(n, 9, o // 32)
        want_bits = (wsign * pattern)[:, None] >= thr[None, :]                    # [position][channel]
        want = np.zeros((9, o // 32), dtype=np.uint32)
        for ch in range(o):
            want[:, ch // 32] |= want_bits[:, ch].astype(np.uint32) << np.uint32(ch % 32)
        np.testing.assert_array_equal(got, np.broadcast_to(want, (n, 9, o // 32)))


def test_position_major_refusals(dev):
    """What the scheme does not cover is refused, not computed some other way."""
    dummy = torch.zeros(1 << 16, dtype=torch.int32, device=dev)
    for shape in [(31, 256, 7, 7, 64, 3, 1, 1), (32, 128, 7, 7, 64, 3, 1, 1), (32, 256, 7, 7, 64, 1, 1, 0),
                  (32, 256, 1, 1, 64, 3, 1, 1)]:
        n, c, h, wd, o, k, s, p = shape
        desc = B.conv_desc(n, c, h, wd, o, k, s, p)
        for variant in POS_VARIANTS:
            assert B.bcnn_conv2d_binary_variant(desc, dummy, dummy, dummy, dummy.data_ptr() + 4096, variant) == B.BCNN_ERR_UNSUPPORTED
    desc = B.conv_desc(32, 256, 7, 7, 64, 3, 1, 1)
    assert B.bcnn_conv2d_binary_variant(desc, dummy, dummy, None, dummy.data_ptr() + 4096,
                                        B.BCNN_VARIANT_MFMA_FP4_P6) == B.BCNN_ERR_UNSUPPORTED   # int32 sums


def test_threshold_extremes(dev):
    rng = np.random.default_rng(99)
    n, c, h, wd, o = 1, 64, 6, 6, 70
    x = rand_pm1(rng, (n, c, h, wd))
    w = rand_pm1(rng, (o, c, 3, 3))
    imin, imax = np.iinfo(np.int32).min, np.iinfo(np.int32).max
    thr = np.zeros(o, dtype=np.int32)
    thr[0::3] = imin
    thr[1::3] = imax
    _, want = oracle_fused(x, w, 1, 1, thr)
    got = gpu_conv(dev, x, w, 1, 1, thr=thr)
    np.testing.assert_array_equal(got, want)
    assert np.all(got[..., -1] >> (o % 32) == 0)  # tail bits of the last word are zero


@pytest.mark.parametrize("rows,c_out", [(1, 1), (50, 32), (777, 70), (4096, 256), (33, 1000), (9, 64)])
def test_standalone_epilogue_matches_oracle(dev, rows, c_out):
    rng = np.random.default_rng(rows + c_out)
    y = rng.integers(-300, 301, size=(rows, c_out)).astype(np.int32)
    thr = rng.integers(-100, 101, size=c_out).astype(np.int32)
    thr[0] = np.iinfo(np.int32).min
    thr[-1] = np.iinfo(np.int32).max if c_out > 1 else thr[-1]
    want = oracle.pack_channels(oracle.threshold_sign(y, thr).reshape(rows, c_out, 1))[:, 0, :]
    out = Guarded(want.size, dev)
    B.check(B.bcnn_threshold_sign_pack(up(y, dev), up(thr, dev), rows, c_out, out.ptr), "thr")
    np.testing.assert_array_equal(out.get().reshape(want.shape), want)


# ------------------------------------------------------------- layer chains
def _oracle_chain(x, ws, ts, stride, pad):
    """Oracle layer by layer: sums -> threshold sign -> next layer's +-1 input.
    Returns the packed output of every layer."""
    cur = x
    packed = []
    for w, t in zip(ws, ts):
        y = oracle.conv2d_pm1(cur, w, stride, pad)
        s = oracle.threshold_sign(y, t)                      # [n, ho, wo, o]
        n, ho, wo, o = s.shape
        packed.append(oracle.pack_channels(s.reshape(n, ho * wo, o).transpose(0, 2, 1)))
        cur = np.ascontiguousarray(s.transpose(0, 3, 1, 2))  # NCHW for the next layer
    return packed


def _gpu_chain(dev, cfg_n, c, h, wd, o, k, stride, pad, xp, wps, thrs, variant):
    """The packed output of every layer; each is the next layer's input on the device."""
    cur = xp
    hh, ww, cc = h, wd, c
    outs = []
    for wp, t in zip(wps, thrs):
        desc = B.conv_desc(cfg_n, cc, hh, ww, o, k, stride, pad)
        try:
            cur = B.conv2d_binary_sign_pack(desc, cur, wp, t, variant=variant)
        except B.BcnnError as e:
            if e.status == B.BCNN_ERR_UNSUPPORTED and variant not in COVER_ALL:
                pytest.skip("variant does not cover this shape")
            raise
        outs.append(cur)
        hh, ww = B.out_shape(desc)
        cc = o
    torch.cuda.synchronize()
    return outs


@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
def test_small_chain_packed_handoff(dev, variant):
    rng = np.random.default_rng(2024)
    n, c, h, wd = 5, 128, 7, 7
    x = rand_pm1(rng, (n, c, h, wd))
    ws = [rand_pm1(rng, (c, c, 3, 3)) for _ in range(3)]
    bound = int(2 * math.sqrt(c * 9))
    ts = [rng.integers(-bound, bound + 1, size=c).astype(np.int32) for _ in range(3)]
    want = _oracle_chain(x, ws, ts, 1, 1)
    xp = B.pack_nchw(up(x, dev))
    wps = [B.pack_nchw(up(w, dev)) for w in ws]
    got = _gpu_chain(dev, n, c, h, wd, c, 3, 1, 1, xp, wps, [up(t, dev) for t in ts], variant)
    for layer, (g, wnt) in enumerate(zip(got, want)):
        np.testing.assert_array_equal(g.cpu().numpy().view(np.uint32), wnt, err_msg="layer %d" % layer)


# ------------------------------------- the five benchmark shapes at full size
@functools.lru_cache(maxsize=None)
def _full_size_oracle(index):
    """The oracle on the whole batch of benchmark shape `index`, evaluated once
    per session and shared by every variant: packed input, packed weights, and
    either the int32 sums or the packed output of every layer of the chain."""
    cfg, x, ws, ts = W.make_inputs(index)
    want = {"x": oracle_pack_nchw(x), "w": [oracle_pack_weights(w) for w in ws]}
    if cfg.fused:
        want["layers"] = _oracle_chain(x, ws, ts, cfg.stride, cfg.pad)
    else:
        want["sums"] = oracle.conv2d_pm1(x, ws[0], cfg.stride, cfg.pad)
    return want


@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("index", [1, 2, 3, 4, 5])
def test_full_size_config_whole_tensor(dev, index, variant):
    """Full-size launch (the one the benchmark times) compared with the oracle
    on the whole output: every image, pixel and channel, after every layer of
    the chain.  Inputs are packed on the GPU from the real-valued tensor, so
    the packing kernel is covered at full size too."""
    cfg, x, ws, ts = W.make_inputs(index)
    want = _full_size_oracle(index)
    x_real = W.real_with_sign(W.seeds(index)[0], x)
    xp = B.pack_nchw(up(x_real, dev))                      # [n, h*w, cw]
    del x_real
    wps = [B.pack_nchw(up(w, dev)) for w in ws]
    assert np.array_equal(xp.cpu().numpy().view(np.uint32), want["x"]), "packed input"
    for wp, wnt in zip(wps, want["w"]):
        assert np.array_equal(wp.cpu().numpy().view(np.uint32), wnt), "packed weights"
    if cfg.fused:
        thr_dev = [up(t, dev) for t in ts]
        got = _gpu_chain(dev, cfg.n, cfg.c_in, cfg.h, cfg.w, cfg.c_out, cfg.k, cfg.stride, cfg.pad,
                         xp, wps, thr_dev, variant)
        assert len(got) == len(want["layers"]) == cfg.layers
        for layer, (g, wnt) in enumerate(zip(got, want["layers"])):
            assert np.array_equal(g.cpu().numpy().view(np.uint32), wnt), "packed output of layer %d" % layer
    else:
        desc = B.conv_desc(cfg.n, cfg.c_in, cfg.h, cfg.w, cfg.c_out, cfg.k, cfg.stride, cfg.pad)
        try:
            got = B.conv2d_binary(desc, xp, wps[0], variant=variant)
        except B.BcnnError as e:
            if e.status == B.BCNN_ERR_UNSUPPORTED and variant not in COVER_ALL:
                pytest.skip("variant does not cover this shape")
            raise
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), want["sums"]), "int32 sums"
