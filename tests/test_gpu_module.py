"""Parity of the convolution-module call (binary convolution, batch-norm scale
and bias, identity addition, PReLU, next module's bias and sign; paper, Section
4.2.1, first paragraph) with the CPU oracle on a real MI355X.

The library evaluates the real-valued part in float32 in a fixed order of
operations (fma, add, multiply, storage rounding), the same the oracle's float
result follows, so the real stream is compared for equality and the packed
bits bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2010_00704_amd import binding as B
from paper_2010_00704_amd import workloads as W
from gpu_helpers import (REAL_IDS, REAL_PARAMS, Guarded, gpu_device, i32, real_code, real_np_dtype, real_seed,
                         real_store, real_values, run_variant, up)

pytestmark = pytest.mark.gpu

VARIANTS = [B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU, B.BCNN_VARIANT_MFMA_FP4]
VARIANT_IDS = ["auto", "valu", "mfma_fp4"]


@pytest.fixture(scope="module")
def dev():
    return gpu_device()


def oracle_module(x, wt, stride, pad, g, b, ident, alpha, c, half):
    y = oracle.conv2d_pm1(x, wt, stride, pad)
    n, ho, wo, o = y.shape
    ident32 = None if ident is None else real_values(ident, half).reshape(y.shape)
    _, r32 = oracle.module_epilogue(y, g, b, ident32, alpha)
    stored = real_store(r32, half)
    cc = c if c is not None else np.zeros(o, dtype=np.float32)
    s = oracle.sign_bias_f32(real_values(stored, half).reshape(n * ho * wo, o, 1), cc)
    bits = oracle.pack_channels(s.reshape(n, ho * wo, o).transpose(0, 2, 1))
    return stored.reshape(n * ho * wo, o), bits


def make_params(seed, m, o, half, grid):
    if grid:   # quarters: exact float arithmetic, so r + c hits 0 exactly now and then
        g = W.uniform_f32(seed, (o,), -2.0, 2.0, steps=16)
        b = W.uniform_f32(seed + 1, (o,), -8.0, 8.0, steps=64)
        ident = W.uniform_f32(seed + 2, (m, o), -16.0, 16.0, steps=128)
        alpha = W.uniform_f32(seed + 3, (o,), 0.0, 1.0, steps=4)
        c = W.uniform_f32(seed + 4, (o,), -4.0, 4.0, steps=32)
    else:
        g = W.uniform_f32(seed, (o,), -1.5, 1.5)
        b = W.uniform_f32(seed + 1, (o,), -30.0, 30.0)
        ident = W.uniform_f32(seed + 2, (m, o), -40.0, 40.0)
        alpha = W.uniform_f32(seed + 3, (o,), 0.05, 0.5)
        c = W.uniform_f32(seed + 4, (o,), -10.0, 10.0)
    ident = real_store(ident, half)
    return g, b, ident, alpha, c


def gpu_module(dev, x, wt, stride, pad, g, b, ident, alpha, c, half, variant, want_r=True, want_bits=True,
               in_place=False):
    n, cin, h, w = x.shape
    o, _, k, _ = wt.shape
    desc = B.conv_desc(n, cin, h, w, o, k, stride, pad)
    ho, wo = B.out_shape(desc)
    m = n * ho * wo
    xp = up(i32(oracle.pack_channels(x.reshape(n, cin, -1))), dev)
    wp = up(i32(oracle.pack_channels(wt.reshape(o, cin, -1))), dev)
    esz = 2 if half else 4
    rbuf = Guarded.of_bytes(m * o * esz, dev)
    idt = None
    if ident is not None:
        if in_place:
            rbuf.put(ident)
            idt = rbuf.ptr
        else:
            idt = up(ident, dev)
    cwo = (o + 31) // 32
    bits = Guarded(m * cwo, dev)
    rc = B.bcnn_conv2d_binary_module(
        desc, xp, wp, up(g, dev), up(b, dev), idt, up(alpha, dev) if alpha is not None else None,
        up(c, dev) if c is not None else None, real_code(half),
        rbuf.ptr if want_r else None, bits.ptr if want_bits else None, variant)
    run_variant(rc, "module", variant)
    r = rbuf.get(real_np_dtype(half), m * o).reshape(m, o) if want_r else None
    xb = bits.get(np.uint32, m * cwo).reshape(n, ho * wo, cwo) if want_bits else None
    return r, xb


MODULE_SHAPES = [
    # n, c_in, h, w, c_out, k, stride, pad
    (2, 128, 24, 24, 128, 1, 1, 0),    # the paper's 1x1 module, matrix-core path
    (1, 256, 33, 31, 64, 1, 1, 0),
    (2, 128, 23, 23, 192, 3, 1, 1),
    (3, 256, 20, 20, 100, 3, 2, 1),    # ragged c_out on the matrix-core path
    (1, 128, 40, 40, 70, 1, 2, 0),
    (2, 64, 14, 14, 64, 1, 1, 0),      # vector-ALU path
    (3, 33, 9, 7, 40, 3, 1, 1),
    (1, 100, 12, 12, 7, 1, 1, 0),
    (40, 96, 14, 14, 96, 3, 1, 1),     # two pixels per lane on the vector-ALU path
]


@pytest.mark.parametrize("shape", MODULE_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("half", REAL_PARAMS, ids=REAL_IDS)
def test_module_matches_oracle(dev, shape, variant, half):
    n, cin, h, w, o, k, stride, pad = shape
    seed = 9500 + sum(v * q for v, q in zip(shape, (3, 5, 7, 11, 13, 17, 19, 23))) + real_seed(half)
    x = W.pm1(seed, (n, cin, h, w), 0.45)
    wt = W.pm1(seed + 1, (o, cin, k, k))
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    m = n * ho * wo
    for grid in (False, True):
        g, b, ident, alpha, c = make_params(seed + 10 + 100 * grid, m, o, half, grid)
        want_r, want_bits = oracle_module(x, wt, stride, pad, g, b, ident, alpha, c, half)
        r, bits = gpu_module(dev, x, wt, stride, pad, g, b, ident, alpha, c, half, variant)
        assert np.array_equal(r, want_r)
        assert np.array_equal(bits, want_bits)


@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("half", REAL_PARAMS, ids=REAL_IDS)
def test_module_optional_parts(dev, variant, half):
    shape = (2, 128, 24, 24, 128, 1, 1, 0) if variant != B.BCNN_VARIANT_VALU else (2, 64, 10, 10, 70, 3, 1, 1)
    n, cin, h, w, o, k, stride, pad = shape
    x = W.pm1(9901, (n, cin, h, w))
    wt = W.pm1(9902, (o, cin, k, k))
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    m = n * ho * wo
    g, b, ident, alpha, c = make_params(9903, m, o, half, True)
    # no identity, no activation, no next bias
    want_r, want_bits = oracle_module(x, wt, stride, pad, g, b, None, None, None, half)
    r, bits = gpu_module(dev, x, wt, stride, pad, g, b, None, None, None, half, variant)
    assert np.array_equal(r, want_r) and np.array_equal(bits, want_bits)
    # each output alone, and the stream updated in place
    want_r, want_bits = oracle_module(x, wt, stride, pad, g, b, ident, alpha, c, half)
    r, _ = gpu_module(dev, x, wt, stride, pad, g, b, ident, alpha, c, half, variant, want_bits=False)
    assert np.array_equal(r, want_r)
    _, bits = gpu_module(dev, x, wt, stride, pad, g, b, ident, alpha, c, half, variant, want_r=False)
    assert np.array_equal(bits, want_bits)
    r, bits = gpu_module(dev, x, wt, stride, pad, g, b, ident, alpha, c, half, variant, in_place=True)
    assert np.array_equal(r, want_r) and np.array_equal(bits, want_bits)


@pytest.mark.parametrize("level", W.TABLE1_MODULES, ids=lambda t: t[0])
@pytest.mark.parametrize("half", REAL_PARAMS, ids=REAL_IDS)
def test_module_table1_shapes(dev, level, half):
    """The 1x1 modules of the paper's network (Table 1), two images each."""
    _, ch, side = level
    n = 2
    seed = 9700 + ch + real_seed(half)
    x = W.pm1(seed, (n, ch, side, side), 0.5)
    wt = W.pm1(seed + 1, (ch, ch, 1, 1))
    m = n * side * side
    g, b, ident, alpha, c = make_params(seed + 2, m, ch, half, False)
    want_r, want_bits = oracle_module(x, wt, 1, 0, g, b, ident, alpha, c, half)
    r, bits = gpu_module(dev, x, wt, 1, 0, g, b, ident, alpha, c, half, B.BCNN_VARIANT_AUTO, in_place=True)
    assert np.array_equal(r, want_r)
    assert np.array_equal(bits, want_bits)


@pytest.mark.parametrize("shape", [(2, 128, 24, 24, 128, 1, 1, 0, 64), (1, 256, 30, 30, 192, 1, 1, 0, 48),
                                   (2, 64, 14, 14, 96, 1, 1, 0, 32), (3, 96, 9, 9, 70, 3, 1, 1, 35),
                                   (2, 128, 20, 20, 100, 1, 1, 0, 25)],
                         ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("half", REAL_PARAMS, ids=REAL_IDS)
def test_module_replicated_identity(dev, shape, variant, half):
    """Section 4.2.2: the identity stream keeps its channels and is replicated by
    bookkeeping; the oracle adds a real copy."""
    n, cin, h, w, o, k, stride, pad, idc = shape
    seed = 9800 + sum(v * q for v, q in zip(shape, (3, 5, 7, 11, 13, 17, 19, 23, 29))) + real_seed(half)
    x = W.pm1(seed, (n, cin, h, w), 0.5)
    wt = W.pm1(seed + 1, (o, cin, k, k))
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    m = n * ho * wo
    g, b, _, alpha, c = make_params(seed + 2, 1, o, half, False)
    ident = W.uniform_f32(seed + 9, (m, idc), -40.0, 40.0)
    ident = real_store(ident, half)
    rep = -(-o // idc)
    ident_full = oracle.replicate_channels(ident, rep, axis=1)[:, :o]
    want_r, want_bits = oracle_module(x, wt, stride, pad, g, b, ident_full, alpha, c, half)
    desc = B.conv_desc(n, cin, h, w, o, k, stride, pad)
    xp = up(i32(oracle.pack_channels(x.reshape(n, cin, -1))), dev)
    wp = up(i32(oracle.pack_channels(wt.reshape(o, cin, -1))), dev)
    rbuf = Guarded.of_bytes(m * o * (2 if half else 4), dev)
    cwo = (o + 31) // 32
    bits = Guarded(m * cwo, dev)
    rc = B.bcnn_conv2d_binary_module(desc, xp, wp, up(g, dev), up(b, dev), up(ident, dev), up(alpha, dev), up(c, dev),
                                     real_code(half), rbuf.ptr, bits.ptr, variant,
                                     identity_channels=idc)
    run_variant(rc, "module", variant)
    assert np.array_equal(rbuf.get(real_np_dtype(half), m * o).reshape(m, o), want_r)
    assert np.array_equal(bits.get(np.uint32, m * cwo).reshape(n, ho * wo, cwo), want_bits)


def test_module_argument_checks(dev):
    desc = B.conv_desc(1, 64, 8, 8, 32, 1, 1, 0)
    x = torch.zeros((64 * 2,), dtype=torch.int32, device=dev)
    w = torch.zeros((32 * 2,), dtype=torch.int32, device=dev)
    g = torch.ones((32,), dtype=torch.float32, device=dev)
    r = torch.zeros((64 * 32,), dtype=torch.float32, device=dev)
    bits = torch.zeros((64,), dtype=torch.int32, device=dev)
    f = B.bcnn_conv2d_binary_module
    assert f(desc, x, w, g, g, None, None, None, B.BCNN_F32, None, None) == B.BCNN_ERR_INVALID_ARG
    assert f(desc, x, w, None, g, None, None, None, B.BCNN_F32, r, bits) == B.BCNN_ERR_INVALID_ARG
    assert f(desc, x, w, g, g, None, None, None, B.BCNN_I8, r, bits) == B.BCNN_ERR_UNSUPPORTED
    assert f(desc, x, w, g, g, None, None, None, B.BCNN_F32, r, x) == B.BCNN_ERR_INVALID_ARG
    assert f(desc, x, w, g, g, None, None, None, B.BCNN_F32, r.data_ptr() + 2, bits) == B.BCNN_ERR_ALIGNMENT
    assert f(desc, x, w, g, g, None, None, None, B.BCNN_F32, r, bits, B.BCNN_VARIANT_MFMA_I8) == B.BCNN_ERR_UNSUPPORTED
    assert f(desc, x, w, g, g, None, None, None, B.BCNN_F32, r, bits) == B.BCNN_OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("half", REAL_PARAMS, ids=REAL_IDS)
def test_module_full_size_1x1(dev, half):
    """The 1x1 benchmark shape as the paper's module (256 -> 256 channels, 56x56,
    batch 32, identity path included), launched at full size and compared with
    the oracle on the whole real stream and all packed words."""
    cfg = W.CONFIGS[1]
    _, x_all, ws, _ = W.make_inputs(2)
    wt = ws[0]
    hw = cfg.h * cfg.w
    m = cfg.n * hw
    g, b, _, alpha, c = make_params(9950, 1, cfg.c_out, half, False)
    ident = W.uniform_f32(9960, (m, cfg.c_out), -40.0, 40.0)
    ident = real_store(ident, half)
    desc = B.conv_desc(cfg.n, cfg.c_in, cfg.h, cfg.w, cfg.c_out, cfg.k, cfg.stride, cfg.pad)
    xp = B.pack_nchw(up(x_all, dev))
    wp = B.pack_nchw(up(wt, dev))
    stream_t = up(ident, dev)                 # updated in place
    bits = torch.empty((cfg.n, hw, cfg.c_out // 32), dtype=torch.int32, device=dev)
    B.check(B.bcnn_conv2d_binary_module(desc, xp, wp, up(g, dev), up(b, dev), stream_t, up(alpha, dev), up(c, dev),
                                        real_code(half), stream_t, bits), "module")
    torch.cuda.synchronize()
    got_r = stream_t.cpu().numpy().reshape(m, cfg.c_out)
    got_bits = bits.cpu().numpy().view(np.uint32)
    want_r, want_bits = oracle_module(x_all, wt, cfg.stride, cfg.pad, g, b, ident, alpha, c, half)
    assert np.array_equal(got_r, want_r)
    assert np.array_equal(got_bits, want_bits)


@pytest.mark.parametrize("variant", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("half", REAL_PARAMS, ids=REAL_IDS)
def test_module_special_values(dev, variant, half):
    """Signed zeros, denormals, the largest finite values and infinities in the
    identity stream, a next bias that holds -0 and cancels stored values exactly:
    the float chain keeps them as the oracle does (denormals are not flushed, a
    value too large for half becomes an infinity, the tie r + c = 0 gives bit 1).
    Slopes stay positive and no term is infinite on both sides, so no NaN arises:
    a NaN's payload is the one thing the two sides need not agree on."""
    shape = (2, 128, 24, 24, 128, 1, 1, 0) if variant != B.BCNN_VARIANT_VALU else (2, 64, 12, 12, 64, 1, 1, 0)
    n, cin, h, w, o, k, stride, pad = shape
    x = W.pm1(9970, (n, cin, h, w))
    wt = W.pm1(9971, (o, cin, k, k))
    m = n * h * w
    g, b, _, alpha, c = make_params(9972, m, o, half, True)
    alpha = np.maximum(alpha, np.float32(0.25))
    if half == "bf16":
        # zero, smallest subnormals (2^-133), largest subnormal, smallest normal, largest finite, infinities
        special = real_store(np.array([0.0, -0.0, 9.2e-41, -9.2e-41, 1.166e-38, 1.1754944e-38, np.inf, -np.inf,
                                       3.3895314e38, -3.3895314e38, 1.0, -2.5, 65504.0], dtype=np.float32), half)
    elif half:
        special = np.array([0.0, -0.0, 6e-8, -6e-8, 6.1e-5, -6.1e-5, np.inf, -np.inf, 65504.0, -65504.0, 1.0, -2.5],
                           dtype=np.float16)
    else:
        special = np.array([0.0, -0.0, 1e-45, -1e-45, 1.1754942e-38, -1.1754942e-38, 1.17549435e-38, np.inf,
                            -np.inf, 3.4e38, -3.4e38, 65504.0, 1e-8, -2.5], dtype=np.float32)
    pick = (W.raw_u64(9973, 0, m * o) % np.uint64(len(special))).astype(np.int64)
    ident = special[pick].reshape(m, o)
    c = c.copy()
    c[0::7] = np.float32(-0.0)
    with np.errstate(over="ignore"):          # values too large for half become infinities, on purpose
        want_r, want_bits = oracle_module(x, wt, stride, pad, g, b, ident, alpha, c, half)
    assert not np.any(np.isnan(real_values(want_r, half)))      # no NaN in play
    # a bias that cancels what the first row stores, so that r + c is exactly zero there
    c2 = c.copy()
    fin = np.isfinite(real_values(want_r[0], half))
    c2[fin] = -real_values(want_r[0], half)[fin]
    for cc in (c, c2):
        with np.errstate(over="ignore"):
            want_r, want_bits = oracle_module(x, wt, stride, pad, g, b, ident, alpha, cc, half)
        r, bits = gpu_module(dev, x, wt, stride, pad, g, b, ident, alpha, cc, half, variant)
        view = np.uint16 if half else np.uint32
        assert np.array_equal(r.view(view), want_r.view(view))            # bit patterns: -0 is not +0
        assert np.array_equal(bits, want_bits)
