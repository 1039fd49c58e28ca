"""The calls chained the way the paper's network uses them (Section 4.2: binary
1x1 convolution modules on a real stream with identity connections, spatial
down-sampling by average pooling on the identity path, channel increase by
replication), packed bits and the real stream handed from call to call on the
device, against the same chain built from the oracle's pieces on the CPU.

  real stream a0 [n, h, w, C], half precision, updated in place
  x0 = pack(sign(a0 + b0))                                   bcnn_pack_bias, channel-last source
  a1, x1 = module(x0, W1; identity a0; next bias b1)         bcnn_conv2d_binary_module, in place
  a2, x2 = module(x1, W2; identity a1; next bias b2)         in place again
  p, xp  = avgpool2x2(a2), pack(sign(p + bp))                bcnn_avgpool_bias_sign_pack
  xr     = pack(sign(replicate(p, R) + br))                  bcnn_pack_bias_replicated
  a3, x3 = module(xr, W3: R*C -> R*C; identity replicate(p)) identity_channels = C
Every intermediate is compared bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2010_00704_amd import binding as B
from paper_2010_00704_amd import workloads as W
from gpu_helpers import Guarded, gpu_device, i32, up

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    return gpu_device()


def bits_of_rows(real_rows, bias):
    """[m, c] real -> packed [m, cw] of sign(real + bias) through the oracle."""
    m, c = real_rows.shape
    s = oracle.sign_bias_f32(real_rows.astype(np.float32).reshape(m, c, 1), bias)
    return oracle.pack_channels(s.reshape(m, c, 1))[:, 0, :], s[:, :, 0]


def oracle_module_rows(sign_rows, n, h, w, wt, g, b, identity_rows, alpha, next_bias):
    """One 1x1 module on channel-last rows: signs [m, c] -> (stream as stored in half, next bits, next signs)."""
    m, c = sign_rows.shape
    x = sign_rows.reshape(n, h, w, c).transpose(0, 3, 1, 2)
    y = oracle.conv2d_pm1(x, wt, 1, 0)                                   # [n, h, w, o]
    o = wt.shape[0]
    _, r32 = oracle.module_epilogue(y, g, b, identity_rows.astype(np.float32).reshape(n, h, w, o), alpha)
    stored = oracle.store_f16(r32).reshape(m, o)
    bits, signs = bits_of_rows(stored, next_bias)
    return stored, bits, signs


CHAINS = [
    # n, h, w, C, replication
    (2, 8, 8, 64, 2),
    (3, 14, 14, 128, 2),
    (1, 12, 10, 96, 3),
    (1, 9, 7, 100, 2),         # odd map, ragged last word
    (8, 56, 56, 256, 2),       # large enough for the matrix-core module kernels
]


@pytest.mark.parametrize("shape", CHAINS, ids=lambda s: "x".join(map(str, s)))
def test_block_chain(dev, shape):
    n, h, w, c, rep = shape
    seed = 30000 + 17 * c + h
    m = n * h * w
    par = lambda k, shp, lo, hi: W.uniform_f32(seed + k, shp, lo, hi)      # noqa: E731
    a0 = oracle.store_f16(par(0, (m, c), -30.0, 30.0))
    b0, b1, b2 = par(1, (c,), -5.0, 5.0), par(2, (c,), -5.0, 5.0), par(3, (c,), -5.0, 5.0)
    w1, w2 = W.pm1(seed + 4, (c, c, 1, 1)), W.pm1(seed + 5, (c, c, 1, 1))
    g1, g2 = par(6, (c,), -0.2, 0.2), par(7, (c,), -0.2, 0.2)
    be1, be2 = par(8, (c,), -3.0, 3.0), par(9, (c,), -3.0, 3.0)
    al1, al2 = par(10, (c,), 0.05, 0.5), par(11, (c,), 0.05, 0.5)
    cr = rep * c
    bp, br, b3 = par(12, (c,), -5.0, 5.0), par(13, (cr,), -5.0, 5.0), par(14, (cr,), -5.0, 5.0)
    w3 = W.pm1(seed + 15, (cr, cr, 1, 1))
    g3, be3, al3 = par(16, (cr,), -0.2, 0.2), par(17, (cr,), -3.0, 3.0), par(18, (cr,), 0.05, 0.5)

    # ---- the oracle's chain
    want_x0, s0 = bits_of_rows(a0, b0)
    want_a1, want_x1, s1 = oracle_module_rows(s0, n, h, w, w1, g1, be1, a0, al1, b1)
    want_a2, want_x2, _ = oracle_module_rows(s1, n, h, w, w2, g2, be2, want_a1, al2, b2)
    _, p32 = oracle.avgpool_nhwc(want_a2.astype(np.float32).reshape(n, h, w, c), 2)
    ho, wo = h // 2, w // 2
    mp = n * ho * wo
    want_p = oracle.store_f16(p32).reshape(mp, c)
    want_xp, _ = bits_of_rows(want_p, bp)
    p_rep = oracle.replicate_channels(want_p, rep, axis=1)
    want_xr, sr = bits_of_rows(p_rep, br)
    want_a3, want_x3, _ = oracle_module_rows(sr, n, ho, wo, w3, g3, be3, p_rep, al3, b3)

    # ---- the same on the GPU, buffers handed from call to call
    cw, cwr = (c + 31) // 32, (cr + 31) // 32
    stream = Guarded.of_bytes(m * c * 2, dev)
    stream.put(a0)
    x0, x1, x2 = Guarded(m * cw, dev), Guarded(m * cw, dev), Guarded(m * cw, dev)
    pooled, xp = Guarded.of_bytes(mp * c * 2, dev), Guarded(mp * cw, dev)
    xr, x3 = Guarded(mp * cwr, dev), Guarded(mp * cwr, dev)
    a3 = Guarded.of_bytes(mp * cr * 2, dev)
    wp1 = up(i32(oracle.pack_channels(w1.reshape(c, c, 1))), dev)
    wp2 = up(i32(oracle.pack_channels(w2.reshape(c, c, 1))), dev)
    wp3 = up(i32(oracle.pack_channels(w3.reshape(cr, cr, 1))), dev)
    d12 = B.conv_desc(n, c, h, w, c, 1, 1, 0)
    d3 = B.conv_desc(n, cr, ho, wo, cr, 1, 1, 0)
    H = B.BCNN_F16
    B.check(B.bcnn_pack_bias(stream.ptr, H, m, c, 1, up(b0, dev), x0.ptr), "pack_bias")
    B.check(B.bcnn_conv2d_binary_module(d12, x0.ptr, wp1, up(g1, dev), up(be1, dev), stream.ptr, up(al1, dev),
                                        up(b1, dev), H, stream.ptr, x1.ptr), "module 1")
    torch.cuda.synchronize()
    got_a1 = stream.get(np.float16, m * c).reshape(m, c).copy()
    B.check(B.bcnn_conv2d_binary_module(d12, x1.ptr, wp2, up(g2, dev), up(be2, dev), stream.ptr, up(al2, dev),
                                        up(b2, dev), H, stream.ptr, x2.ptr), "module 2")
    B.check(B.bcnn_avgpool_bias_sign_pack(stream.ptr, H, n, h, w, c, 2, up(bp, dev), pooled.ptr, xp.ptr), "avgpool")
    B.check(B.bcnn_pack_bias_replicated(pooled.ptr, H, mp, c, 1, rep, up(br, dev), xr.ptr), "pack_bias_replicated")
    B.check(B.bcnn_conv2d_binary_module(d3, xr.ptr, wp3, up(g3, dev), up(be3, dev), pooled.ptr, up(al3, dev),
                                        up(b3, dev), H, a3.ptr, x3.ptr, identity_channels=c), "module 3")

    assert np.array_equal(x0.get(np.uint32).reshape(m, cw), want_x0), "first binarisation"
    assert np.array_equal(got_a1, want_a1), "stream after module 1"
    assert np.array_equal(x1.get(np.uint32).reshape(m, cw), want_x1), "bits after module 1"
    assert np.array_equal(stream.get(np.float16, m * c).reshape(m, c), want_a2), "stream after module 2"
    assert np.array_equal(x2.get(np.uint32).reshape(m, cw), want_x2), "bits after module 2"
    assert np.array_equal(pooled.get(np.float16, mp * c).reshape(mp, c), want_p), "pooled stream"
    assert np.array_equal(xp.get(np.uint32).reshape(mp, cw), want_xp), "bits of the pooled stream"
    assert np.array_equal(xr.get(np.uint32).reshape(mp, cwr), want_xr), "bits of the replicated stream"
    assert np.array_equal(a3.get(np.float16, mp * cr).reshape(mp, cr), want_a3), "stream after the wider module"
    assert np.array_equal(x3.get(np.uint32).reshape(mp, cwr), want_x3), "bits after the wider module"
