"""GPU parity of bcnn_avgpool_bias_sign_pack (paper, Section 4.2.3: the average
pooling on the identity path of a down-sampling block, fused with the bias +
sign + pack of the binary 1x1 module behind it) against the CPU oracle, bit for
bit on the pooled real map and on the packed bits.
"""
import numpy as np
import pytest

import oracle
from paper_2010_00704_amd import binding as B
from paper_2010_00704_amd import workloads as W
from gpu_helpers import (REAL_IDS, REAL_PARAMS, Guarded, gpu_device, oracle_bits_of_sign, real_code, real_np_dtype,
                         real_store, real_values, up)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    return gpu_device()


def expected(src, s, bias, half):
    """Oracle side: the float chain, the value as stored, bias + sign, packed."""
    _, p32 = oracle.avgpool_nhwc(real_values(src, half), s)
    stored = real_store(p32, half)
    n, ho, wo, c = stored.shape
    b = np.zeros(c, dtype=np.float32) if bias is None else bias
    sgn = oracle.sign_bias_f32(real_values(stored, half).reshape(n * ho * wo, c, 1), b)
    return stored, oracle_bits_of_sign(sgn.reshape(n, ho, wo, c))


def source(seed, shape, half):
    # a few magnitudes so that additions round, and exact zeros so that the tie of the sign shows up
    a = W.uniform_f32(seed, shape, -40.0, 40.0, steps=320)
    a = a * np.where(W.uniform_f32(seed + 1, shape, 0.0, 1.0) < 0.2, np.float32(1e-3), np.float32(1.0))
    return real_store(a.astype(np.float32), half)


def run(dev, src, s, bias, half, want_pooled=True, want_bits=True, misalign=0):
    n, h, w, c = src.shape
    ho, wo = h // s, w // s
    esz = 2 if half else 4
    stored, bits = expected(src, s, bias, half)
    src_buf = Guarded.of_bytes(src.size * esz + 64, dev)
    raw = np.zeros(src.size * esz + misalign * esz, dtype=np.uint8)
    raw[misalign * esz:] = src.view(np.uint8).reshape(-1)
    src_buf.put(raw)
    out = Guarded.of_bytes(stored.size * esz, dev)
    pk = Guarded(bits.size, dev)
    rc = B.bcnn_avgpool_bias_sign_pack(src_buf.ptr + misalign * esz, real_code(half), n, h, w, c, s,
                                       None if bias is None else up(bias, dev),
                                       out.ptr if want_pooled else None, pk.ptr if want_bits else None)
    B.check(rc, "avgpool")
    if want_pooled:
        got = out.get(real_np_dtype(half), stored.size).reshape(stored.shape)
        assert np.array_equal(got, stored)
    if want_bits:
        assert np.array_equal(pk.get(np.uint32).reshape(bits.shape), bits)
    assert (ho, wo) == stored.shape[1:3]


SHAPES = [
    # n, h, w, c, s
    (2, 8, 8, 32, 2),          # one word, one DPP group per pixel
    (1, 14, 14, 64, 2),
    (3, 9, 11, 96, 2),         # odd sizes: last row and column dropped
    (2, 12, 12, 100, 2),       # channels a multiple of 4, ragged last word
    (2, 6, 6, 4, 2),           # one live lane per group
    (1, 9, 9, 36, 3),
    (1, 16, 12, 64, 4),
    (1, 10, 10, 40, 5),        # run-time window size
    (2, 7, 7, 33, 2),          # channels not a multiple of 4: the ballot kernel
    (1, 6, 9, 1, 3),
    (1, 8, 8, 130, 2),
    (2, 5, 5, 64, 1),          # S = 1: bias + sign + pack of the map itself
    (1, 2, 2, 256, 2),         # a single output pixel
]


@pytest.mark.parametrize("half", REAL_PARAMS, ids=REAL_IDS)
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_avgpool_bias_sign_pack(dev, shape, half):
    n, h, w, c, s = shape
    src = source(21000 + 7 * c + s, (n, h, w, c), half)
    bias = W.uniform_f32(21500 + c, (c,), -10.0, 10.0)
    run(dev, src, s, bias, half)


@pytest.mark.parametrize("half", REAL_PARAMS, ids=REAL_IDS)
def test_optional_arguments_and_alignment(dev, half):
    src = source(22000, (2, 8, 10, 64), half)
    bias = W.uniform_f32(22001, (64,), -10.0, 10.0)
    run(dev, src, 2, None, half)                          # no bias: the sign of the pooled value
    run(dev, src, 2, bias, half, want_pooled=False)       # bits only
    run(dev, src, 2, bias, half, want_bits=False)         # real map only
    run(dev, src, 2, bias, half, misalign=1)              # rows not vector aligned: the ballot kernel


def test_sign_of_exact_zero_and_ties(dev):
    """A window that sums to zero gives +0 and bit 1 without bias; a bias that
    cancels the pooled value exactly gives bit 1, one ulp below gives 0."""
    src = np.zeros((1, 2, 4, 32), dtype=np.float32)
    src[0, :, 0:2, :] = np.array([[1.5, -1.5], [2.25, -2.25]], dtype=np.float32)[:, :, None]
    src[0, :, 2:4, :] = 3.0
    bias = np.full(32, -3.0, dtype=np.float32)
    bias[1::2] = np.nextafter(np.float32(-3.0), np.float32(-4.0))
    run(dev, src, 2, None, False)
    run(dev, src, 2, bias, False)
    stored, bits = expected(src, 2, bias, False)
    assert np.all(stored[0, 0, 0] == 0.0) and np.all(stored[0, 0, 1] == 3.0)
    assert bits[0, 1, 0] == 0x55555555 and bits[0, 0, 0] == 0


@pytest.mark.parametrize("level,half", [("level1", True), ("level2", True), ("level3", False), ("level2", "bf16")])
def test_table1_transitions_full_size(dev, level, half):
    """The down-sampling steps of the paper's Table 1 at batch 32 (map sizes
    112 -> 56 -> 28 -> 14 with the channel counts of the level that is left),
    whole tensors compared."""
    c, hw = {"level1": (64, 112), "level2": (128, 56), "level3": (256, 28)}[level]
    src = source(23000 + c, (32, hw, hw, c), half)
    bias = W.uniform_f32(23500 + c, (c,), -10.0, 10.0)
    run(dev, src, 2, bias, half)


def test_rejects_bad_arguments(dev):
    src = up(np.zeros((1, 4, 4, 8), dtype=np.float32), dev)
    out = up(np.zeros((1, 2, 2, 8), dtype=np.float32), dev)
    bits = up(np.zeros((1, 2, 2, 1), dtype=np.int32), dev)
    f = B.bcnn_avgpool_bias_sign_pack
    assert f(None, B.BCNN_F32, 1, 4, 4, 8, 2, None, out, bits) == B.BCNN_ERR_INVALID_ARG
    assert f(src, B.BCNN_F32, 1, 4, 4, 8, 2, None, None, None) == B.BCNN_ERR_INVALID_ARG
    assert f(src, B.BCNN_F32, 1, 4, 4, 8, 0, None, out, bits) == B.BCNN_ERR_INVALID_ARG
    assert f(src, B.BCNN_F32, 1, 4, 4, 8, 5, None, out, bits) == B.BCNN_ERR_INVALID_ARG      # empty pooled map
    assert f(src, B.BCNN_F32, 1, 64, 64, 8, 9, None, out, bits) == B.BCNN_ERR_UNSUPPORTED
    assert f(src, B.BCNN_I8, 1, 4, 4, 8, 2, None, out, bits) == B.BCNN_ERR_UNSUPPORTED
    assert f(src, B.BCNN_F32, 1, 4, 4, 8, 2, None, src, bits) == B.BCNN_ERR_INVALID_ARG       # in place
    assert f(src, B.BCNN_F32, 1, 4, 4, 8, 2, None, out.data_ptr() + 2, bits) == B.BCNN_ERR_ALIGNMENT
