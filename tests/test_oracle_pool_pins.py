"""Pins for the oracle of the average pooling on the identity path of a
down-sampling block (paper, Section 4.2.3).  CPU only; checks
``oracle.avgpool_nhwc`` against hand-worked values, library pooling, a reshape
+ mean, exactly rounded rational arithmetic and closed forms.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pool_hand_worked.json")


def _golden():
    with open(GOLDEN) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _golden(), ids=lambda c: c["name"])
def test_hand_worked_pooling(case):
    a = np.array(case["a"], dtype=np.float32)
    p64, p32 = oracle.avgpool_nhwc(a, case["s"])
    want = np.array(case["p"], dtype=np.float64)
    assert p64.shape == want.shape and np.array_equal(p64, want)
    chain = np.array(case.get("p_float_chain", case["p"]), dtype=np.float32)
    assert np.array_equal(p32, chain)
    if "bias" in case:
        n, ho, wo, c = p32.shape
        bits = oracle.sign_bias_f32(p32.reshape(n * ho * wo, c, 1), np.array(case["bias"], dtype=np.float32))
        assert np.array_equal(bits.reshape(n, ho, wo, c), np.array(case["bits"], dtype=np.int8))


def _random_map(seed, shape):
    rng = np.random.default_rng(seed)
    return (rng.normal(scale=20.0, size=shape) * rng.choice([1.0, 1e-3, 1e3], size=shape)).astype(np.float32)


@pytest.mark.parametrize("shape,s", [((2, 8, 6, 5), 2), ((1, 9, 12, 3), 3), ((3, 7, 9, 4), 2), ((1, 11, 5, 2), 4),
                                     ((2, 5, 5, 7), 5)])
def test_against_library_pooling(shape, s):
    """torch's avg_pool2d in float64 on the channel-first view; its default
    (no padding, floor) drops incomplete windows as the oracle does."""
    a = _random_map(10 + s, shape)
    p64, p32 = oracle.avgpool_nhwc(a, s)
    lib = F.avg_pool2d(torch.from_numpy(a.astype(np.float64)).permute(0, 3, 1, 2), kernel_size=s, stride=s)
    lib = lib.permute(0, 2, 3, 1).numpy()
    assert p64.shape == lib.shape == (shape[0], shape[1] // s, shape[2] // s, shape[3])
    scale = np.abs(a).max()
    assert np.allclose(p64, lib, rtol=0, atol=1e-13 * scale)
    # the float chain: s*s - 1 additions and one division, each within half an ulp of a value <= sum |x|
    n, h, w, c = shape
    ho, wo = h // s, w // s
    mag = np.abs(a[:, :ho * s, :wo * s].astype(np.float64)).reshape(n, ho, s, wo, s, c).sum(axis=(2, 4))
    assert np.all(np.abs(p32 - p64) <= 2.0**-24 * mag)
    assert np.abs(p32 - p64).max() > 0


def test_against_reshape_and_mean():
    a = _random_map(20, (2, 6, 10, 3))
    p64, _ = oracle.avgpool_nhwc(a, 2)
    want = a.astype(np.float64).reshape(2, 3, 2, 5, 2, 3).mean(axis=(2, 4))
    assert np.allclose(p64, want, rtol=1e-14, atol=0)


def _round_to_f32(q):
    c = np.float32(float(q))
    cands = [c, np.nextafter(c, np.float32(-np.inf)), np.nextafter(c, np.float32(np.inf))]
    dist = [abs(Fraction(float(v)) - q) for v in cands]
    best = min(dist)
    winners = [v for v, d in zip(cands, dist) if d == best]
    if len(winners) > 1:
        winners = [v for v in winners if (v.view(np.uint32) & 1) == 0]
    return winners[0]


@pytest.mark.parametrize("s", [2, 3])
def test_float_chain_is_raster_order_with_one_rounding_per_step(s):
    a = _random_map(30 + s, (1, 2 * s, 3 * s, 2))
    _, p32 = oracle.avgpool_nhwc(a, s)
    for oh in range(2):
        for ow in range(3):
            for c in range(2):
                acc = None
                for u in range(s):
                    for v in range(s):
                        x = Fraction(float(a[0, oh * s + u, ow * s + v, c]))
                        acc = x if acc is None else Fraction(float(_round_to_f32(acc + x)))
                want = _round_to_f32(acc / (s * s))
                assert float(want) == float(p32[0, oh, ow, c])


def test_closed_forms():
    a = _random_map(40, (2, 8, 8, 6))
    p64, p32 = oracle.avgpool_nhwc(a, 2)
    # S = 1 is no pooling at all
    q64, q32 = oracle.avgpool_nhwc(a, 1)
    assert np.array_equal(q32, a) and np.array_equal(q64, a.astype(np.float64))
    # a constant map stays constant (any window size; 2.5 * 9 and 2.5 * 16 are exact)
    for s in (2, 3, 4):
        c64, c32 = oracle.avgpool_nhwc(np.full((1, 12, 12, 3), 2.5, dtype=np.float32), s)
        assert np.all(c64 == 2.5) and np.all(c32 == 2.5)
    # scaling by a power of two and negation commute with every rounding
    d64, d32 = oracle.avgpool_nhwc(-4.0 * a, 2)
    assert np.array_equal(d32, -4.0 * p32) and np.array_equal(d64, -4.0 * p64)
    # pooling twice by 2 is pooling once by 4 in exact arithmetic
    r64, _ = oracle.avgpool_nhwc(a, 4)
    h64, _ = oracle.avgpool_nhwc(a.astype(np.float64).astype(np.float32), 2)
    twice = h64.reshape(2, 2, 2, 2, 2, 6).mean(axis=(2, 4))
    assert np.allclose(r64, twice, rtol=1e-12, atol=1e-12)
    # one bright pixel per window: the mean is that pixel / S^2, whichever corner holds it
    for u in range(2):
        for v in range(2):
            z = np.zeros((1, 4, 4, 1), dtype=np.float32)
            z[0, u::2, v::2, 0] = 8.0
            o64, o32 = oracle.avgpool_nhwc(z, 2)
            assert np.all(o64 == 2.0) and np.all(o32 == 2.0)


def test_bad_arguments():
    a = np.zeros((1, 3, 3, 2), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.avgpool_nhwc(a, 0)
    with pytest.raises(ValueError):
        oracle.avgpool_nhwc(a, 4)
    with pytest.raises(ValueError):
        oracle.avgpool_nhwc(a[0], 1)
