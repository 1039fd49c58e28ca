"""Pins for the oracle of the convolution module's real-valued epilogue (paper,
Section 4.2.1, first paragraph: batch norm, identity addition, PReLU, then the
next module's bias and sign).  CPU only; checks ``oracle.module_epilogue``
against hand-worked values, library operators, the integer-threshold form of
the identity-free chain and exactly rounded rational arithmetic.
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "module_hand_worked.json")


def _golden():
    with open(GOLDEN) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _golden(), ids=lambda c: c["name"])
def test_hand_worked_module_epilogue(case):
    y = np.array(case["y"], dtype=np.int32)
    ident = None if case["identity"] is None else np.array(case["identity"], dtype=np.float32)
    r64, r32 = oracle.module_epilogue(y, case["g"], case["b"], ident, case["a"])
    want = np.array(case["r"], dtype=np.float64)
    assert np.array_equal(r64, want) and np.array_equal(r32.astype(np.float64), want)
    bits = oracle.sign_bias_f32(r32.reshape(y.shape[0], y.shape[1], 1), np.array(case["c"], dtype=np.float32))
    assert np.array_equal(bits[:, :, 0], np.array(case["bits"], dtype=np.int8))


def _random_case(seed, rows=40, o=24, with_identity=True):
    rng = np.random.default_rng(seed)
    y = rng.integers(-300, 301, size=(rows, o)).astype(np.int32)
    g = rng.normal(size=o).astype(np.float32)
    b = rng.normal(scale=30, size=o).astype(np.float32)
    ident = rng.normal(scale=50, size=(rows, o)).astype(np.float32) if with_identity else None
    a = rng.uniform(0.05, 0.5, size=o).astype(np.float32)
    return y, g, b, ident, a


def test_against_library_operators():
    """scale*y + bias, + identity, torch's prelu, all in float64."""
    y, g, b, ident, a = _random_case(1)
    r64, r32 = oracle.module_epilogue(y, g, b, ident, a)
    t = torch.from_numpy(y.astype(np.float64)) * torch.from_numpy(g.astype(np.float64)) + \
        torch.from_numpy(b.astype(np.float64)) + torch.from_numpy(ident.astype(np.float64))
    want = F.prelu(t.T.unsqueeze(0), torch.from_numpy(a.astype(np.float64))).squeeze(0).T.numpy()
    assert np.allclose(r64, want, rtol=0, atol=1e-10)
    # the float result: three roundings (fma, add, multiply), each half an ulp of a value no larger than mag
    mag = np.abs(g.astype(np.float64) * y) + np.abs(b.astype(np.float64)) + np.abs(ident.astype(np.float64))
    assert np.all(np.abs(r32 - r64) <= 3 * 2.0**-24 * mag)
    assert np.abs(r32 - r64).max() > 0


def _round_to_f32(q):
    c = np.float32(float(q))
    cands = [c, np.nextafter(c, np.float32(-np.inf)), np.nextafter(c, np.float32(np.inf))]
    dist = [abs(Fraction(float(v)) - q) for v in cands]
    best = min(dist)
    winners = [v for v, d in zip(cands, dist) if d == best]
    if len(winners) > 1:
        winners = [v for v in winners if (v.view(np.uint32) & 1) == 0]
    return winners[0]


def test_float_result_is_three_correct_roundings():
    y, g, b, ident, a = _random_case(2, rows=6, o=8)
    _, r32 = oracle.module_epilogue(y, g, b, ident, a)
    for m in range(y.shape[0]):
        for o in range(y.shape[1]):
            t = _round_to_f32(Fraction(float(g[o])) * int(y[m, o]) + Fraction(float(b[o])))
            t = _round_to_f32(Fraction(float(t)) + Fraction(float(ident[m, o])))
            if not t >= 0:
                t = _round_to_f32(Fraction(float(a[o])) * Fraction(float(t)))
            assert float(t) == float(r32[m, o])


def test_identity_free_chain_is_an_integer_threshold():
    """sign(g*y + b) = (y >= ceil(-b/g)) for g > 0 and (y <= floor(-b/g)) for
    g < 0: the form the fused integer epilogue uses.  Scales and biases are
    binary fractions so that the float evaluation is exact."""
    rng = np.random.default_rng(3)
    o = 16
    y = rng.integers(-40, 41, size=(200, o)).astype(np.int32)
    g = (rng.integers(1, 9, size=o) / 4.0 * rng.choice([-1, 1], size=o)).astype(np.float32)
    b = (rng.integers(-64, 65, size=o) / 8.0).astype(np.float32)
    _, r32 = oracle.module_epilogue(y, g, b, None, None)
    bits = oracle.sign_f32(r32)
    for ch in range(o):
        q = Fraction(-float(b[ch])) / Fraction(float(g[ch]))
        if g[ch] > 0:
            thr = math.ceil(q)
            want = oracle.threshold_sign(y[:, ch:ch + 1], np.array([thr], dtype=np.int32))[:, 0]
        else:
            thr = math.floor(q)
            # y <= thr  <=>  -y >= -thr: the same threshold routine on the negated sums
            want = oracle.threshold_sign(-y[:, ch:ch + 1], np.array([-thr], dtype=np.int32))[:, 0]
        assert np.array_equal(bits[:, ch], want)


def test_special_cases():
    y, g, b, ident, a = _random_case(4)
    r64, r32 = oracle.module_epilogue(y, g, b, ident, a)
    # slope 1 is no activation at all
    r64_1, r32_1 = oracle.module_epilogue(y, g, b, ident, np.ones_like(a))
    r64_n, r32_n = oracle.module_epilogue(y, g, b, ident, None)
    assert np.array_equal(r32_1, r32_n) and np.array_equal(r64_1, r64_n)
    # non-negative pre-activations pass unchanged, negative ones are scaled
    assert np.array_equal(r32[r32_n >= 0], r32_n[r32_n >= 0])
    neg = r32_n < 0
    assert neg.any() and np.array_equal(r32[neg], (np.broadcast_to(a, r32.shape)[neg] * r32_n[neg]).astype(np.float32))
    # zero identity is no identity
    _, r32_z = oracle.module_epilogue(y, g, b, np.zeros_like(ident), a)
    _, r32_0 = oracle.module_epilogue(y, g, b, None, a)
    assert np.array_equal(r32_z, r32_0)
    # the sums enter linearly: unit scale, zero bias, no identity, no activation returns them
    _, r32_y = oracle.module_epilogue(y, np.ones_like(g), np.zeros_like(b), None, None)
    assert np.array_equal(r32_y, y.astype(np.float32))


def test_channel_replication_is_a_plain_copy():
    """Channel k = j*C + c of the replicated tensor is channel c (checked with
    explicit loops), on either layout used by the tests."""
    rng = np.random.default_rng(7)
    x = rng.normal(size=(2, 5, 3)).astype(np.float32)          # [outer, C, inner]
    y = oracle.replicate_channels(x, 3)
    assert y.shape == (2, 15, 3)
    for a in range(2):
        for k in range(15):
            for i in range(3):
                assert y[a, k, i] == x[a, k % 5, i]
    rows = rng.normal(size=(4, 6)).astype(np.float32)          # [rows, C]
    z = oracle.replicate_channels(rows, 2, axis=1)
    assert z.shape == (4, 12) and all(z[m, k] == rows[m, k % 6] for m in range(4) for k in range(12))
    assert np.array_equal(oracle.replicate_channels(x, 1), x)
    with pytest.raises(ValueError):
        oracle.replicate_channels(x, 0)


def test_module_tail_continues_the_batch_norm_output():
    """Identity addition and PReLU applied to a given sum z: fed with the
    batch-norm output itself it must reproduce the whole epilogue; library
    prelu in double; hand-worked values of M1 with z = g*y + b."""
    y, g, b, ident, a = _random_case(5)
    t64, t32 = oracle.module_epilogue(y, g, b, None, None)          # batch norm alone
    want64, want32 = oracle.module_epilogue(y, g, b, ident, a)
    r64, r32 = oracle.module_tail(t64, t32, ident, a)
    assert np.array_equal(r32, want32) and np.array_equal(r64, want64)
    tt = torch.from_numpy(t64) + torch.from_numpy(ident.astype(np.float64))
    lib = F.prelu(tt.T.unsqueeze(0), torch.from_numpy(a.astype(np.float64))).squeeze(0).T.numpy()
    assert np.allclose(r64, lib, rtol=0, atol=1e-12)
    case = _golden()[0]
    z = np.array(case["g"]) * np.array(case["y"], dtype=np.float64) + np.array(case["b"])   # exact binary fractions
    r64, r32 = oracle.module_tail(z, z.astype(np.float32), np.array(case["identity"], dtype=np.float32), case["a"])
    assert np.array_equal(r64, np.array(case["r"])) and np.array_equal(r32, np.array(case["r"], dtype=np.float32))
    # no identity, no slope: z passes through
    r64, r32 = oracle.module_tail(t64, t32, None, None)
    assert np.array_equal(r32, t32) and np.array_equal(r64, t64)
