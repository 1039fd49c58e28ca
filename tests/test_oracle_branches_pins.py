"""Pins for the oracle of the F x F = F*F shifted 1x1 branches construction
(paper, Section 4.2.1, last paragraph; Figure 2, bottom).  Everything here runs
on the CPU and checks ``oracle.branches_*`` / ``oracle.sign_bias_f32`` against
things other than themselves: hand-worked values, a library real-valued
convolution, the plain binary-convolution definition, closed forms and the
floating-point error bound of the float chain.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "branches_hand_worked.json")


def _signs(spec, shape):
    flat = []

    def walk(v):
        if isinstance(v, str):
            flat.extend(1 if ch == "+" else -1 for ch in v if ch in "+-")
        else:
            for e in v:
                walk(e)
    walk(spec)
    return np.array(flat, dtype=np.int8).reshape(shape)


def _golden():
    with open(GOLDEN) as f:
        return json.load(f)


def _rand_pm1(rng, shape, p=0.5):
    return np.where(rng.random(shape) < p, 1, -1).astype(np.int8)


# ---------------------------------------------------------------- hand-worked
@pytest.mark.parametrize("case", _golden()["cases"], ids=lambda c: c["name"])
def test_hand_worked_branches(case):
    b, c, h, w = case["xb_shape"]
    xb = _signs(case["xb"], (b, 1, c, h, w))
    wt = _signs(case["w"], case["w_shape"])
    z64, z32 = oracle.branches_pm1(xb, np.array(case["padv"], dtype=np.int8), wt,
                                   np.array(case["g"], dtype=np.float32),
                                   np.array(case["h"], dtype=np.float32),
                                   case["stride"], case["pad"])
    want = np.array(case["z"], dtype=np.float64)[None]
    # every value in the file is exactly representable and every partial sum too
    assert np.array_equal(z64, want)
    assert np.array_equal(z32.astype(np.float64), want)


@pytest.mark.parametrize("case", _golden()["real_cases"], ids=lambda c: c["name"])
def test_hand_worked_from_real_tensor(case):
    a = np.array(case["a"], dtype=np.float32)[None]
    wt = _signs(case["w"], case["w_shape"])
    z = oracle.branches_real(a, np.array(case["b"], dtype=np.float32), wt,
                             np.array(case["g"], dtype=np.float32),
                             np.array(case["h"], dtype=np.float32), case["stride"], case["pad"])
    assert np.array_equal(z, np.array(case["z"], dtype=np.float64)[None])


# ------------------------------------------------- against a library real conv
def _padded(x, padv, pad):
    """[N,C,H,W] +-1 -> float64 tensor with a border of padv[c] of width pad."""
    n, c, h, w = x.shape
    out = np.empty((n, c, h + 2 * pad, w + 2 * pad), dtype=np.float64)
    out[:] = padv.astype(np.float64)[None, :, None, None]
    out[:, :, pad:pad + h, pad:pad + w] = x
    return out


@pytest.mark.parametrize("shape", [(2, 5, 6, 7, 4, 3, 1, 1), (1, 33, 5, 5, 3, 3, 2, 1),
                                   (2, 8, 4, 6, 5, 3, 1, 0), (1, 3, 7, 4, 2, 3, 2, 0),
                                   (3, 6, 3, 3, 4, 1, 1, 0), (2, 4, 5, 5, 3, 1, 2, 0)])
@pytest.mark.parametrize("shared", [True, False])
def test_against_real_valued_library_convolution(shape, shared):
    """sum_t g_t[o] * (1x1 binary conv of branch t) is a real convolution whose
    filter is g[t][o] * w[o][c][u][v]; with one tensor per branch it is the sum
    over t of convolutions with a filter that is zero except at tap t."""
    n, c, h, w, o, f, stride, pad = shape
    p = f * f
    rng = np.random.default_rng(hash(shape) % 2**32 + shared)
    xb = _rand_pm1(rng, (1 if shared else p, n, c, h, w))
    padv = _rand_pm1(rng, (p, c))
    if shared:
        padv[:] = padv[0]            # one border value per channel, so one padded tensor serves all taps
    wt = _rand_pm1(rng, (o, c, f, f))
    g = rng.normal(size=(p, o)).astype(np.float32)
    hb = rng.normal(size=(o,)).astype(np.float32)
    z64, z32 = oracle.branches_pm1(xb, padv, wt, g, hb, stride, pad)

    want = torch.zeros((n, o, z64.shape[1], z64.shape[2]), dtype=torch.float64)
    for t in range(p):
        filt = torch.zeros((o, c, f, f), dtype=torch.float64)
        u, v = divmod(t, f)
        filt[:, :, u, v] = torch.from_numpy(wt[:, :, u, v].astype(np.float64)) * \
            torch.from_numpy(g[t].astype(np.float64))[:, None]
        src = torch.from_numpy(_padded(xb[0 if shared else t], padv[t], pad))
        want += F.conv2d(src, filt, stride=stride)
    want += torch.from_numpy(hb.astype(np.float64))[None, :, None, None]
    want = want.permute(0, 2, 3, 1).numpy()
    assert np.allclose(z64, want, rtol=0, atol=1e-9)
    assert np.allclose(z32, want, rtol=0, atol=1e-3)


def test_zero_contribution_padding_is_library_zero_padding():
    rng = np.random.default_rng(5)
    n, c, h, w, o, f = 2, 7, 5, 6, 3, 3
    x = _rand_pm1(rng, (1, n, c, h, w))
    wt = _rand_pm1(rng, (o, c, f, f))
    g = rng.normal(size=(9, o)).astype(np.float32)
    z64, _ = oracle.branches_pm1(x, np.zeros((9, c), dtype=np.int8), wt, g, None, 1, 1)
    filt = torch.from_numpy(wt.astype(np.float64)) * \
        torch.from_numpy(g.astype(np.float64).T.reshape(o, 1, f, f))
    want = F.conv2d(torch.from_numpy(x[0].astype(np.float64)), filt, stride=1, padding=1)
    assert np.allclose(z64, want.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-9)


# ------------------------------------------- reduction to the plain binary conv
@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
def test_unit_scales_reduce_to_the_plain_binary_convolution(stride, pad):
    """All g = 1, h = 0, padded taps -1: z is the integer binary convolution."""
    rng = np.random.default_rng(11 + stride + pad)
    n, c, h, w, o = 2, 40, 6, 5, 6
    x = _rand_pm1(rng, (n, c, h, w))
    wt = _rand_pm1(rng, (o, c, 3, 3))
    y = oracle.conv2d_pm1(x, wt, stride, pad)
    z64, z32, yt = oracle.branches_pm1(x[None], -np.ones((9, c), dtype=np.int8), wt,
                                       np.ones((9, o), dtype=np.float32), None, stride, pad, taps=True)
    assert np.array_equal(z64, y.astype(np.float64))
    assert np.array_equal(z32, y.astype(np.float32))
    assert np.array_equal(yt.sum(axis=-1), y)
    assert np.abs(yt).max() <= c and np.all((yt - c) % 2 == 0)


def test_taps_are_1x1_integer_matrix_products():
    """Each branch is a 1x1 binary convolution: an integer matrix product of
    the shifted pixels with that tap's weight slice."""
    rng = np.random.default_rng(3)
    n, c, h, w, o = 1, 9, 4, 4, 5
    xb = _rand_pm1(rng, (9, n, c, h, w))
    padv = _rand_pm1(rng, (9, c))
    wt = _rand_pm1(rng, (o, c, 3, 3))
    _, _, yt = oracle.branches_pm1(xb, padv, wt, np.ones((9, o), dtype=np.float32), None, 1, 1, taps=True)
    for t in range(9):
        u, v = divmod(t, 3)
        for oh in range(h):
            for ow in range(w):
                ih, iw = oh - 1 + u, ow - 1 + v
                pix = xb[t, 0, :, ih, iw] if (0 <= ih < h and 0 <= iw < w) else padv[t]
                want = wt[:, :, u, v].astype(np.int64) @ pix.astype(np.int64)
                assert np.array_equal(yt[0, oh, ow, :, t], want)


def test_literal_evaluation_equals_the_binarised_one():
    """sign(shifted + b_t) per branch, zero fill before the bias: the literal
    evaluation from the real tensor equals the evaluation on sign_bias outputs
    with padded value sign(b_t[c])."""
    rng = np.random.default_rng(17)
    n, c, h, w, o = 2, 6, 5, 4, 3
    a = rng.normal(size=(n, c, h, w)).astype(np.float32)
    b = rng.normal(scale=0.7, size=(9, c)).astype(np.float32)
    b[2, 1] = 0.0                     # sign(0 + 0) = +1 at the border
    wt = _rand_pm1(rng, (o, c, 3, 3))
    g = rng.normal(size=(9, o)).astype(np.float32)
    hh = rng.normal(size=(9, o)).astype(np.float32)
    for stride in (1, 2):
        z_real = oracle.branches_real(a, b, wt, g, hh, stride, 1)
        xb = np.stack([oracle.sign_bias_f32(a.reshape(n, c, h * w), b[t]).reshape(n, c, h, w)
                       for t in range(9)])
        padv = np.where(b >= 0, 1, -1).astype(np.int8)
        z64, _ = oracle.branches_pm1(xb, padv, wt, g, None, stride, 1)
        assert np.allclose(z_real, z64 + hh.astype(np.float64).sum(axis=0), rtol=0, atol=1e-9)


@pytest.mark.parametrize("p,stride", [(2, 1), (3, 2), (5, 1)])
def test_parallel_branches_are_a_1x1_convolution_over_concatenated_channels(p, stride):
    """P parallel 1x1 branches with unit scales: the branch tensors stacked
    along the channel axis, convolved with the branch filters stacked the same
    way (the plain binary convolution, pinned elsewhere); with real scales, a
    library real-valued 1x1 convolution over the same stack."""
    rng = np.random.default_rng(41 + p)
    n, c, h, w, o = 2, 9, 5, 4, 6
    xb = _rand_pm1(rng, (p, n, c, h, w))
    wt = _rand_pm1(rng, (o, c, p))
    padv = -np.ones((p, c), dtype=np.int8)
    x_cat = np.concatenate([xb[t] for t in range(p)], axis=1)                 # [n, p*c, h, w]
    w_cat = np.concatenate([wt[:, :, t] for t in range(p)], axis=1)[:, :, None, None]
    y = oracle.conv2d_pm1(x_cat, w_cat, stride, 0)
    z64, z32, yt = oracle.branches_pm1(xb, padv, wt, np.ones((p, o), dtype=np.float32), None, stride, 0, taps=True)
    assert np.array_equal(z64, y.astype(np.float64)) and np.array_equal(z32, y.astype(np.float32))
    assert yt.shape[-1] == p and np.array_equal(yt.sum(-1), y)
    g = rng.normal(size=(p, o)).astype(np.float32)
    hb = rng.normal(size=(o,)).astype(np.float32)
    z64, _ = oracle.branches_pm1(xb, padv, wt, g, hb, stride, 0)
    filt = np.concatenate([wt[:, :, t] * g[t].astype(np.float64)[:, None] for t in range(p)], axis=1)
    want = F.conv2d(torch.from_numpy(x_cat.astype(np.float64)), torch.from_numpy(filt)[:, :, None, None],
                    stride=stride) + torch.from_numpy(hb.astype(np.float64))[None, :, None, None]
    assert np.allclose(z64, want.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-9)
    # a shared tensor: every branch reads the same pixels
    zs, _ = oracle.branches_pm1(xb[:1], padv, wt, g, hb, stride, 0)
    zr, _ = oracle.branches_pm1(np.repeat(xb[:1], p, axis=0), padv, wt, g, hb, stride, 0)
    assert np.array_equal(zs, zr)


def test_branch_count_must_fit_the_filter():
    x = np.ones((1, 1, 2, 4, 4), dtype=np.int8)
    with pytest.raises(ValueError):
        oracle.branches_pm1(x, np.ones((9, 2), dtype=np.int8), np.ones((3, 2, 3, 3), dtype=np.int8),
                            np.ones((8, 3), dtype=np.float32))


# ----------------------------------------------------------- closed forms
def test_closed_forms():
    rng = np.random.default_rng(23)
    n, c, h, w, o = 1, 12, 4, 5, 4
    x = _rand_pm1(rng, (1, n, c, h, w))
    wt = _rand_pm1(rng, (o, c, 3, 3))
    padv = _rand_pm1(rng, (9, c))
    g = rng.normal(size=(9, o)).astype(np.float32)
    hb = rng.normal(size=(o,)).astype(np.float32)
    z, _ = oracle.branches_pm1(x, padv, wt, g, hb, 1, 1)
    # linear in g: doubling every scale doubles z - h (exact, powers of two)
    z2, _ = oracle.branches_pm1(x, padv, wt, 2 * g, hb, 1, 1)
    assert np.array_equal(z2 - hb.astype(np.float64), 2 * (z - hb.astype(np.float64)))
    # odd in the weights
    zn, _ = oracle.branches_pm1(x, padv, -wt, g, hb, 1, 1)
    assert np.allclose(zn - hb.astype(np.float64), -(z - hb.astype(np.float64)), rtol=0, atol=1e-12)
    # odd in (inputs, padded values) jointly
    zi, _ = oracle.branches_pm1(-x, -padv, wt, g, hb, 1, 1)
    assert np.allclose(zi - hb.astype(np.float64), -(z - hb.astype(np.float64)), rtol=0, atol=1e-12)
    # a branch with zero scale does not matter, whatever its tensor holds
    g0 = g.copy()
    g0[4] = 0
    xb = np.repeat(x, 9, axis=0)
    za, _ = oracle.branches_pm1(xb, padv, wt, g0, hb, 1, 1)
    xb[4] = -xb[4]
    zb, _ = oracle.branches_pm1(xb, padv, wt, g0, hb, 1, 1)
    assert np.array_equal(za, zb)
    # all +1 operands and padded values, no stride: z = C * sum_t g_t + h
    ones = np.ones((1, n, c, h, w), dtype=np.int8)
    zc, _ = oracle.branches_pm1(ones, np.ones((9, c), dtype=np.int8), np.ones((o, c, 3, 3), dtype=np.int8),
                                g, hb, 1, 1)
    want = c * g.astype(np.float64).sum(axis=0) + hb.astype(np.float64)
    assert np.allclose(zc, np.broadcast_to(want, zc.shape), rtol=0, atol=1e-9)


def test_float_chain_stays_within_its_rounding_bound():
    """The float evaluation is h, then one fused multiply-add per branch; each
    of the P roundings is at most half an ulp of a partial sum, and no partial
    sum exceeds |h| + sum_t |g_t y_t|."""
    rng = np.random.default_rng(29)
    n, c, h, w, o = 2, 200, 6, 6, 8
    x = _rand_pm1(rng, (1, n, c, h, w), p=0.3)
    wt = _rand_pm1(rng, (o, c, 3, 3))
    padv = _rand_pm1(rng, (9, c))
    g = rng.normal(size=(9, o)).astype(np.float32)
    hb = rng.normal(scale=20, size=(o,)).astype(np.float32)
    z64, z32, yt = oracle.branches_pm1(x, padv, wt, g, hb, 1, 1, taps=True)
    mag = np.abs(hb.astype(np.float64)) + (np.abs(g.astype(np.float64)).T[None, None, None] * np.abs(yt)).sum(-1)
    assert np.all(np.abs(z32.astype(np.float64) - z64) <= 9 * 2.0**-24 * mag)
    assert np.abs(z32.astype(np.float64) - z64).max() > 0      # and it is a float chain, not the double sum
    # the chain itself, redone in exact rational arithmetic with one correct rounding per step
    for idx in [(0, 0, 0, 0), (1, 3, 5, 7), (0, 2, 2, 3), (1, 5, 0, 4)]:
        acc = np.float32(hb[idx[3]])
        for t in range(9):
            acc = _round_to_f32(Fraction(float(g[t, idx[3]])) * int(yt[idx][t]) + Fraction(float(acc)))
        assert float(acc) == float(z32[idx])


def _round_to_f32(q):
    """Nearest float32 to the rational q (ties to even mantissa)."""
    c = np.float32(float(q))
    cands = [c, np.nextafter(c, np.float32(-np.inf)), np.nextafter(c, np.float32(np.inf))]
    dist = [abs(Fraction(float(v)) - q) for v in cands]
    best = min(dist)
    winners = [v for v, d in zip(cands, dist) if d == best]
    if len(winners) > 1:
        winners = [v for v in winners if (v.view(np.uint32) & 1) == 0]
    return winners[0]


# ------------------------------------------------------------- bias-then-sign
def test_sign_bias_is_the_exact_sign_of_the_sum():
    """Rounding a float sum never changes its sign or makes a non-zero sum
    zero, so sign(fl(x + b)) must equal the sign of the exact sum."""
    rng = np.random.default_rng(31)
    x = rng.normal(size=(3, 5, 11)).astype(np.float32)
    b = rng.normal(size=(5,)).astype(np.float32)
    x[0, 1, 3] = -b[1]                # exact cancellation -> +1
    x[1, 2, 0] = np.nextafter(-b[2], np.float32(-np.inf), dtype=np.float32)   # just below -> -1
    x[2, 0, 5] = np.nan
    x[2, 4, 1] = 1e-45                # denormal
    b[3] = 0.0
    x[0, 3, 0] = -0.0
    s = oracle.sign_bias_f32(x, b)
    exact = x.astype(np.float64) + b.astype(np.float64)[None, :, None]
    want = np.where(exact >= 0, 1, -1)
    assert np.array_equal(s, want)
    assert s[0, 1, 3] == 1 and s[1, 2, 0] == -1 and s[2, 0, 5] == -1 and s[0, 3, 0] == 1
    # zero bias is the plain sign
    assert np.array_equal(oracle.sign_bias_f32(x, np.zeros(5, dtype=np.float32)), oracle.sign_f32(x))
