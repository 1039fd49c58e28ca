"""Pins of the CPU oracle against things other than itself (no GPU).

The oracle (oracle/bcnn_oracle.c) is the definition of the binary CNN-style 2D
convolution written as nested loops.  Each test here compares it with an
independent source of truth: hand-worked values (tests/golden), a brute-force
float evaluation on an explicitly padded tensor, torch's convolution, an
integer matrix product, the xor/popcount identity, closed forms, invariants.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")


def _signs(spec, shape):
    """'+-+/-+-' style strings (or nested lists of them) -> int8 +-1 array."""
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
def test_hand_worked_convolutions(case):
    x = _signs(case["x"], [1] + case["x_shape"])
    w = _signs(case["w"], case["w_shape"])
    y = oracle.conv2d_pm1(x, w, case["stride"], case["pad"])
    assert y.shape[0] == 1
    np.testing.assert_array_equal(y[0], np.array(case["y"], dtype=np.int32))


@pytest.mark.parametrize("case", _golden()["pack_cases"], ids=lambda c: c["name"])
def test_hand_worked_packing(case):
    s = -np.ones((1, case["channels"], 1), dtype=np.int8)
    s[0, case["plus_channels"], 0] = 1
    words = oracle.pack_channels(s)
    assert words.dtype == np.uint32
    np.testing.assert_array_equal(words[0, 0], np.array(case["words"], dtype=np.uint32))


@pytest.mark.parametrize("case", _golden()["threshold_cases"], ids=lambda c: c["name"])
def test_hand_worked_threshold(case):
    y = np.array([case["y"]], dtype=np.int32)
    s = oracle.threshold_sign(y, np.array(case["thr"], dtype=np.int32))
    np.testing.assert_array_equal(s[0], np.array(case["signs"], dtype=np.int8))
    word = oracle.pack_channels(s.reshape(1, -1, 1))
    assert int(word[0, 0, 0]) == case["word"]


# ------------------------------------------------- brute force, float, padded
def _brute_float(x, w, stride, pad):
    """Textbook double sum in float64 on a tensor that is physically padded
    with -1, pure Python loops over outputs (tiny shapes only)."""
    n, c, h, wd = x.shape
    o, _, kh, kw = w.shape
    xp = -np.ones((n, c, h + 2 * pad, wd + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + h, pad:pad + wd] = x
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    y = np.zeros((n, ho, wo, o), dtype=np.float64)
    wf = w.astype(np.float64)
    for a in range(n):
        for i in range(ho):
            for j in range(wo):
                patch = xp[a, :, i * stride:i * stride + kh, j * stride:j * stride + kw]
                for q in range(o):
                    y[a, i, j, q] = float((patch * wf[q]).sum())
    return y


@pytest.mark.parametrize("shape", [
    # n, c, h, w, o, k, stride, pad
    (2, 3, 5, 4, 4, 3, 1, 1), (1, 5, 6, 7, 3, 3, 2, 1), (2, 4, 3, 3, 2, 3, 1, 0),
    (1, 7, 4, 5, 5, 1, 1, 0), (1, 2, 5, 5, 3, 1, 2, 0), (1, 3, 1, 1, 2, 3, 1, 1),
    (1, 1, 2, 2, 1, 3, 2, 1), (2, 33, 4, 3, 3, 3, 2, 1), (1, 2, 7, 5, 2, 3, 2, 0),
])
def test_against_brute_force_float(shape):
    n, c, h, wd, o, k, s, p = shape
    rng = np.random.default_rng(hash(shape) % (1 << 32))
    x = _rand_pm1(rng, (n, c, h, wd), 0.4)
    w = _rand_pm1(rng, (o, c, k, k))
    y = oracle.conv2d_pm1(x, w, s, p)
    ref = _brute_float(x, w, s, p)
    assert y.shape == ref.shape
    np.testing.assert_array_equal(y.astype(np.float64), ref)


# ------------------------------------------------------------ library routines
@pytest.mark.parametrize("shape", [
    (2, 64, 14, 14, 32, 3, 1, 1), (1, 40, 9, 11, 17, 3, 2, 1), (2, 96, 8, 8, 24, 1, 1, 0),
    (1, 16, 13, 10, 8, 1, 2, 0), (1, 8, 6, 6, 4, 3, 1, 0),
])
def test_against_torch_conv2d(shape):
    """F.conv2d on +-1 floats with a -1 border equals the oracle exactly
    (all partial sums are small integers, exact in float32)."""
    n, c, h, wd, o, k, s, p = shape
    rng = np.random.default_rng(7 + sum(shape))
    x = _rand_pm1(rng, (n, c, h, wd), 0.3)
    w = _rand_pm1(rng, (o, c, k, k))
    xt = torch.from_numpy(x.astype(np.float32))
    xt = torch.nn.functional.pad(xt, (p, p, p, p), value=-1.0)
    ref = torch.nn.functional.conv2d(xt, torch.from_numpy(w.astype(np.float32)), stride=s)
    ref = ref.permute(0, 2, 3, 1).numpy()  # NCHW -> NHWC
    y = oracle.conv2d_pm1(x, w, s, p)
    np.testing.assert_array_equal(y, ref.astype(np.int32))
    assert np.all(ref == np.round(ref))


def test_1x1_is_integer_matrix_product():
    """The lowering to a matrix product: for a 1x1 filter, Y[M,O] = A[M,K] W[O,K]^T."""
    rng = np.random.default_rng(11)
    n, c, h, wd, o = 3, 70, 5, 6, 19
    x = _rand_pm1(rng, (n, c, h, wd))
    w = _rand_pm1(rng, (o, c, 1, 1))
    a = x.transpose(0, 2, 3, 1).reshape(n * h * wd, c).astype(np.int64)
    ref = a @ w.reshape(o, c).astype(np.int64).T
    y = oracle.conv2d_pm1(x, w, 1, 0).reshape(n * h * wd, o)
    np.testing.assert_array_equal(y, ref)


# ------------------------------------------------------- xor/popcount identity
def test_dot_equals_k_minus_twice_popcount_of_xor():
    """sum a_i b_i = K - 2 popcount(bits(a) xor bits(b)) for +-1 vectors: the
    oracle's sum (as a 1x1 convolution of one pixel) against the identity
    evaluated with Python integers on the oracle-independent bit strings."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        k = int(rng.integers(1, 301))
        a = _rand_pm1(rng, (k,), rng.random())
        b = _rand_pm1(rng, (k,))
        y = int(oracle.conv2d_pm1(a.reshape(1, k, 1, 1), b.reshape(1, k, 1, 1), 1, 0)[0, 0, 0, 0])
        abits = sum(1 << i for i in range(k) if a[i] > 0)
        bbits = sum(1 << i for i in range(k) if b[i] > 0)
        assert y == k - 2 * bin(abits ^ bbits).count("1")
        # and through the oracle's own packing: same identity on packed words
        pa = oracle.pack_channels(a.reshape(1, k, 1))[0, 0]
        pb = oracle.pack_channels(b.reshape(1, k, 1))[0, 0]
        pop = sum(bin(int(u) ^ int(v)).count("1") for u, v in zip(pa, pb))
        assert y == k - 2 * pop


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("k,s,p", [(1, 1, 0), (3, 1, 0), (3, 2, 0), (3, 1, 1), (3, 2, 1)])
def test_closed_forms_and_invariants(k, s, p):
    rng = np.random.default_rng(100 + 10 * k + 3 * s + p)
    n, c, h, wd, o = 2, 12, 7, 6, 5
    kk = c * k * k
    ones_x = np.ones((n, c, h, wd), dtype=np.int8)
    ones_w = np.ones((o, c, k, k), dtype=np.int8)
    y = oracle.conv2d_pm1(ones_x, ones_w, s, p)
    if p == 0:
        assert np.all(y == kk)  # every tap real: K
    else:
        # interior outputs see only real taps; a corner output of a 3x3 window sees 4 real, 5 padded
        assert y[0, 0, 0, 0] == c * (4 - 5)
        assert y.max() == kk
    x = _rand_pm1(rng, (n, c, h, wd), 0.35)
    w = _rand_pm1(rng, (o, c, k, k))
    y = oracle.conv2d_pm1(x, w, s, p)
    assert np.all(np.abs(y) <= kk)
    assert np.all((y - kk) % 2 == 0)  # y = K - 2*mismatches
    np.testing.assert_array_equal(oracle.conv2d_pm1(x, -w, s, p), -y)  # odd in w, padding or not
    if p == 0:
        np.testing.assert_array_equal(oracle.conv2d_pm1(-x, w, s, p), -y)  # odd in x without padding
    # channel replication R times on both operands multiplies the sum by R
    y3 = oracle.conv2d_pm1(np.tile(x, (1, 3, 1, 1)), np.tile(w, (1, 3, 1, 1)), s, p)
    np.testing.assert_array_equal(y3, 3 * y)
    # images are independent
    np.testing.assert_array_equal(oracle.conv2d_pm1(x[1:], w, s, p), y[1:])
    # output extent
    assert y.shape == (n, (h + 2 * p - k) // s + 1, (wd + 2 * p - k) // s + 1, o)
    assert oracle.out_dim(h, k, s, p) == y.shape[1]


def test_padding_equals_minus_sum_of_weights():
    """A padded tap contributes -sum_c w: y(-1 pad) = y(0 pad) - sum of the
    weights under padded taps; checked at the (0,0) corner of a 3x3 window."""
    rng = np.random.default_rng(3)
    c, o = 9, 4
    x = _rand_pm1(rng, (1, c, 5, 5))
    w = _rand_pm1(rng, (o, c, 3, 3))
    y = oracle.conv2d_pm1(x, w, 1, 1)
    xf = torch.from_numpy(x.astype(np.float32))
    zero_pad = torch.nn.functional.conv2d(xf, torch.from_numpy(w.astype(np.float32)), padding=1)
    zero_pad = zero_pad.permute(0, 2, 3, 1).numpy().astype(np.int64)
    w64 = w.astype(np.int64)
    corner_pad_taps = w64[:, :, 0, :].sum(axis=(1, 2)) + w64[:, :, 1:, 0].sum(axis=(1, 2))
    np.testing.assert_array_equal(y[0, 0, 0], zero_pad[0, 0, 0] - corner_pad_taps)


def test_single_output_entry_matches_full_tensor():
    rng = np.random.default_rng(17)
    x = _rand_pm1(rng, (2, 10, 6, 7))
    w = _rand_pm1(rng, (6, 10, 3, 3))
    y = oracle.conv2d_pm1(x, w, 2, 1)
    idx = np.array([(a, i, j, q) for a in range(2) for i in range(y.shape[1])
                    for j in range(y.shape[2]) for q in range(6)], dtype=np.int32)
    got = oracle.conv2d_pm1_at(x, w, idx, 2, 1)
    np.testing.assert_array_equal(got, y.reshape(-1))
    # and the brute-force float pin applies to it directly
    ref = _brute_float(x, w, 2, 1).reshape(-1)
    np.testing.assert_array_equal(got.astype(np.float64), ref)
    with pytest.raises(ValueError):
        oracle.conv2d_pm1_at(x, w, np.array([[0, 99, 0, 0]], dtype=np.int32), 2, 1)


# ------------------------------------------------------------- sign, threshold
def test_sign_of_special_values():
    x = np.array([0.0, -0.0, 1e-45, -1e-45, np.inf, -np.inf, np.nan, 3.5, -2.0], dtype=np.float32)
    np.testing.assert_array_equal(oracle.sign_f32(x), np.array([1, 1, 1, -1, 1, -1, -1, 1, -1], dtype=np.int8))


def test_threshold_extremes_and_monotonicity():
    rng = np.random.default_rng(23)
    y = rng.integers(-50, 51, size=(40, 37)).astype(np.int32)
    lo = np.full(37, np.iinfo(np.int32).min, dtype=np.int32)
    hi = np.full(37, np.iinfo(np.int32).max, dtype=np.int32)
    assert np.all(oracle.threshold_sign(y, lo) == 1)
    assert np.all(oracle.threshold_sign(y, hi) == -1)
    t1 = rng.integers(-20, 21, size=37).astype(np.int32)
    s1 = oracle.threshold_sign(y, t1)
    s2 = oracle.threshold_sign(y, t1 + 5)
    assert np.all(s2 <= s1)  # raising a threshold can only turn +1 into -1
    np.testing.assert_array_equal(s1, np.where(y >= t1[None, :], 1, -1))
    # packed form: tail bits of the last word stay zero even when every bit is on
    words = oracle.pack_channels(oracle.threshold_sign(y, lo).reshape(40, 37, 1))
    assert np.all(words[:, 0, 0] == 0xFFFFFFFF) and np.all(words[:, 0, 1] == 0x1F)


# ------------------------------------------------------------------- packing
@pytest.mark.parametrize("c", [1, 31, 32, 33, 64, 65])
@pytest.mark.parametrize("inner", [1, 5])
def test_pack_roundtrip_and_bit_positions(c, inner):
    rng = np.random.default_rng(c * 10 + inner)
    s = _rand_pm1(rng, (3, c, inner))
    p = oracle.pack_channels(s)
    assert p.shape == (3, inner, (c + 31) // 32)
    np.testing.assert_array_equal(oracle.unpack_channels(p, c), s)
    # independent bit extraction with Python integers
    for a in range(3):
        for i in range(inner):
            for ch in range(c):
                bit = (int(p[a, i, ch // 32]) >> (ch % 32)) & 1
                assert bit == (1 if s[a, ch, i] > 0 else 0)
            if c % 32:
                assert int(p[a, i, -1]) >> (c % 32) == 0  # tail bits are zero


def test_pack_matches_numpy_packbits():
    """LSB-first 32-bit words on a little-endian host are numpy's
    packbits(bitorder='little') bytes."""
    rng = np.random.default_rng(29)
    s = _rand_pm1(rng, (4, 96, 7))
    p = oracle.pack_channels(s)
    bits = (s.transpose(0, 2, 1) > 0).astype(np.uint8)  # [outer, inner, C]
    ref = np.packbits(bits, axis=-1, bitorder="little").view("<u4")
    np.testing.assert_array_equal(p, ref.reshape(p.shape))
