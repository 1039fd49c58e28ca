"""Pins for the oracle's 16-bit storage rounding of the real stream
(``oracle.store_f16``, ``oracle.store_bf16``, ``oracle.load_bf16``): hand-worked
codes incl. ties, subnormals, overflow and special values, the conversions of
three independent libraries (numpy's float16 cast, Python's struct format "e",
torch's bfloat16 cast), exact rational arithmetic, and properties that fix the
rounding rule (nearest, ties to even, monotone, idempotent).  CPU only.
"""
import json
import math
import os
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "storage_hand_worked.json")


def _value(x):
    if isinstance(x, str):
        return {"inf": np.float32(np.inf), "-inf": np.float32(-np.inf), "nan": np.float32(np.nan),
                "-0": np.float32(-0.0)}[x]
    v = math.ldexp(x[0], x[1])
    assert float(np.float32(v)) == v, "golden inputs must be exact in float32"
    return np.float32(v)


def _cases(kind):
    with open(GOLDEN) as f:
        return json.load(f)[kind]


@pytest.mark.parametrize("case", _cases("f16"), ids=lambda c: c["code"] + "_" + str(c["x"]))
def test_hand_worked_f16(case):
    got = oracle.store_f16(np.array([_value(case["x"])], dtype=np.float32)).view(np.uint16)[0]
    assert int(got) == int(case["code"], 16), case["why"]


@pytest.mark.parametrize("case", _cases("bf16"), ids=lambda c: c["code"] + "_" + str(c["x"]))
def test_hand_worked_bf16(case):
    code, back = oracle.store_bf16(np.array([_value(case["x"])], dtype=np.float32))
    assert int(code[0]) == int(case["code"], 16), case["why"]
    again = oracle.load_bf16(code)
    assert np.array_equal(again.view(np.uint32), back.view(np.uint32)) or (np.isnan(again[0]) and np.isnan(back[0]))


def _samples(seed, count=200000):
    """Floats of every magnitude the formats care about: random bit patterns,
    values around the halfway points, subnormal ranges, the overflow edge."""
    rng = np.random.default_rng(seed)
    bits = rng.integers(0, 1 << 32, size=count, dtype=np.uint64).astype(np.uint32)
    a = bits.view(np.float32)
    b = (rng.standard_normal(count) * 10.0 ** rng.uniform(-9, 6, size=count)).astype(np.float32)
    c = (rng.integers(-(1 << 12), 1 << 12, size=count) * np.float32(2.0) ** rng.integers(-30, 8, size=count)).astype(np.float32)
    x = np.concatenate([a, b, c])
    return x[~np.isnan(x)]


def test_f16_matches_numpy_cast():
    x = _samples(1)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16)
    assert np.array_equal(oracle.store_f16(x).view(np.uint16), want.view(np.uint16))


def test_f16_matches_struct_format_e():
    x = _samples(2, 3000)
    got = oracle.store_f16(x).view(np.uint16)
    for v, g in zip(x.tolist(), got.tolist()):
        try:
            want = struct.unpack("<H", struct.pack("<e", v))[0]
        except OverflowError:              # struct refuses what rounds to infinity
            want = 0xFC00 if v < 0 else 0x7C00
        assert g == want, v


def test_f16_every_code_is_a_fixed_point():
    codes = np.arange(1 << 16, dtype=np.uint16)
    vals = codes.view(np.float16).astype(np.float32)       # exact widening
    keep = ~np.isnan(vals)
    assert np.array_equal(oracle.store_f16(vals[keep]).view(np.uint16), codes[keep])
    assert np.all(np.isnan(oracle.store_f16(vals[~keep]).astype(np.float32)))


def test_bf16_matches_torch_cast():
    x = _samples(3)
    want = torch.from_numpy(x).to(torch.bfloat16)
    code, back = oracle.store_bf16(x)
    assert np.array_equal(code.view(np.int16), want.view(torch.int16).numpy())
    assert np.array_equal(back.view(np.uint32), want.to(torch.float32).numpy().view(np.uint32))


def test_bf16_every_code_is_a_fixed_point_and_loads_as_the_top_half_of_a_float():
    codes = np.arange(1 << 16, dtype=np.uint16)
    vals = oracle.load_bf16(codes)
    top = (codes.astype(np.uint32) << 16).view(np.float32)   # a bfloat16 is the upper half of the float32 of equal value
    keep = ~np.isnan(top)
    assert np.array_equal(vals[keep].view(np.uint32), top[keep].view(np.uint32))
    assert np.all(np.isnan(vals[~keep]))
    code, _ = oracle.store_bf16(vals[keep])
    assert np.array_equal(code, codes[keep])


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_nearest_ties_to_even_in_exact_arithmetic(kind):
    """For finite results: no representable value is closer than the stored one,
    and at a tie the stored code is even."""
    fbits, emin = (10, -14) if kind == "f16" else (7, -126)
    x = _samples(4, 4000)
    if kind == "f16":
        back = oracle.store_f16(x).astype(np.float32)
        code = oracle.store_f16(x).view(np.uint16)
    else:
        code, back = oracle.store_bf16(x)
    checked = 0
    for v, b, c in zip(x.tolist(), back.tolist(), code.tolist()):
        if math.isinf(b) or math.isinf(v):
            continue
        fv, fb = Fraction(v), Fraction(b)
        e = max(emin, math.frexp(abs(b))[1] - 1) if b != 0 else emin
        step = Fraction(2) ** (e - fbits)
        # the neighbour below |b| may sit in the exponent below, where steps are half as wide
        lower_step = step / 2 if (b != 0 and abs(fb) == Fraction(2) ** e and e > emin) else step
        err = abs(fv - fb)
        assert err <= step / 2 and (abs(fv) >= abs(fb) or err <= lower_step / 2), (v, b)
        if err == step / 2 or (abs(fv) < abs(fb) and err == lower_step / 2):
            assert c % 2 == 0, (v, b)
        checked += 1
    assert checked > 2000


@pytest.mark.parametrize("kind", ["f16", "bf16"])
def test_monotone(kind):
    x = np.sort(_samples(5, 50000))
    x = x[np.isfinite(x)]
    back = oracle.store_f16(x).astype(np.float32) if kind == "f16" else oracle.store_bf16(x)[1]
    assert np.all(back[1:] >= back[:-1])            # (inf >= inf holds; a difference would be NaN there)
