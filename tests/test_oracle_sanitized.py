"""The oracle's C files and the host-side checks under AddressSanitizer and
UndefinedBehaviorSanitizer.  The files are compiled with gcc
-fsanitize=address,undefined into executables of their own
(tests/host/oracle_san_driver.c, tests/host/div_by_check.cpp, tests/host/pos_plan_check.cpp) and run on the
hand-worked cases and on seeded shapes with ragged sizes; any report ends the
run with a non-zero status.  Outputs are compared with the hand-worked values
and with the ordinary build of the oracle.  CPU only.
"""
import glob
import json
import os
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
       "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="2")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_san_driver")
    srcs = sorted(glob.glob(os.path.join(ROOT, "oracle", "*.c")))
    assert len(srcs) == 3
    subprocess.run(["gcc", "-std=c11", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra"] + SAN +
                   [os.path.join(ROOT, "tests", "host", "oracle_san_driver.c")] + srcs + ["-lm", "-o", exe], check=True)
    return exe


def _run(exe, tmp_path, op, dims, inputs, outputs):
    """inputs: list of arrays; outputs: list of (dtype, shape).  Returns the output arrays."""
    paths = []
    for i, arr in enumerate(inputs):
        p = str(tmp_path / ("in%d.bin" % i))
        np.ascontiguousarray(arr).tofile(p)
        paths.append(p)
    outs = [str(tmp_path / ("out%d.bin" % i)) for i in range(len(outputs))]
    proc = subprocess.run([exe, op] + [str(d) for d in dims] + paths + outs, env=ENV, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=300)
    assert proc.returncode == 0, proc.stdout
    assert "runtime error" not in proc.stdout and "Sanitizer" not in proc.stdout, proc.stdout
    return [np.fromfile(p, dtype=dt).reshape(shape) for p, (dt, shape) in zip(outs, outputs)]


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


def _hand_worked():
    with open(os.path.join(ROOT, "tests", "golden", "hand_worked.json")) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _hand_worked(), ids=lambda c: c["name"])
def test_hand_worked_convolutions_under_sanitizers(driver, tmp_path, case):
    c, h, w = case["x_shape"]
    o, _, k, _ = case["w_shape"]
    x = _signs(case["x"], (1, c, h, w))
    wt = _signs(case["w"], case["w_shape"])
    want = np.array(case["y"], dtype=np.int32)
    ho, wo = want.shape[:2]
    thr = np.zeros(o, dtype=np.int32)
    y, s, packed, unpacked = _run(driver, tmp_path, "conv", [1, c, h, w, o, k, case["stride"], case["pad"]],
                                  [x, wt, thr],
                                  [(np.int32, (ho, wo, o)), (np.int8, (ho, wo, o)), (np.uint32, (1, ho * wo, (o + 31) // 32)),
                                   (np.int8, (1, o, ho * wo))])
    assert np.array_equal(y, want)
    assert np.array_equal(s, np.where(want >= 0, 1, -1))
    assert np.array_equal(unpacked[0].T.reshape(ho, wo, o), s)


@pytest.mark.parametrize("shape", [(2, 33, 5, 7, 35, 3, 2, 1), (1, 1, 1, 1, 1, 1, 1, 0), (3, 65, 4, 3, 31, 3, 1, 1),
                                   (2, 7, 6, 6, 64, 1, 2, 0), (1, 3, 2, 2, 5, 3, 1, 1)])
def test_ragged_shapes_under_sanitizers_match_the_ordinary_build(driver, tmp_path, shape):
    n, c, h, w, o, k, stride, pad = shape
    rng = np.random.default_rng(sum(shape))
    x = rng.choice(np.array([-1, 1], dtype=np.int8), size=(n, c, h, w))
    wt = rng.choice(np.array([-1, 1], dtype=np.int8), size=(o, c, k, k))
    thr = rng.integers(-c, c + 1, size=o).astype(np.int32)
    want_y = oracle.conv2d_pm1(x, wt, stride, pad)
    _, ho, wo, _ = want_y.shape
    want_s = oracle.threshold_sign(want_y, thr)
    want_p = oracle.pack_channels(want_s.reshape(n, ho * wo, o).transpose(0, 2, 1))
    y, s, packed, unpacked = _run(driver, tmp_path, "conv", shape, [x, wt, thr],
                                  [(np.int32, want_y.shape), (np.int8, want_s.shape), (np.uint32, want_p.shape),
                                   (np.int8, (n, o, ho * wo))])
    assert np.array_equal(y, want_y) and np.array_equal(s, want_s) and np.array_equal(packed, want_p)
    assert np.array_equal(unpacked, want_s.reshape(n, ho * wo, o).transpose(0, 2, 1))
    # the branch construction on the same operands: shifted branches (F = k) with pad values from {-1, 0, +1}
    p = k * k
    xb = rng.choice(np.array([-1, 1], dtype=np.int8), size=(p, n, c, h, w))
    padv = rng.integers(-1, 2, size=(p, c)).astype(np.int8)
    g = rng.uniform(-1.5, 1.5, size=(p, o)).astype(np.float32)
    hb = rng.uniform(-5, 5, size=o).astype(np.float32)
    for shared in (0, 1):
        src = xb[:1] if shared else xb
        want64, want32 = oracle.branches_pm1(src, padv, wt, g, hb, stride, pad)
        z64, z32 = _run(driver, tmp_path, "branches", [n, c, h, w, o, k, p, stride, pad, shared],
                        [src, padv, wt, g, hb], [(np.float64, want64.shape), (np.float32, want32.shape)])
        assert np.array_equal(z64, want64) and np.array_equal(z32, want32)


def test_module_pool_and_storage_under_sanitizers(driver, tmp_path):
    with open(os.path.join(ROOT, "tests", "golden", "module_hand_worked.json")) as f:
        m1 = json.load(f)["cases"][0]
    y = np.array(m1["y"], dtype=np.int32)
    arrs = [np.array(m1[k], dtype=np.float32) for k in ("g", "b", "identity", "a", "c")]
    r64, r32, bits = _run(driver, tmp_path, "module", [y.shape[0], y.shape[1]], [y] + arrs,
                          [(np.float64, y.shape), (np.float32, y.shape), (np.int8, y.shape)])
    assert np.array_equal(r64, np.array(m1["r"])) and np.array_equal(r32, np.array(m1["r"], dtype=np.float32))
    assert np.array_equal(bits, np.array(m1["bits"], dtype=np.int8))
    rng = np.random.default_rng(7)
    a = rng.uniform(-8, 8, size=(2, 7, 5, 3)).astype(np.float32)
    for s in (1, 2, 3):
        want64, want32 = oracle.avgpool_nhwc(a, s)
        p64, p32 = _run(driver, tmp_path, "pool", [2, 7, 5, 3, s], [a], [(np.float64, want64.shape), (np.float32, want32.shape)])
        assert np.array_equal(p64, want64) and np.array_equal(p32, want32)
    with open(os.path.join(ROOT, "tests", "golden", "storage_hand_worked.json")) as f:
        gold = json.load(f)
    import math
    special = {"inf": np.inf, "-inf": -np.inf, "nan": np.nan, "-0": -0.0}
    for kind, col in (("f16", 0), ("bf16", 2)):
        xs = np.array([special[c["x"]] if isinstance(c["x"], str) else math.ldexp(*c["x"]) for c in gold[kind]],
                      dtype=np.float32)
        outs = _run(driver, tmp_path, "store", [xs.size], [xs],
                    [(np.uint16, xs.shape), (np.float32, xs.shape), (np.uint16, xs.shape), (np.float32, xs.shape),
                     (np.float32, xs.shape)])
        assert [int(v) for v in outs[col]] == [int(c["code"], 16) for c in gold[kind]]


def test_division_constants_under_sanitizers(tmp_path):
    exe = str(tmp_path / "div_by_check_san")
    subprocess.run(["g++", "-std=c++17", "-I", os.path.join(ROOT, "paper_2010_00704_amd", "csrc")] + SAN +
                   [os.path.join(ROOT, "tests", "host", "div_by_check.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert out.returncode == 0, out.stdout
    assert "mismatches: 0" in out.stdout and "runtime error" not in out.stdout


def test_position_major_plan_under_sanitizers(tmp_path):
    exe = str(tmp_path / "pos_plan_check_san")
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", os.path.join(ROOT, "paper_2010_00704_amd", "csrc")] + SAN +
                   [os.path.join(ROOT, "tests", "host", "pos_plan_check.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert out.returncode == 0, out.stdout
    assert "mismatches: 0" in out.stdout and "runtime error" not in out.stdout
