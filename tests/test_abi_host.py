"""Host-side checks of libbcnn.so that need no GPU: the library loads, exports
every function include/bcnn.h declares, and rejects bad arguments before any
launch (validation never dereferences the data pointers)."""
import ctypes
import os
import re

import numpy as np

from paper_2010_00704_amd import binding as B
from paper_2010_00704_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # aligned, non-null, never dereferenced by the host checks


def _declared():
    names = set()
    for header in ("bcnn.h", "bcnn_diag.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(bcnn_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_function():
    names = _declared()
    assert set(B.EXPORTS) == set(names)
    L = B.lib()
    for name in names:
        assert getattr(L, name) is not None


def test_out_dim_and_status_strings():
    assert B.bcnn_out_dim(56, 3, 2, 1) == 28
    assert B.bcnn_out_dim(14, 3, 1, 1) == 14
    assert B.bcnn_out_dim(7, 1, 1, 0) == 7
    assert B.bcnn_out_dim(5, 3, 2, 0) == 2
    assert B.bcnn_out_dim(1, 3, 1, 0) == 0
    for code in (0, -1, -2, -3, -4, -99):
        assert isinstance(B.bcnn_status_string(code), str) and B.bcnn_status_string(code)


def _conv(desc, x=FAKE, w=FAKE + 0x1000, y=FAKE + 0x2000):
    return B.lib().bcnn_conv2d_binary(ctypes.byref(desc), x, w, y, None)


def test_conv_rejects_bad_descriptors_without_launching():
    good = dict(n=1, c_in=64, h=14, w=14, c_out=64, kh=3, kw=3, stride=1, pad=1)

    def rc(**kw):
        d = dict(good)
        d.update(kw)
        return _conv(B.bcnn_conv_desc(**d))
    assert rc(n=0) == B.BCNN_ERR_INVALID_ARG
    assert rc(c_in=0) == B.BCNN_ERR_INVALID_ARG
    assert rc(c_out=-3) == B.BCNN_ERR_INVALID_ARG
    assert rc(kh=5, kw=5) == B.BCNN_ERR_UNSUPPORTED
    assert rc(kh=3, kw=1) == B.BCNN_ERR_UNSUPPORTED
    assert rc(kh=2, kw=2) == B.BCNN_ERR_UNSUPPORTED
    assert rc(stride=3) == B.BCNN_ERR_UNSUPPORTED
    assert rc(stride=0) == B.BCNN_ERR_INVALID_ARG
    assert rc(pad=2) == B.BCNN_ERR_UNSUPPORTED
    assert rc(kh=1, kw=1, pad=1) == B.BCNN_ERR_UNSUPPORTED
    assert rc(h=1, w=1, pad=0) == B.BCNN_ERR_INVALID_ARG  # 3x3 window does not fit
    assert rc(n=1 << 20, h=1 << 10, w=1 << 10) == B.BCNN_ERR_UNSUPPORTED  # beyond 2^31 elements
    d = B.bcnn_conv_desc(**good)
    assert _conv(d, x=None) == B.BCNN_ERR_INVALID_ARG
    assert _conv(d, w=None) == B.BCNN_ERR_INVALID_ARG
    assert _conv(d, y=None) == B.BCNN_ERR_INVALID_ARG
    assert _conv(d, x=FAKE + 2) == B.BCNN_ERR_ALIGNMENT
    assert _conv(d, y=FAKE) == B.BCNN_ERR_INVALID_ARG  # output aliases input
    assert B.lib().bcnn_conv2d_binary(None, FAKE, FAKE, FAKE, None) == B.BCNN_ERR_INVALID_ARG
    L = B.lib()
    assert L.bcnn_conv2d_binary_sign_pack(ctypes.byref(d), FAKE, FAKE + 64, None, FAKE + 128, None) \
        == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_conv2d_binary_variant(ctypes.byref(d), FAKE, FAKE + 64, None, FAKE + 128, 77, None) \
        == B.BCNN_ERR_INVALID_ARG


def test_pack_and_threshold_reject_bad_arguments():
    L = B.lib()
    assert L.bcnn_pack(None, 0, 1, 32, 1, FAKE, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_pack(FAKE, 0, 0, 32, 1, FAKE + 64, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_pack(FAKE, 9, 1, 32, 1, FAKE + 64, None) == B.BCNN_ERR_UNSUPPORTED
    assert L.bcnn_pack(FAKE + 2, 0, 1, 32, 1, FAKE + 64, None) == B.BCNN_ERR_ALIGNMENT
    assert L.bcnn_pack(FAKE + 2, 2, 1, 32, 1, FAKE + 66, None) == B.BCNN_ERR_ALIGNMENT
    assert L.bcnn_pack(FAKE, 0, 1 << 40, 32, 1, FAKE + 64, None) == B.BCNN_ERR_UNSUPPORTED
    assert L.bcnn_threshold_sign_pack(FAKE, None, 4, 32, FAKE + 64, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_threshold_sign_pack(FAKE, FAKE + 64, 0, 32, FAKE + 128, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_threshold_sign_pack(FAKE, FAKE + 64, 4, 32, FAKE + 1, None) == B.BCNN_ERR_ALIGNMENT
    assert L.bcnn_diag_copy_u32(None, FAKE, 4, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_diag_valu_peak(None, 1, 1, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_diag_store_u32(FAKE, 6, 0, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_diag_store_u32(FAKE + 4, 8, 0, None) == B.BCNN_ERR_ALIGNMENT
    assert L.bcnn_diag_read_u32(FAKE, 8, None, 0, None) == B.BCNN_ERR_INVALID_ARG


# ---- the seeded input generator (shared by the oracle side and the GPU side) ----
def test_generator_is_counter_based_and_reproducible():
    a = W.pm1(42, (3, 5, 7), 0.5)
    b = W.pm1(42, (3, 5, 7), 0.5)
    np.testing.assert_array_equal(a, b)
    assert set(np.unique(a)) <= {-1, 1}
    assert not np.array_equal(a, W.pm1(43, (3, 5, 7), 0.5))
    # element i does not depend on how many elements are drawn
    np.testing.assert_array_equal(W.pm1(42, (50,), 0.5)[:20], W.pm1(42, (20,), 0.5))
    big = W.pm1(7, (1 << 18,), 0.3)
    assert abs((big > 0).mean() - 0.3) < 0.01
    t = W.thresholds(9, 1000, 72)
    assert t.min() >= -72 and t.max() <= 72 and t.dtype == np.int32
    assert len(np.unique(t)) > 100


def test_subset_of_images_matches_full_batch():
    cfg, x_all, ws, ts = W.make_inputs(1)
    assert x_all.shape == (1, 64, 14, 14) and ws[0].shape == (64, 64, 3, 3) and ts[0] is None
    cfg3 = W.CONFIGS[2]
    full = W.pm1(W.seeds(3)[0], (4, cfg3.c_in, cfg3.h, cfg3.w), cfg3.p_x)
    _, sub, _, thr = W.make_inputs(3, images=[3, 1])
    np.testing.assert_array_equal(sub[0], full[3])
    np.testing.assert_array_equal(sub[1], full[1])
    assert thr[0].shape == (256,) and abs(int(thr[0].max())) <= 288
    assert abs((sub > 0).mean() - 0.3) < 0.02


def test_real_values_carry_the_requested_signs():
    s = W.pm1(5, (2, 40, 9), 0.5)
    r = W.real_with_sign(5, s)
    assert r.dtype == np.float32 and r.shape == s.shape
    np.testing.assert_array_equal(np.sign(r).astype(np.int8), s)
    assert np.all(np.abs(r) >= 0.5) and np.all(np.abs(r) < 1.5)


def test_config_table_matches_the_stated_shapes():
    ops = [W.binary_ops(c) for c in W.CONFIGS]
    assert ops[0] == 2 * 196 * 64 * 576
    assert ops[1] == 2 * 100352 * 256 * 256
    assert ops[2] == 2 * 50176 * 256 * 2304
    assert ops[3] == 2 * 50176 * 512 * 2304
    assert ops[4] == 4 * 2 * 12544 * 1024 * 9216
    assert W.out_hw(W.CONFIGS[3]) == (28, 28)


def test_widened_entry_points_reject_bad_arguments():
    """bcnn_pack_bias[_replicated], the pooling call, the branch calls and the module call check
    their arguments on the host before any launch."""
    L = B.lib()
    d3 = B.bcnn_conv_desc(n=1, c_in=64, h=8, w=8, c_out=32, kh=3, kw=3, stride=1, pad=1)
    d1 = B.bcnn_conv_desc(n=1, c_in=64, h=8, w=8, c_out=32, kh=1, kw=1, stride=1, pad=0)
    x, w, g, z, p = FAKE, FAKE + 0x1000, FAKE + 0x2000, FAKE + 0x3000, FAKE + 0x4000
    # pack with bias / replication
    assert L.bcnn_pack_bias(x, B.BCNN_F32, 1, 32, 4, None, z, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_pack_bias(x, B.BCNN_F32, 1, 32, 4, g + 2, z, None) == B.BCNN_ERR_ALIGNMENT
    assert L.bcnn_pack_bias(x, 9, 1, 32, 4, g, z, None) == B.BCNN_ERR_UNSUPPORTED
    assert L.bcnn_pack_bias_replicated(x, B.BCNN_F32, 1, 32, 4, 0, g, z, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_pack_bias_replicated(x, B.BCNN_F32, 1, 0, 4, 2, g, z, None) == B.BCNN_ERR_INVALID_ARG
    assert L.bcnn_pack_bias_replicated(x, B.BCNN_F32, 1, 1 << 30, 4, 4, g, z, None) == B.BCNN_ERR_UNSUPPORTED
    # average pooling + bias + sign + pack
    a = L.bcnn_avgpool_bias_sign_pack
    assert a(None, B.BCNN_F32, 1, 4, 4, 8, 2, None, z, p, None) == B.BCNN_ERR_INVALID_ARG
    assert a(x, B.BCNN_F32, 1, 4, 4, 8, 2, None, None, None, None) == B.BCNN_ERR_INVALID_ARG
    assert a(x, B.BCNN_F32, 1, 4, 4, 8, 0, None, z, p, None) == B.BCNN_ERR_INVALID_ARG
    assert a(x, B.BCNN_F32, 1, 4, 4, 8, 5, None, z, p, None) == B.BCNN_ERR_INVALID_ARG       # empty pooled map
    assert a(x, B.BCNN_F32, 1, 64, 64, 8, 9, None, z, p, None) == B.BCNN_ERR_UNSUPPORTED
    assert a(x, B.BCNN_I8, 1, 4, 4, 8, 2, None, z, p, None) == B.BCNN_ERR_UNSUPPORTED
    assert a(x, B.BCNN_F32, 1, 4, 4, 8, 2, None, x, p, None) == B.BCNN_ERR_INVALID_ARG        # in place
    assert a(x, B.BCNN_F32, 1, 4, 4, 8, 2, g + 2, z, p, None) == B.BCNN_ERR_ALIGNMENT
    assert a(x, B.BCNN_F16, 1, 4, 4, 8, 2, None, z + 1, p, None) == B.BCNN_ERR_ALIGNMENT
    assert a(x, B.BCNN_F32, 1 << 20, 1 << 10, 1 << 10, 8, 2, None, z, p, None) == B.BCNN_ERR_UNSUPPORTED
    # branches
    f = L.bcnn_conv2d_binary_branches
    assert f(ctypes.byref(d3), 9, x, 0, w, None, 0, g, None, None, 0, None) == B.BCNN_ERR_INVALID_ARG
    assert f(ctypes.byref(d3), 8, x, 0, w, None, 0, g, None, z, 0, None) == B.BCNN_ERR_INVALID_ARG
    assert f(ctypes.byref(d1), 0, x, 0, w, None, 0, g, None, z, 0, None) == B.BCNN_ERR_INVALID_ARG
    assert f(ctypes.byref(d1), 2000, x, 0, w, None, 0, g, None, z, 0, None) == B.BCNN_ERR_UNSUPPORTED
    assert f(ctypes.byref(d3), 9, x, 1, w, None, 0, g, None, z, 0, None) == B.BCNN_ERR_INVALID_ARG  # stride < tensor
    assert f(ctypes.byref(d3), 9, x, 0, w, None, 5, g, None, z, 0, None) == B.BCNN_ERR_INVALID_ARG  # pad mode
    assert f(ctypes.byref(d3), 9, x, 0, w, p + 1, 0, g, None, z, 0, None) == B.BCNN_ERR_ALIGNMENT
    assert f(ctypes.byref(d3), 9, x, 0, w, None, 0, g, None, z, 77, None) == B.BCNN_ERR_UNSUPPORTED  # variant
    assert f(ctypes.byref(d3), 9, x, 0, w, None, 0, g, None, z, B.BCNN_VARIANT_MFMA_FP4, None) \
        == B.BCNN_ERR_UNSUPPORTED                                                  # c_in not a multiple of 256
    assert L.bcnn_conv2d_binary_branches_sign_pack(ctypes.byref(d3), 9, x, 0, w, None, 0, g, None, x, 0, None) \
        == B.BCNN_ERR_INVALID_ARG                                                  # output aliases input
    # module
    def ep(**kw):
        base = dict(bn_scale=g, bn_bias=g + 0x100, identity=None, prelu_slope=None, next_bias=None,
                    real_dtype=B.BCNN_F32, identity_channels=0)
        base.update(kw)
        return B.bcnn_module_epilogue(**base)
    m = L.bcnn_conv2d_binary_module
    assert m(ctypes.byref(d1), x, w, None, z, p, 0, None) == B.BCNN_ERR_INVALID_ARG
    assert m(ctypes.byref(d1), x, w, ctypes.byref(ep()), None, None, 0, None) == B.BCNN_ERR_INVALID_ARG
    assert m(ctypes.byref(d1), x, w, ctypes.byref(ep(bn_scale=None)), z, p, 0, None) == B.BCNN_ERR_INVALID_ARG
    assert m(ctypes.byref(d1), x, w, ctypes.byref(ep(real_dtype=B.BCNN_I8)), z, p, 0, None) == B.BCNN_ERR_UNSUPPORTED
    assert m(ctypes.byref(d1), x, w, ctypes.byref(ep(identity_channels=33)), z, p, 0, None) == B.BCNN_ERR_INVALID_ARG
    assert m(ctypes.byref(d1), x, w, ctypes.byref(ep(identity=z, identity_channels=16)), z, p, 0, None) \
        == B.BCNN_ERR_INVALID_ARG                                                  # replicated identity in place
    assert m(ctypes.byref(d1), x, w, ctypes.byref(ep(real_dtype=B.BCNN_F16)), z + 1, p, 0, None) == B.BCNN_ERR_ALIGNMENT
    assert m(ctypes.byref(d1), x, w, ctypes.byref(ep()), z, p, B.BCNN_VARIANT_MFMA_I8, None) == B.BCNN_ERR_UNSUPPORTED
    assert m(ctypes.byref(d1), x, w, ctypes.byref(ep()), z, p, B.BCNN_VARIANT_MFMA_FP4, None) == B.BCNN_ERR_UNSUPPORTED
