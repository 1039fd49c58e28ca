"""Seeded synthetic inputs and the five benchmark layer shapes.

This module holds no arithmetic of the method (no sign, no packing, no
convolution): it only draws reproducible random tensors and names the layer
shapes.  Tests and the benchmark hand the same arrays to the CPU oracle and to
the HIP library.

Generator: counter based, so any element can be produced without the others.
Element ``i`` of stream ``seed`` is ``mix(seed * A + (i + 1) * G)`` where
``mix`` is the splitmix64 output function (Steele, Lea, Flood 2014) and ``G``
its golden-ratio increment; the top 24 bits give a uniform in [0, 1).
"""
from collections import namedtuple

import numpy as np

_G = np.uint64(0x9E3779B97F4A7C15)
_A = np.uint64(0xD1342543DE82EF95)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def raw_u64(seed, start, count):
    """64-bit outputs for counters start .. start+count-1 of stream ``seed``."""
    with np.errstate(over="ignore"):
        base = np.uint64(seed) * _A
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        return _mix(base + idx * _G)


def _fill(shape, fn, dtype):
    total = int(np.prod(shape, dtype=np.int64))
    out = np.empty(total, dtype=dtype)
    for s in range(0, total, _CHUNK):
        n = min(_CHUNK, total - s)
        out[s:s + n] = fn(s, n)
    return out.reshape(shape)


def pm1(seed, shape, p=0.5):
    """int8 tensor of +-1, P(+1) = p, element order = C order of ``shape``."""
    cut = np.uint64(int(round(p * (1 << 24))))

    def fn(s, n):
        u24 = raw_u64(seed, s, n) >> np.uint64(40)
        return np.where(u24 < cut, 1, -1).astype(np.int8)
    return _fill(shape, fn, np.int8)


def real_with_sign(seed, signs):
    """float32 tensor whose sign pattern is ``signs`` (+-1) and whose
    magnitude is 0.5 + u, u uniform in [0, 1): a real-valued feature map whose
    binarisation is known, for the packing step."""
    flat = np.ascontiguousarray(signs).reshape(-1)

    def fn(s, n):
        u = (raw_u64(seed ^ 0x5EED, s, n) & np.uint64(0xFFFFFF)).astype(np.float32) / np.float32(1 << 24)
        return (np.float32(0.5) + u) * flat[s:s + n].astype(np.float32)
    return _fill(signs.shape, fn, np.float32)


def uniform_f32(seed, shape, lo, hi, steps=None):
    """float32 tensor uniform on [lo, hi).  With ``steps`` the values lie on the
    grid lo + k * (hi - lo) / steps, k = 0 .. steps-1 (choose lo, hi and steps so
    that the grid is exact in float32, e.g. quarters), which makes exact ties
    between sums of such values likely."""
    lo32, span = np.float32(lo), np.float32(hi) - np.float32(lo)

    def fn(s, n):
        u24 = (raw_u64(seed, s, n) >> np.uint64(40)).astype(np.float64)
        if steps is not None:
            k = np.floor(u24 * steps / float(1 << 24))
            return (lo32 + (k * (float(span) / steps)).astype(np.float32)).astype(np.float32)
        return (lo32 + (u24 / float(1 << 24)).astype(np.float32) * span).astype(np.float32)
    return _fill(shape, fn, np.float32)


def thresholds(seed, count, bound):
    """int32 thresholds, uniform on the closed integer interval [-bound, bound]."""
    r = raw_u64(seed, 0, count) >> np.uint64(11)
    return (r % np.uint64(2 * bound + 1)).astype(np.int64).astype(np.int32) - np.int32(bound)


Layer = namedtuple("Layer", "name n c_in h w c_out k stride pad p_x fused layers")

# The five layer shapes the throughput metric is quoted on.  p_x = P(input = +1);
# weights are always symmetric.  ``fused`` layers end in threshold + sign + repack,
# the others return int32 sums.  ``layers`` > 1 is a chain of equal layers whose
# packed output feeds the next.
CONFIGS = (
    Layer("cfg1_3x3_c64_14", 1, 64, 14, 14, 64, 3, 1, 1, 0.5, False, 1),
    Layer("cfg2_1x1_c256_56", 32, 256, 56, 56, 256, 1, 1, 0, 0.5, False, 1),
    Layer("cfg3_3x3_c256_28_fused", 64, 256, 28, 28, 256, 3, 1, 1, 0.3, True, 1),
    Layer("cfg4_3x3s2_c256_512_56_fused", 64, 256, 56, 56, 512, 3, 2, 1, 0.5, True, 1),
    Layer("cfg5_chain4_3x3_c1024_7_fused", 256, 1024, 7, 7, 1024, 3, 1, 1, 0.5, True, 4),
)


# The binary 1x1 convolution modules of the paper's network, one per level of its
# Table 1 (channels = RC, map = H/S x W/S; C_in = C_out because of the identity
# path), per image.  A second workload: tiny K at many pixels (stem) to large K
# at 49 pixels (level 5).
TABLE1_MODULES = (
    ("stem", 32, 224), ("level1", 64, 112), ("level2", 128, 56),
    ("level3", 256, 28), ("level4", 512, 14), ("level5", 1024, 7),
)


def out_hw(cfg):
    ho = (cfg.h + 2 * cfg.pad - cfg.k) // cfg.stride + 1
    wo = (cfg.w + 2 * cfg.pad - cfg.k) // cfg.stride + 1
    return ho, wo


def k_total(cfg):
    return cfg.c_in * cfg.k * cfg.k


def binary_ops(cfg):
    """2 * M * N * K per layer times the number of layers (one binary
    multiply-accumulate counted as two binary operations; padded taps count)."""
    ho, wo = out_hw(cfg)
    return 2 * cfg.n * ho * wo * cfg.c_out * k_total(cfg) * cfg.layers


def seeds(index, layer=0):
    """(x, w, thr) seeds of config ``index`` (1-based) and chain layer."""
    return 1000 + index, 2000 + index + 100 * layer, 3000 + index + 100 * layer


def make_inputs(index, images=None):
    """Logical tensors of config ``index`` (1-based).

    Returns (cfg, x [n,c,h,w] int8, [w_l [o,c,k,k] int8], [thr_l int32 or None]).
    ``images``, if given, is a list of image indices: only those images are
    generated (their values are the same as in the full batch).
    """
    cfg = CONFIGS[index - 1]
    sx, _, _ = seeds(index)
    per_image = cfg.c_in * cfg.h * cfg.w
    if images is None:
        x = pm1(sx, (cfg.n, cfg.c_in, cfg.h, cfg.w), cfg.p_x)
    else:
        cut = np.uint64(int(round(cfg.p_x * (1 << 24))))
        x = np.empty((len(images), cfg.c_in, cfg.h, cfg.w), dtype=np.int8)
        for j, n in enumerate(images):
            u24 = raw_u64(sx, n * per_image, per_image) >> np.uint64(40)
            x[j] = np.where(u24 < cut, 1, -1).astype(np.int8).reshape(cfg.c_in, cfg.h, cfg.w)
    ws, ts = [], []
    for layer in range(cfg.layers):
        _, sw, st = seeds(index, layer)
        ws.append(pm1(sw, (cfg.c_out, cfg.c_in, cfg.k, cfg.k), 0.5))
        ts.append(thresholds(st, cfg.c_out, k_total(cfg) // 8) if cfg.fused else None)
    return cfg, x, ws, ts
