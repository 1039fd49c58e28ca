"""Helpers shared by the GPU parity tests: guarded device buffers, uploads and
the oracle-side packing of logical +-1 tensors."""
import numpy as np
import pytest
import torch

import oracle
from paper_2010_00704_amd import binding as B

GUARD = 64              # words on each side of every output
SENTINEL = 0x5A5A5A5A


class Guarded:
    """A device buffer of `words` 32-bit words with sentinel bands around it
    that must stay untouched."""

    def __init__(self, words, dev):
        self.words = int(words)
        self.buf = torch.full((self.words + 2 * GUARD,), SENTINEL, dtype=torch.int32, device=dev)

    @classmethod
    def of_bytes(cls, nbytes, dev):
        return cls((int(nbytes) + 3) // 4, dev)

    @property
    def ptr(self):
        return self.buf.data_ptr() + 4 * GUARD

    def put(self, a):
        """Copies the bytes of a numpy array to the start of the buffer."""
        flat = torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1))
        self.buf.view(torch.uint8)[4 * GUARD:4 * GUARD + flat.numel()] = flat.to(self.buf.device)

    def get(self, dtype=np.uint32, count=None):
        """The buffer's contents as `dtype` (the first `count` elements if given)
        after checking both guard bands."""
        torch.cuda.synchronize()
        host = self.buf.cpu().numpy()
        assert np.all(host[:GUARD] == SENTINEL), "write before the output buffer"
        assert np.all(host[GUARD + self.words:] == SENTINEL), "write past the output buffer"
        data = host[GUARD:GUARD + self.words].view(dtype)
        return data if count is None else data[:count]


# ---- storage types of the real stream.  A test parameter `half` is False (float32), True (IEEE
# half) or "bf16"; 16-bit values travel as numpy float16 arrays, bfloat16 as uint16 bit patterns.
REAL_PARAMS = [False, True, "bf16"]
REAL_IDS = ["f32", "f16", "bf16"]


def real_code(half):
    return B.BCNN_BF16 if half == "bf16" else (B.BCNN_F16 if half else B.BCNN_F32)


def real_np_dtype(half):
    return np.uint16 if half == "bf16" else (np.float16 if half else np.float32)


def real_store(v32, half):
    """float32 values -> the array as a stream of this type stores it (the oracle's rounding)."""
    if half == "bf16":
        return oracle.store_bf16(v32)[0]
    return oracle.store_f16(v32) if half else np.ascontiguousarray(v32, dtype=np.float32)


def real_values(stored, half):
    """stored array -> its values as float32 (exact)."""
    if half == "bf16":
        return oracle.load_bf16(stored)
    return stored.astype(np.float32)


def real_seed(half):
    return 2 if half == "bf16" else int(bool(half))


def gpu_device():
    assert torch.cuda.is_available(), "these tests need the GPU"
    B.lib()
    return torch.device("cuda:0")


def up(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def i32(a):
    """uint32 numpy -> int32 view (torch has no uint32 tensors)."""
    return np.ascontiguousarray(a).view(np.int32)


# variants that must take every shape the library supports: a refusal from one of them is a failure
COVER_ALL = (B.BCNN_VARIANT_AUTO, B.BCNN_VARIANT_VALU)


def run_variant(rc, what, variant):
    """A forced matrix-core variant may not cover a shape: that is a skip.  The
    default choice and the vector-ALU kernel cover everything, so from them
    (and for any other status) "unsupported" is a failure."""
    if rc == B.BCNN_ERR_UNSUPPORTED and variant not in COVER_ALL:
        pytest.skip("variant does not cover this shape")
    B.check(rc, what)


def oracle_pack_nchw(x):
    """[n, c, *spatial] +-1 -> packed [n, prod(spatial), cw] (the oracle's packer)."""
    n, c = x.shape[:2]
    return oracle.pack_channels(x.reshape(n, c, -1))


def oracle_pack_vectors(v):
    """[rows, c] +-1 -> packed [rows, cw] (pad words, one vector per row)."""
    return oracle.pack_channels(v[:, :, None])[:, 0, :]


def oracle_bits_of_sign(s):
    """[n, ho, wo, o] +-1 -> packed [n, ho*wo, cwo]."""
    n, ho, wo, o = s.shape
    return oracle.pack_channels(s.reshape(n, ho * wo, o).transpose(0, 2, 1))
