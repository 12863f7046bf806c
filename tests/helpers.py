"""Test-side helpers: an independent numpy bit packer and small utilities.

The packer here is the harness's own (numpy packbits); it is not the library's
bnn_pack_bits and not part of the oracle.
"""
import numpy as np


def pack_pm1(a):
    """+-1 (or any int) array [..., k] -> uint32 [..., ceil(k/32)]; bit = (value > 0),
    element t in word t//32 at bit t%32 (LSB first), tail bits zero."""
    a = np.asarray(a)
    k = a.shape[-1]
    kw = (k + 31) // 32
    bits = (a > 0).astype(np.uint8)
    if kw * 32 != k:
        padw = [(0, 0)] * (a.ndim - 1) + [(0, kw * 32 - k)]
        bits = np.pad(bits, padw)
    packed = np.packbits(bits, axis=-1, bitorder="little")
    return np.ascontiguousarray(packed).view(np.uint32).reshape(a.shape[:-1] + (kw,))


def unpack_words(words, k):
    """uint32 [..., kw] -> +-1 int8 [..., k]."""
    words = np.ascontiguousarray(words, dtype=np.uint32)
    b = np.unpackbits(words.view(np.uint8), axis=-1, bitorder="little")[..., :k]
    return (2 * b.astype(np.int8) - 1).astype(np.int8)
