"""The compressed format of Section 3.2 as one bit stream, with the blocked n_patch widths of
Section 5.2 (test infrastructure).

The paper gives the format as the triple (w^c_1..l, n_patch, d_patch) per bit-plane and the sizes
of its parts (Eq. (2)); the order of bits inside a stream is not stated.  Reading used here, per
plane, planes one after another without padding:

  1. l fields of n_in bits: w^c of each slice (slice order = row-major over the padded matrix);
  2. for each block of `block_slices` consecutive slices (the last one may be shorter): 8 bits
     holding the width w_b of the block's n_patch fields, then one field of w_b bits per slice.
     w_b = ceil(lg(max n_patch of the block + 1)): the smallest width that can hold the maximum
     (the printed ceil(lg max(p)) cannot when max(p) is a power of two);
  3. sum(n_patch) fields of ceil(lg n_out) bits: the patch positions, slice by slice, ascending.

Fields are little endian (bit j of the field = bit j of the value; x_j for w^c) and bit k of the
stream is bit k % 8 of byte k / 8.  The 8-bit width of a block is bookkeeping the paper does not
count; `sizes` reports it separately so that the rest can be compared with Eq. (2).
"""
import math
from dataclasses import dataclass

import numpy as np


def field_width(max_value: int) -> int:
    """Bits needed to hold every value in 0..max_value."""
    return int(max_value).bit_length()


def position_bits(n_out: int) -> int:
    return math.ceil(math.log2(n_out))


@dataclass
class StreamSizes:
    wc_bits: int
    n_patch_bits: int
    d_patch_bits: int
    header_bits: int

    @property
    def total_bits(self) -> int:
        return self.wc_bits + self.n_patch_bits + self.d_patch_bits + self.header_bits


def _fields_to_bits(values: np.ndarray, width: int) -> np.ndarray:
    values = np.asarray(values, dtype=np.uint64).reshape(-1)
    if width == 0 or values.size == 0:
        return np.zeros(0, np.uint8)
    return ((values[:, None] >> np.arange(width, dtype=np.uint64)) & np.uint64(1)).astype(np.uint8).reshape(-1)


def _bits_to_fields(bits: np.ndarray, count: int, width: int) -> np.ndarray:
    if width == 0 or count == 0:
        return np.zeros(count, np.uint64)
    b = bits.reshape(count, width).astype(np.uint64)
    return (b << np.arange(width, dtype=np.uint64)).sum(axis=1)


def sizes(n_in: int, n_out: int, n_patch: np.ndarray, block_slices: int) -> StreamSizes:
    """n_patch: (q, l).  Sizes in bits of the four parts, summed over planes."""
    n_patch = np.asarray(n_patch)
    q, l = n_patch.shape
    np_bits = hdr = 0
    for p in range(q):
        for a in range(0, l, block_slices):
            blk = n_patch[p, a:a + block_slices]
            np_bits += blk.size * field_width(int(blk.max()))
            hdr += 8
    return StreamSizes(wc_bits=q * l * n_in, n_patch_bits=np_bits,
                       d_patch_bits=int(n_patch.sum()) * position_bits(n_out), header_bits=hdr)


def write_stream(n_in: int, n_out: int, w_c: np.ndarray, n_patch: np.ndarray, d_patch, block_slices: int) -> bytes:
    """w_c: (q, l) integers (bit j = x_j); n_patch: (q, l); d_patch: per plane, flat positions."""
    w_c = np.asarray(w_c)
    n_patch = np.asarray(n_patch)
    q, l = n_patch.shape
    parts = []
    for p in range(q):
        parts.append(_fields_to_bits(w_c[p], n_in))
        for a in range(0, l, block_slices):
            blk = n_patch[p, a:a + block_slices]
            w = field_width(int(blk.max()))
            parts.append(_fields_to_bits(np.array([w]), 8))
            parts.append(_fields_to_bits(blk, w))
        parts.append(_fields_to_bits(np.asarray(d_patch[p]), position_bits(n_out)))
    bits = np.concatenate(parts) if parts else np.zeros(0, np.uint8)
    return np.packbits(bits, bitorder="little").tobytes()


def read_stream(n_in: int, n_out: int, q: int, l: int, data: bytes, block_slices: int):
    """Inverse of write_stream: (w_c (q, l) uint64, n_patch (q, l) int64, d_patch list per plane)."""
    bits = np.unpackbits(np.frombuffer(data, dtype=np.uint8), bitorder="little")
    pos = 0
    w_c = np.zeros((q, l), np.uint64)
    n_patch = np.zeros((q, l), np.int64)
    d_patch = []
    for p in range(q):
        w_c[p] = _bits_to_fields(bits[pos:pos + l * n_in], l, n_in)
        pos += l * n_in
        for a in range(0, l, block_slices):
            cnt = min(block_slices, l - a)
            w = int(_bits_to_fields(bits[pos:pos + 8], 1, 8)[0])
            pos += 8
            n_patch[p, a:a + cnt] = _bits_to_fields(bits[pos:pos + cnt * w], cnt, w)
            pos += cnt * w
        tot = int(n_patch[p].sum())
        pb = position_bits(n_out)
        d_patch.append(_bits_to_fields(bits[pos:pos + tot * pb], tot, pb).astype(np.int64))
        pos += tot * pb
    return w_c, n_patch, d_patch
