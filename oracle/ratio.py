"""Compression ratio r of Section 3.2, Eq. (2) (test infrastructure).

r = m n / ( (n_in / n_out) m n  +  l * width(n_patch)  +  sum_j p_j * ceil(lg n_out) )

per bit-plane, with l = ceil(m n / n_out) slices and p_j the j-th n_patch.  The printed
field width ceil(lg max(p)) cannot hold the value max(p) when max(p) is a power of two
(it is 0 bits for max(p) = 1), so both that literal width and ceil(lg(max(p) + 1)) are
offered; the second is the one reported as the honest figure.
"""
import math

import numpy as np


def n_patch_field_bits(max_p: int, literal: bool = False) -> int:
    if max_p <= 0:
        return 0
    if literal:
        return math.ceil(math.log2(max_p)) if max_p > 1 else 0
    return math.ceil(math.log2(max_p + 1))


def compressed_bits(mn: int, n_in: int, n_out: int, n_patch: np.ndarray, literal: bool = False) -> float:
    """Bits of one encrypted bit-plane: w^c stream + n_patch fields + d_patch entries.

    `mn` is the element count the slices cover (the padded matrix)."""
    n_patch = np.asarray(n_patch)
    l = math.ceil(mn / n_out)
    if n_patch.size != l:
        raise ValueError("one n_patch per slice expected")
    wc_bits = (n_in / n_out) * mn
    np_bits = l * n_patch_field_bits(int(n_patch.max(initial=0)), literal)
    dp_bits = int(n_patch.sum()) * math.ceil(math.log2(n_out))
    return wc_bits + np_bits + dp_bits


def compression_ratio(mn: int, n_in: int, n_out: int, n_patch: np.ndarray, literal: bool = False) -> float:
    return mn / compressed_bits(mn, n_in, n_out, n_patch, literal)


def memory_reduction(mn: int, n_in: int, n_out: int, n_patch: np.ndarray, literal: bool = False) -> float:
    """1 - 1/r, the quantity plotted in Section 3.3."""
    return 1.0 - 1.0 / compression_ratio(mn, n_in, n_out, n_patch, literal)


def bits_per_weight(enc, literal: bool = False, blocks: int = 1) -> float:
    """Quantisation-stream bits per real weight (m*n, not the padded count) over all planes.

    blocks > 1 applies the blocked n_patch assignment of Section 5.2: the n_patch field
    width is chosen per block of consecutive slices instead of once for the plane."""
    total = 0.0
    mn_pad = enc.m * enc.n_pad
    for p in range(enc.q):
        npch = np.asarray(enc.n_patch[p])
        wc_bits = (enc.n_in / enc.n_out) * mn_pad
        dp_bits = int(npch.sum()) * math.ceil(math.log2(enc.n_out))
        np_bits = 0
        for blk in np.array_split(npch, blocks):
            np_bits += blk.size * n_patch_field_bits(int(blk.max(initial=0)), literal)
        total += wc_bits + np_bits + dp_bits
    return total / (enc.m * enc.n)
