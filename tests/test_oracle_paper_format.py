"""Pins of oracle/paper_format.py: a stream written out by hand, the sizes against Eq. (2)'s terms
(oracle/ratio.py, itself pinned by a hand-computed r), and the round trip."""
import math

import numpy as np
import pytest

from helpers import encoded_workload
from oracle import paper_format, ratio


def test_hand_written_stream():
    """q = 1, l = 3 slices, n_in = 4, n_out = 8 (3-bit positions), blocks of 2 slices.
    w^c = 0b0101, 0b0011, 0b1000; n_patch = 2, 0, 1; d_patch = [1, 6], [], [7].
      w^c fields, low bit first:        1010 1100 0001
      block 0: width 2 -> 01000000, fields 2 -> 01, 0 -> 00
      block 1: width 1 -> 10000000, field 1 -> 1
      positions (3 bits): 1 -> 100, 6 -> 011, 7 -> 111
    Bit string:  1010 1100 0001 01000000 01 00 10000000 1 100 011 111
    """
    data = paper_format.write_stream(4, 8, np.array([[0b0101, 0b0011, 0b1000]]), np.array([[2, 0, 1]]),
                                     [np.array([1, 6, 7])], block_slices=2)
    bitstr = "101011000001" + "01000000" + "0100" + "10000000" + "1" + "100011111"
    want = np.packbits(np.array([int(c) for c in bitstr], np.uint8), bitorder="little").tobytes()
    assert data == want
    s = paper_format.sizes(4, 8, np.array([[2, 0, 1]]), 2)
    assert (s.wc_bits, s.n_patch_bits, s.d_patch_bits, s.header_bits) == (12, 5, 9, 16)
    assert s.total_bits == len(bitstr)
    w_c, n_patch, d_patch = paper_format.read_stream(4, 8, 1, 3, data, 2)
    assert w_c.tolist() == [[5, 3, 8]] and n_patch.tolist() == [[2, 0, 1]] and d_patch[0].tolist() == [1, 6, 7]


def test_field_widths():
    assert [paper_format.field_width(v) for v in (0, 1, 2, 3, 4, 7, 8, 255, 256)] == [0, 1, 2, 2, 3, 3, 4, 8, 9]
    assert [paper_format.position_bits(n) for n in (64, 128, 192, 256)] == [6, 7, 8, 8]


@pytest.mark.parametrize("name,m,n,n_out,n_in,S", [("large_q1", 64, 512, 64, 8, None), ("lstm", 45, 200, 192, 20, None),
                                                  ("fc6", 33, 130, 128, 16, 0.7), ("tiny", 70, 256, 64, 13, None)])
def test_sizes_against_eq2_and_round_trip(name, m, n, n_out, n_in, S):
    wl, enc = encoded_workload(name, m, n, S=S, n_out=n_out, n_in=n_in)
    w_c = (enc.w_c.astype(np.uint64) << np.arange(enc.n_in, dtype=np.uint64)).sum(axis=2)
    # one block per plane: the three counted parts are Eq. (2)'s denominator, plane by plane
    s = paper_format.sizes(enc.n_in, enc.n_out, enc.n_patch, enc.l)
    eq2 = sum(ratio.compressed_bits(enc.m * enc.n_pad, enc.n_in, enc.n_out, enc.n_patch[p]) for p in range(enc.q))
    assert s.wc_bits + s.n_patch_bits + s.d_patch_bits == pytest.approx(eq2, abs=1e-6)
    assert s.header_bits == 8 * enc.q
    for blk in (enc.l, 32, 7):
        s = paper_format.sizes(enc.n_in, enc.n_out, enc.n_patch, blk)
        data = paper_format.write_stream(enc.n_in, enc.n_out, w_c, enc.n_patch, enc.d_patch, blk)
        assert len(data) == math.ceil(s.total_bits / 8)
        w2, np2, dp2 = paper_format.read_stream(enc.n_in, enc.n_out, enc.q, enc.l, data, blk)
        assert np.array_equal(w2, w_c) and np.array_equal(np2, enc.n_patch)
        assert all(np.array_equal(a, b) for a, b in zip(dp2, enc.d_patch))
    # smaller blocks never need more n_patch bits (Section 5.2's point), headers aside
    assert paper_format.sizes(enc.n_in, enc.n_out, enc.n_patch, 32).n_patch_bits <= \
        paper_format.sizes(enc.n_in, enc.n_out, enc.n_patch, enc.l).n_patch_bits
