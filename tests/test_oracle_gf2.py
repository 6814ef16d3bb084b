"""Pins for the oracle's XOR-gate network (Section 3.1)."""
import itertools

import numpy as np
import pytest

from oracle import gf2


def test_stacked_identity_repeats_input():
    n_in = 5
    M = np.vstack([np.eye(n_in, dtype=np.uint8)] * 3)
    x = np.array([[1, 0, 1, 1, 0], [0, 0, 0, 0, 1]], dtype=np.uint8)
    y = gf2.xor_network(M, x)
    assert np.array_equal(y, np.tile(x, (1, 3)))


def test_zero_and_all_ones_networks():
    rng = np.random.default_rng(0)
    x = rng.integers(0, 2, size=(50, 9), dtype=np.uint8)
    assert not gf2.xor_network(np.zeros((12, 9), np.uint8), x).any()
    y = gf2.xor_network(np.ones((12, 9), np.uint8), x)
    parity = x.sum(axis=1) % 2
    assert np.array_equal(y, np.repeat(parity[:, None], 12, axis=1))


def test_unit_inputs_give_columns():
    rng = np.random.default_rng(1)
    M = rng.integers(0, 2, size=(64, 16), dtype=np.uint8)
    y = gf2.xor_network(M, np.eye(16, dtype=np.uint8))
    assert np.array_equal(y, M.T)


def test_hand_computed_example():
    # y0 = x0^x2, y1 = x1, y2 = x0^x1^x2, y3 = 0
    M = np.array([[1, 0, 1], [0, 1, 0], [1, 1, 1], [0, 0, 0]], dtype=np.uint8)
    for x in itertools.product([0, 1], repeat=3):
        y = gf2.xor_network(M, np.array(x, dtype=np.uint8))
        assert list(y) == [x[0] ^ x[2], x[1], x[0] ^ x[1] ^ x[2], 0]


@pytest.mark.parametrize("n_out,n_in", [(8, 4), (64, 8), (64, 12), (200, 10)])
def test_row_parity_equals_column_xor_on_all_inputs(n_out, n_in):
    rng = np.random.default_rng(n_out * 100 + n_in)
    M = rng.integers(0, 2, size=(n_out, n_in), dtype=np.uint8)
    xs = gf2.int_to_bits(np.arange(1 << n_in), n_in)
    a = gf2.xor_network(M, xs)
    b = gf2.xor_network_columns(M, xs)
    assert np.array_equal(a, b)
    # brute force, bit by bit, on a sample of inputs
    for t in rng.integers(0, 1 << n_in, size=20):
        x = xs[t]
        for i in rng.integers(0, n_out, size=8):
            assert a[t, i] == (int(np.dot(M[i].astype(int), x.astype(int))) & 1)


def test_linearity():
    rng = np.random.default_rng(7)
    M = rng.integers(0, 2, size=(64, 24), dtype=np.uint8)
    x = rng.integers(0, 2, size=(100, 24), dtype=np.uint8)
    y = rng.integers(0, 2, size=(100, 24), dtype=np.uint8)
    assert np.array_equal(gf2.xor_network(M, x ^ y), gf2.xor_network(M, x) ^ gf2.xor_network(M, y))
    assert not gf2.xor_network(M, np.zeros(24, np.uint8)).any()


def test_bit_packing_roundtrip():
    rng = np.random.default_rng(3)
    b = rng.integers(0, 2, size=(10, 64), dtype=np.uint8)
    v = gf2.bits_to_int(b)
    assert v.dtype == np.uint64
    assert np.array_equal(gf2.int_to_bits(v, 64), b)
    assert gf2.bits_to_int(np.array([1, 0, 1, 1]))== 13
