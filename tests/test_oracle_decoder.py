"""Pins for the oracle's decode / dequantise / product, and for the ratio formula."""
import math

import numpy as np
import pytest

from oracle import decoder, encoder, gf2, ratio
from synth_inputs import CONFIGS, bf16_bits_to_f32, make_workload


def _encoded(name, m, n):
    wl = make_workload(CONFIGS[name], m=m, n=n, keep_W=True)
    return wl, encoder.encode(wl.keep, wl.planes, wl.alpha, wl.M, wl.n)


def _hand_encoded():
    """A 2 x 8 matrix, n_out = 4, n_in = 2, written by hand (no encoder involved)."""
    M = np.array([[1, 0], [0, 1], [1, 1], [0, 0]], dtype=np.uint8)
    # slices: row0 -> s0,s1 ; row1 -> s2,s3.  w^c chosen by hand:
    w_c = np.array([[[1, 0], [0, 1], [1, 1], [0, 0]]], dtype=np.uint8)
    # M w^c: s0 -> 1,0,1,0 ; s1 -> 0,1,1,0 ; s2 -> 1,1,0,0 ; s3 -> 0,0,0,0
    n_patch = np.array([[0, 1, 0, 2]], dtype=np.int32)
    d_patch = [np.array([3, 0, 2], dtype=np.int64)]          # s1: flip bit 3; s3: flip bits 0, 2
    keep = np.array([[1, 1, 0, 1, 0, 1, 1, 1], [1, 0, 0, 0, 1, 0, 1, 1]], dtype=bool)
    alpha = np.array([[0.5, 2.0]], dtype=np.float32)
    return encoder.Encoded(m=2, n=8, n_pad=8, n_in=2, n_out=4, q=1, M=M, w_c=w_c,
                           n_patch=n_patch, d_patch=d_patch, keep=keep, alpha=alpha)


def test_hand_computed_decode():
    enc = _hand_encoded()
    dec = decoder.decrypt_planes(enc)[0].astype(int)
    assert dec.tolist() == [[1, 0, 1, 0, 0, 1, 1, 1], [1, 1, 0, 0, 1, 0, 1, 0]]
    W = decoder.dequantize_f32(enc)
    assert W.tolist() == [[0.5, -0.5, 0.0, -0.5, 0.0, 0.5, 0.5, 0.5], [2.0, 0.0, 0.0, 0.0, 2.0, 0.0, 2.0, -2.0]]
    X = np.arange(16, dtype=np.float64).reshape(8, 2)
    Y = decoder.spmm_f64(enc, X)
    want = [[sum(W[r, c] * X[c, b] for c in range(8)) for b in range(2)] for r in range(2)]
    assert np.allclose(Y, want, rtol=0, atol=1e-12)
    packed = decoder.pack_planes_u64(decoder.masked_planes(enc), 4)
    # masked: row0 = 1000|0111, row1 = 1000|1010 (element 0 of a slice is bit 0 of its word)
    assert packed.tolist() == [[0b0001, 0b1110, 0b0001, 0b0101]]


def test_dense_fp32_sums_planes_left_to_right():
    """Three planes with scales (1, 2^-24, 2^-24), written by hand: in fp32, (1 + 2^-24) + 2^-24 is 1 (each
    addition is a tie that rounds to the even neighbour 1.0) while 1 + (2^-24 + 2^-24) is 1 + 2^-23; with
    signs (-, -, -) the mirror image.  Only the left-to-right order gives exactly +-1."""
    M = np.array([[1, 0], [0, 1], [1, 1], [0, 0]], dtype=np.uint8)
    w_c = np.array([[[1, 0]], [[1, 0]], [[1, 0]]], dtype=np.uint8)       # every plane decodes to 1,0,1,0
    tiny = np.float32(2.0 ** -24)
    alpha = np.array([[1.0], [tiny], [tiny]], dtype=np.float32)
    enc = encoder.Encoded(m=1, n=4, n_pad=4, n_in=2, n_out=4, q=3, M=M, w_c=w_c,
                          n_patch=np.zeros((3, 1), dtype=np.int32), d_patch=[np.zeros(0, dtype=np.int64)] * 3,
                          keep=np.ones((1, 4), dtype=bool), alpha=alpha)
    W = decoder.dequantize_f32(enc)
    assert W.dtype == np.float32
    assert W.tolist() == [[1.0, -1.0, 1.0, -1.0]]
    right_to_left = np.float32(1.0) + (tiny + tiny)
    assert right_to_left != np.float32(1.0)                               # the other order is visibly different
    # the fp64 reference keeps all three terms
    assert decoder.dequantize_f64(enc)[0, 0] == 1.0 + 2.0 ** -23
    # a different order of the planes changes the fp32 result: (2^-24 + 2^-24) + 1 = 1 + 2^-23
    enc.alpha = alpha[::-1].copy()
    assert decoder.dequantize_f32(enc)[0, 0] == right_to_left


def test_masked_planes_equal_quantised_bits_exactly():
    wl, enc = _encoded("lstm", 64, 200)
    assert np.array_equal(decoder.masked_planes(enc), wl.planes)


def test_dense_decode_reproduces_the_quantiser_output():
    """alpha, mask and bits all survive: W_dec == keep * sum_p alpha_p (2 b_p - 1), an independent
    reconstruction straight from the generator's planes."""
    wl, enc = _encoded("fc6", 48, 320)
    want = np.zeros((wl.m, wl.n_pad), dtype=np.float64)
    for p in range(wl.cfg.q):
        want += (2.0 * wl.planes[p] - 1.0) * wl.alpha[p].astype(np.float64)[:, None]
    want = np.where(wl.keep, want, 0.0)[:, :wl.n]
    assert np.array_equal(decoder.dequantize_f64(enc), want)
    w32 = decoder.dequantize_f32(enc)
    assert w32.dtype == np.float32
    assert np.allclose(w32, want, rtol=1e-6, atol=0)
    # greedy binary coding shrinks the residual: a decoded 2-bit matrix is closer to W than 1-bit
    err2 = np.linalg.norm((want - wl.W)[wl.keep[:, :wl.n]])
    one = np.where(wl.keep, (2.0 * wl.planes[0] - 1.0) * wl.alpha[0].astype(np.float64)[:, None], 0.0)[:, :wl.n]
    err1 = np.linalg.norm((one - wl.W)[wl.keep[:, :wl.n]])
    assert err2 < 0.75 * err1


def test_ternary_special_case_and_identity_X():
    wl, enc = _encoded("tiny", 64, 128)
    enc.alpha[:] = 1.0
    W = decoder.dequantize_f64(enc)
    assert set(np.unique(W)) <= {-1.0, 0.0, 1.0}
    assert np.array_equal(W != 0, wl.keep[:, :wl.n])
    assert np.array_equal(W > 0, wl.planes[0][:, :wl.n])
    Y = decoder.spmm_f64(enc, np.eye(wl.n))
    assert np.array_equal(Y, W)
    x = np.random.default_rng(0).standard_normal((wl.n, 1))
    y = decoder.spmm_f64(enc, x)
    for r in (0, 17, 63):
        pos = x[(W[r] > 0), 0].sum()
        neg = x[(W[r] < 0), 0].sum()
        assert abs(y[r, 0] - (pos - neg)) < 1e-10


def test_bf16_rounding_of_dense_output():
    vals = np.array([1.0, -1.0, 0.0, 1.00390625, 1.01171875, 3.0e38, 1.0e-40, -2.5], dtype=np.float32)
    got = decoder.round_f32_to_bf16_bits(vals)
    # 1.00390625 = 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80);
    # 1.01171875 = 1 + 2^-7 + 2^-8 is a tie between 0x3F81 and 0x3F82 -> even (0x3F82)
    assert got[:5].tolist() == [0x3F80, 0xBF80, 0x0000, 0x3F80, 0x3F82]
    back = bf16_bits_to_f32(got)
    assert np.all(np.abs(back[[5, 7]] - vals[[5, 7]]) <= np.abs(vals[[5, 7]]) * 2.0 ** -8)


def test_ratio_hand_computed(golden):
    # m n = 128, n_out = 8, n_in = 4 -> l = 16; patches p = [0]*13 + [1, 2, 1]
    p = np.array([0] * 13 + [1, 2, 1])
    # literal width ceil(lg 2) = 1 bit; +1 reading ceil(lg 3) = 2 bits; d_patch entries ceil(lg 8) = 3 bits
    lit = 128 / (0.5 * 128 + 16 * 1 + 4 * 3)
    hon = 128 / (0.5 * 128 + 16 * 2 + 4 * 3)
    assert math.isclose(ratio.compression_ratio(128, 4, 8, p, literal=True), lit)
    assert math.isclose(ratio.compression_ratio(128, 4, 8, p), hon)
    assert math.isclose(ratio.memory_reduction(128, 4, 8, p), 1 - 1 / hon)
    # no patches at all: r = n_out / n_in; at n_in = n_out (1 - S) this is 1 / (1 - S)
    assert math.isclose(ratio.compression_ratio(6400, 20, 200, np.zeros(32, int)), float(golden["ideal_ratio_S090"]))
    assert ratio.n_patch_field_bits(1, literal=True) == 0 and ratio.n_patch_field_bits(1) == 1
    assert ratio.n_patch_field_bits(4, literal=True) == 2 and ratio.n_patch_field_bits(4) == 3
    assert math.ceil(math.log2(64)) == int(golden["d_patch_bits_n_out_64"])


@pytest.mark.parametrize("name,base", [("tiny", 0.25), ("fc6", 0.5), ("large_q1", 0.125), ("large_q2", 0.25)])
def test_bits_per_weight_is_stream_plus_patch_overhead(name, base):
    """bits/weight = (n_in / n_out) q + patch overhead (no column padding in these shapes)."""
    wl, enc = _encoded(name, 128, 512)
    bpw = ratio.bits_per_weight(enc)
    over = 0.0
    for p in range(enc.q):
        over += enc.l * ratio.n_patch_field_bits(int(enc.n_patch[p].max())) + 6 * int(enc.n_patch[p].sum())
    assert math.isclose(bpw, base + over / (wl.m * wl.n), rel_tol=1e-12)
    assert bpw >= base
    # blocked n_patch assignment (Section 5.2) can only shrink the n_patch fields
    assert ratio.bits_per_weight(enc, blocks=16) <= bpw + 1e-12


def test_lstm_shape_counts_padding_in_the_stream():
    wl, enc = _encoded("lstm", 32, 3000)
    assert wl.n_pad == 3008 and enc.l == 32 * 47
    base = 3 * (24 / 64) * 3008 / 3000
    assert ratio.bits_per_weight(enc) >= base
    assert math.isclose(base, 1.128, abs_tol=5e-4)
