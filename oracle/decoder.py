"""Online path by its plain definition (test infrastructure): decrypt, patch, mask,
dequantise, multiply.

Section 3.1: w = M w^c over GF(2).  Section 3.2 / 5.1: the bits at the d_patch positions of
each slice are flipped (n_patch of them per slice).  The pruning mask zeroes the don't-care
positions (Fig. 11, stream (A)).  Binary-coding dequantisation: W[r, c] = keep * sum_p alpha[p, r] *
(2 b_p[r, c] - 1) (Section 3.1, multi-bit quantised weights as binary matrices with scales).
The product Y = W X is the consumer the paper's Fig. 1 measures.
"""
import numpy as np

from .encoder import Encoded
from .gf2 import xor_network


def decrypt_planes(enc: Encoded) -> np.ndarray:
    """Decrypted and patched bit-planes, bool (q, m, n_pad); don't-care positions hold
    whatever the XOR network produced (not yet masked)."""
    out = np.empty((enc.q, enc.l, enc.n_out), dtype=bool)
    for p in range(enc.q):
        w = xor_network(enc.M, enc.w_c[p]).astype(bool)                 # w = M w^c
        slice_of_patch = np.repeat(np.arange(enc.l), enc.n_patch[p])    # n_patch entries per slice
        if slice_of_patch.size != enc.d_patch[p].size:
            raise ValueError("n_patch does not add up to the length of d_patch")
        np.logical_xor.at(w, (slice_of_patch, enc.d_patch[p]), True)    # flip
        out[p] = w
    return out.reshape(enc.q, enc.m, enc.n_pad)


def masked_planes(enc: Encoded) -> np.ndarray:
    """Bit-planes with pruned and padding positions forced to 0, bool (q, m, n_pad)."""
    return decrypt_planes(enc) & enc.keep[None]


def pack_planes_u64(planes: np.ndarray, n_out: int = 64) -> np.ndarray:
    """(q, m, n_pad) bool -> (q, l) uint64, bit i of word s = element i of slice s."""
    q = planes.shape[0]
    sl = planes.reshape(q, -1, n_out).astype(np.uint64)
    w = np.uint64(1) << np.arange(n_out, dtype=np.uint64)
    return (sl * w).sum(axis=-1, dtype=np.uint64)


def dequantize_f32(enc: Encoded) -> np.ndarray:
    """Dense fp32 weights (m, n): planes summed left to right in fp32, pruned -> +0.0."""
    b = decrypt_planes(enc)
    acc = np.zeros((enc.m, enc.n_pad), dtype=np.float32)
    for p in range(enc.q):
        sign = np.where(b[p], np.float32(1.0), np.float32(-1.0))
        term = (sign * enc.alpha[p][:, None]).astype(np.float32)        # exact: +-alpha
        acc = term if p == 0 else (acc + term).astype(np.float32)
    return np.where(enc.keep, acc, np.float32(0.0))[:, :enc.n]


def round_f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) of fp32 values, round-to-nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    keep_hi = u >> np.uint64(16)
    rem = u & np.uint64(0xFFFF)
    half = np.uint64(0x8000)
    up = (rem > half) | ((rem == half) & ((keep_hi & np.uint64(1)) == np.uint64(1)))
    return (keep_hi + up.astype(np.uint64)).astype(np.uint16)


def dequantize_f64(enc: Encoded) -> np.ndarray:
    """Dense weights in fp64 from the exact values of the fp32 scales, (m, n)."""
    b = decrypt_planes(enc)
    acc = np.zeros((enc.m, enc.n_pad), dtype=np.float64)
    for p in range(enc.q):
        acc += np.where(b[p], 1.0, -1.0) * enc.alpha[p].astype(np.float64)[:, None]
    return np.where(enc.keep, acc, 0.0)[:, :enc.n]


def spmm_f64(enc: Encoded, X_exact: np.ndarray) -> np.ndarray:
    """Y = W X in fp64; X_exact holds exactly the stored activation values (n, B)."""
    return dequantize_f64(enc) @ np.asarray(X_exact, dtype=np.float64)
