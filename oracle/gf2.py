"""XOR-gate network over GF(2) (test infrastructure; see package docstring).

Section 3.1: the network is a fixed binary matrix M of shape (n_out, n_in); output
bit i is the XOR of the inputs j with M[i, j] = 1, i.e. y = M x over GF(2).
"""
import numpy as np


def xor_network(M: np.ndarray, x: np.ndarray) -> np.ndarray:
    """y[..., i] = (sum_j M[i, j] * x[..., j]) mod 2, the definition of Section 3.1.

    M: {0,1} array (n_out, n_in); x: {0,1} array (..., n_in).  Returns uint8 (..., n_out).
    The sum is taken in float64 (exact for these small integers) so that BLAS can
    serve as the matmul step.
    """
    M = np.asarray(M)
    x = np.asarray(x)
    s = x.astype(np.float64) @ M.astype(np.float64).T
    return (np.rint(s).astype(np.int64) & 1).astype(np.uint8)


def xor_network_columns(M: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Same map written as the XOR of the columns of M selected by the set bits of x.

    A second, independent formulation used only to cross-check `xor_network`.
    """
    M = np.asarray(M, dtype=np.uint8)
    x = np.asarray(x, dtype=np.uint8)
    y = np.zeros(x.shape[:-1] + (M.shape[0],), dtype=np.uint8)
    for j in range(M.shape[1]):
        y ^= x[..., j:j + 1] & M[:, j]
    return y


def bits_to_int(bits: np.ndarray) -> np.ndarray:
    """Pack the last axis (bit j has weight 2^j) into uint64."""
    bits = np.asarray(bits, dtype=np.uint64)
    w = np.uint64(1) << np.arange(bits.shape[-1], dtype=np.uint64)
    return (bits * w).sum(axis=-1, dtype=np.uint64)


def int_to_bits(v: np.ndarray, nbits: int) -> np.ndarray:
    """Unpack uint64 into a trailing axis of nbits {0,1} uint8 values (bit j = weight 2^j)."""
    v = np.asarray(v, dtype=np.uint64)
    sh = np.arange(nbits, dtype=np.uint64)
    return ((v[..., None] >> sh) & np.uint64(1)).astype(np.uint8)
