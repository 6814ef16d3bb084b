"""Offline encoder: slicing, Algorithm 1 over all slices, compressed format (test infrastructure).

Section 3.1: every binary matrix W_i^q (one per quantisation bit) is flattened and cut
into l vectors of n_out elements.  Section 3.2 / Algorithm 1: each vector w^q is encrypted
to w^c (n_in bits) plus the patch data n_patch, d_patch.  The compressed format is
(w^c_1..l, n_patch, d_patch) per bit-plane, plus the pruning mask and the per-row scales
that the quantiser produced.

`encode_plane` runs Algorithm 1 for all slices at once: the loop over care positions is
the paper's loop; instead of recomputing the RREF from scratch after every append it keeps
the RREF of the accepted rows and reduces the new row against it (the appended row makes
the system unsolvable exactly when it reduces to 0 ... 0 | 1).  `patch_search.patch_search`
is the from-scratch version; the tests require both to agree bit for bit.
"""
from dataclasses import dataclass
from typing import List

import numpy as np

from .gf2 import xor_network


def slice_plane(a: np.ndarray, n_out: int) -> np.ndarray:
    """Flatten a (m, n_pad) matrix row-major and cut it into (l, n_out) vectors."""
    m, n_pad = a.shape
    if (m * n_pad) % n_out:
        raise ValueError("matrix size must be a multiple of n_out after column padding")
    return a.reshape(-1, n_out)


def _lowest_set_bit_index(v: np.ndarray) -> np.ndarray:
    """Index of the lowest set bit of each nonzero uint64 (float64 log2 of an exact power of two)."""
    low = v & (~v + np.uint64(1))
    return np.rint(np.log2(low.astype(np.float64))).astype(np.int64)


def encode_plane(care: np.ndarray, bits: np.ndarray, M: np.ndarray):
    """Algorithm 1 for every slice of one bit-plane.

    care, bits: bool (l, n_out).  M: {0,1} (n_out, n_in), n_in <= 62.
    Returns (w_c uint8 (l, n_in), n_patch int32 (l,), d_patch int64 flat, slice order then ascending).
    """
    M = np.asarray(M, dtype=np.uint8)
    n_out, n_in = M.shape
    l = care.shape[0]
    one = np.uint64(1)
    rhs_bit = np.uint64(n_in)
    coef_mask = np.uint64((1 << n_in) - 1)
    # row i of M as an integer: bit j = M[i, j]
    M_int = [np.uint64(sum(int(M[i, j]) << j for j in range(n_in))) for i in range(n_out)]
    # basis[s, j]: accepted (reduced) row of slice s whose pivot is column j, 0 if none.
    basis = np.zeros((l, n_in), dtype=np.uint64)
    dropped = np.zeros((l, n_out), dtype=bool)
    for i in range(n_out):                                # care positions in ascending order
        idx = np.flatnonzero(care[:, i])
        if idx.size == 0:
            continue
        row = M_int[i] | (bits[idx, i].astype(np.uint64) << rhs_bit)
        B = basis[idx]
        for j in range(n_in):                             # reduce against the accepted rows
            hit = (((row >> np.uint64(j)) & one) == one) & (B[:, j] != 0)
            row = np.where(hit, row ^ B[:, j], row)
        coef = row & coef_mask
        unsolvable = (coef == 0) & ((row >> rhs_bit) == one)
        dropped[idx[unsolvable], i] = True                # row 0..0|1: the equation is removed
        new = np.flatnonzero(coef != 0)
        if new.size:
            piv = _lowest_set_bit_index(coef[new])
            rnew = row[new]
            Bn = B[new]
            for j in range(n_in):                         # keep the accepted rows reduced
                hit = ((Bn[:, j] >> piv.astype(np.uint64)) & one) == one
                Bn[:, j] = np.where(hit, Bn[:, j] ^ rnew, Bn[:, j])
            Bn[np.arange(new.size), piv] = rnew
            B[new] = Bn
            basis[idx] = B
    # solve with free variables = 0: x_j is the right-hand side of the row with pivot j
    w_c = ((basis >> rhs_bit) & one).astype(np.uint8)
    # decrypt and compare on the care positions
    w_dd = xor_network(M, w_c).astype(bool)
    mism = care & (w_dd != bits)
    if not np.array_equal(mism, dropped):
        raise AssertionError("mismatch set differs from the set of removed equations")
    n_patch = mism.sum(axis=1).astype(np.int32)
    d_patch = np.nonzero(mism)[1].astype(np.int64)        # row-major nonzero: slice order, ascending
    return w_c, n_patch, d_patch


def encode_plane_exhaustive(care: np.ndarray, bits: np.ndarray, M: np.ndarray):
    """Section 5.2 (minimising n_patch for small n_in): list all 2^n_in inputs with their outputs
    through the XOR-gate network and keep, per slice, an input with the fewest mismatched care
    bits; among those the smallest one as an integer (bit j = x_j).  Same return value as
    `encode_plane`.  Work grows as l * 2^n_in * n_out: meant for n_in <= 16."""
    M = np.asarray(M, dtype=np.uint8)
    n_out, n_in = M.shape
    if n_in > 16:
        raise ValueError("exhaustive search is limited to n_in <= 16")
    xs = ((np.arange(1 << n_in)[:, None] >> np.arange(n_in)) & 1).astype(np.uint8)
    ys = xor_network(M, xs).astype(bool)                         # (2^n_in, n_out): every output
    care = np.asarray(care, dtype=bool)
    bits = np.asarray(bits, dtype=bool)
    l = care.shape[0]
    w_c = np.zeros((l, n_in), dtype=np.uint8)
    mism = np.zeros((l, n_out), dtype=bool)
    step = max(1, (1 << 22) >> n_in)                             # slices per chunk
    ysf = ys.astype(np.float64)
    for a in range(0, l, step):
        c = care[a:a + step]
        t = bits[a:a + step] & c
        # mismatches of input v on slice s = sum over care bits of (y_v xor t_s)
        #   = sum_i c_si y_vi + sum_i t_si - 2 sum_i t_si y_vi   (t is zero outside the care set);
        # small integers, exact in float64
        dist = (c.astype(np.float64) - 2.0 * t.astype(np.float64)) @ ysf.T + t.sum(axis=1)[:, None]
        best = np.argmin(dist, axis=1)                           # first minimum = smallest integer
        w_c[a:a + step] = xs[best]
        mism[a:a + step] = c & (ys[best] != bits[a:a + step])
    n_patch = mism.sum(axis=1).astype(np.int32)
    d_patch = np.nonzero(mism)[1].astype(np.int64)
    return w_c, n_patch, d_patch


@dataclass
class Encoded:
    """The compressed format of Section 3.2 for one weight matrix (all bit-planes)."""
    m: int
    n: int
    n_pad: int
    n_in: int
    n_out: int
    q: int
    M: np.ndarray                 # uint8 (n_out, n_in)
    w_c: np.ndarray               # uint8 (q, l, n_in)
    n_patch: np.ndarray           # int32 (q, l)
    d_patch: List[np.ndarray]     # per plane: int64 flat list, slice order then ascending position
    keep: np.ndarray              # bool (m, n_pad), the pruning mask (index stream)
    alpha: np.ndarray             # float32 (q, m)

    @property
    def l(self) -> int:
        return self.m * self.n_pad // self.n_out


def encode(keep: np.ndarray, planes: np.ndarray, alpha: np.ndarray, M: np.ndarray, n: int,
           exhaustive: bool = False) -> Encoded:
    """Encrypt all bit-planes of a pruned, binary-coded matrix.

    keep: bool (m, n_pad); planes: bool (q, m, n_pad); alpha: float32 (q, m); n: real column count.
    exhaustive: the 2^n_in search of Section 5.2 in place of Algorithm 1.
    """
    M = np.asarray(M, dtype=np.uint8)
    n_out, n_in = M.shape
    q, m, n_pad = planes.shape
    care = slice_plane(keep, n_out)
    w_c, n_patch, d_patch = [], [], []
    one_plane = encode_plane_exhaustive if exhaustive else encode_plane
    for p in range(q):
        wc, npch, dp = one_plane(care, slice_plane(planes[p], n_out), M)
        w_c.append(wc)
        n_patch.append(npch)
        d_patch.append(dp)
    return Encoded(m=m, n=n, n_pad=n_pad, n_in=n_in, n_out=n_out, q=q, M=M,
                   w_c=np.stack(w_c), n_patch=np.stack(n_patch), d_patch=d_patch,
                   keep=np.asarray(keep, dtype=bool), alpha=np.asarray(alpha, dtype=np.float32))
