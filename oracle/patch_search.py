"""Algorithm 1 (Patch-Searching) step by step, and the exhaustive search of Section 5.2.

Test infrastructure; small inputs only (pure Python loops).  One slice at a time, in
the paper's notation: w^q in {0, x, 1}^n_out given as (care, bits), M in {0,1}^(n_out x n_in).
"""
import numpy as np

from .gf2 import xor_network


def make_rref(mat: np.ndarray) -> np.ndarray:
    """Reduced row-echelon form over GF(2) of an augmented matrix (k, n_in + 1).

    Pivots are searched in the first n_in columns only (the last column is the
    right-hand side), from the lowest column index up.  Zero rows sink to the bottom.
    """
    a = np.array(mat, dtype=np.uint8) & 1
    k, ncol = a.shape
    r = 0
    for c in range(ncol - 1):
        piv = None
        for i in range(r, k):
            if a[i, c]:
                piv = i
                break
        if piv is None:
            continue
        if piv != r:
            a[[r, piv]] = a[[piv, r]]
        for i in range(k):
            if i != r and a[i, c]:
                a[i] ^= a[r]
        r += 1
        if r == k:
            break
    return a


def is_solved(rref: np.ndarray) -> bool:
    """The system is solvable iff no row reads 0 ... 0 | 1 (Section 3.3)."""
    coef = rref[:, :-1]
    rhs = rref[:, -1]
    return not bool(np.any((coef.sum(axis=1) == 0) & (rhs == 1)))


def solve_free_zero(rref: np.ndarray, n_in: int) -> np.ndarray:
    """A solution of a consistent RREF system with every free variable set to 0."""
    x = np.zeros(n_in, dtype=np.uint8)
    for row in rref:
        nz = np.flatnonzero(row[:-1])
        if nz.size:
            x[nz[0]] = row[-1]
    return x


def patch_search(care: np.ndarray, bits: np.ndarray, M: np.ndarray):
    """Algorithm 1.  Returns (n_patch, d_patch, w_c, dropped).

    care, bits: length-n_out arrays; bits is only read where care is set.
    d_patch: ascending 0-based positions to flip after decryption.
    dropped: the care positions whose equation was removed inside the loop.
    """
    M = np.asarray(M, dtype=np.uint8)
    n_out, n_in = M.shape
    mat = np.zeros((0, n_in + 1), dtype=np.uint8)
    dropped = []
    for i in np.flatnonzero(care):                       # only not-pruned bits, ascending
        row = np.concatenate([M[i], [1 if bits[i] else 0]]).astype(np.uint8)
        mat = np.vstack([mat, row[None, :]])             # append (M_i1 .. M_i,n_in, w_i)
        rref = make_rref(mat)
        if not is_solved(rref):
            mat = mat[:-1]                               # remove the last row again
            dropped.append(int(i))
    rref = make_rref(mat) if mat.shape[0] else mat
    w_c = solve_free_zero(rref, n_in)
    w_dd = xor_network(M, w_c)                           # decrypted slice
    d_patch = [int(i) for i in np.flatnonzero(care) if w_dd[i] != (1 if bits[i] else 0)]
    return len(d_patch), d_patch, w_c, dropped


def exhaustive_min_patches(care: np.ndarray, bits: np.ndarray, M: np.ndarray):
    """Section 5.2: list all 2^n_in inputs and their outputs, return the minimum
    number of mismatched care bits and one input attaining it."""
    M = np.asarray(M, dtype=np.uint8)
    n_out, n_in = M.shape
    xs = ((np.arange(1 << n_in)[:, None] >> np.arange(n_in)) & 1).astype(np.uint8)
    ys = xor_network(M, xs)
    idx = np.flatnonzero(care)
    target = np.asarray(bits, dtype=np.uint8)[idx]
    dist = (ys[:, idx] != target).sum(axis=1)
    best = int(dist.argmin())
    return int(dist[best]), xs[best]
