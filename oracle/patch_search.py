"""Algorithm 1 of Section 3.3 (patch searching) one slice at a time, and the exhaustive search of Section 5.2.

Test infrastructure; small inputs only (pure Python loops).  One slice at a time, in
the paper's notation: w^q in {0, x, 1}^n_out given as (care, bits), M in {0,1}^(n_out x n_in).
"""
import numpy as np

from .gf2 import xor_network


def row_reduce(system: np.ndarray) -> np.ndarray:
    """Reduced row-echelon form over GF(2) of a system [coefficients | right-hand side], shape (k, n_in + 1).

    Only the n_in coefficient columns can hold a pivot; they are scanned from the lowest index up.
    Rows without a pivot end up below the others.
    """
    a = np.array(system, dtype=np.uint8) & 1
    n_rows, n_cols = a.shape
    top = 0                                           # rows above `top` already own a pivot
    for col in range(n_cols - 1):
        below = np.flatnonzero(a[top:, col])
        if below.size == 0:
            continue
        src = top + int(below[0])
        if src != top:
            a[[top, src]] = a[[src, top]]
        others = np.flatnonzero(a[:, col])
        others = others[others != top]
        a[others] ^= a[top]                           # clear the column everywhere else
        top += 1
        if top == n_rows:
            break
    return a


def has_solution(reduced: np.ndarray) -> bool:
    """A reduced system is solvable unless one of its rows says 0 = 1 (Section 3.3)."""
    empty_left = ~reduced[:, :-1].any(axis=1)
    return not bool((empty_left & (reduced[:, -1] == 1)).any())


def solution_with_free_zero(reduced: np.ndarray, n_in: int) -> np.ndarray:
    """The solution of a solvable reduced system in which every variable without a pivot is 0."""
    x = np.zeros(n_in, dtype=np.uint8)
    for row in reduced:
        cols = np.flatnonzero(row[:-1])
        if cols.size:
            x[cols[0]] = row[-1]
    return x


def patch_search(care: np.ndarray, bits: np.ndarray, M: np.ndarray):
    """Algorithm 1, Section 3.3.  Returns (n_patch, d_patch, w_c, dropped).

    care, bits: length-n_out arrays; bits is only read where care is set.  Every kept weight i asks for
    (row i of M) . w^c = bits[i]; the requests are taken in ascending position and one is accepted only if
    the accepted ones together with it can still be met.  w^c then solves the accepted requests, and the
    patches are the kept positions that M w^c gets wrong.
    d_patch: ascending 0-based positions to flip after decryption.
    dropped: the kept positions whose request was refused.
    """
    M = np.asarray(M, dtype=np.uint8)
    n_out, n_in = M.shape
    wanted = [1 if bits[i] else 0 for i in range(n_out)]
    accepted = np.zeros((0, n_in + 1), dtype=np.uint8)      # one row [M_i | wanted bit] per accepted request
    dropped = []
    for i in np.flatnonzero(care):
        trial = np.vstack([accepted, np.append(M[i], wanted[i]).astype(np.uint8)[None, :]])
        if has_solution(row_reduce(trial)):
            accepted = trial
        else:
            dropped.append(int(i))
    w_c = solution_with_free_zero(row_reduce(accepted), n_in) if accepted.shape[0] else np.zeros(n_in, np.uint8)
    decrypted = xor_network(M, w_c)
    d_patch = [int(i) for i in np.flatnonzero(care) if decrypted[i] != wanted[i]]
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


def exhaustive_min_patches_in_parts(care: np.ndarray, bits: np.ndarray, M: np.ndarray, part_bits: int = 16):
    """Section 5.2 for wider inputs (the paper calls n_in below 30 practical): the same listing of all 2^n_in
    inputs, taken 2^part_bits inputs at a time so that it fits in memory.  Returns (fewest mismatched care bits,
    the smallest input, read as an integer with bit j = x_j, that attains it, as a bit vector).

    The parts are visited in ascending order of the inputs and a later part replaces the best so far only when
    it is strictly better, so that among equally good inputs the smallest integer wins, as in the one-part listing.
    """
    M = np.asarray(M, dtype=np.uint8)
    n_out, n_in = M.shape
    part_bits = min(part_bits, n_in)
    idx = np.flatnonzero(care)
    target = np.asarray(bits, dtype=np.uint8)[idx]
    low = np.arange(1 << part_bits, dtype=np.int64)
    best_dist, best_x = None, None
    for high in range(1 << (n_in - part_bits)):
        ints = low + (high << part_bits)
        xs = ((ints[:, None] >> np.arange(n_in)) & 1).astype(np.uint8)
        ys = xor_network(M, xs)
        dist = (ys[:, idx] != target).sum(axis=1)
        k = int(dist.argmin())                      # first minimum of the part = its smallest input
        if best_dist is None or int(dist[k]) < best_dist:
            best_dist, best_x = int(dist[k]), xs[k]
    return best_dist, best_x

