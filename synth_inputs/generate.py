"""Seeded generators for the synthetic workloads (NumPy only, no method arithmetic).

Recipe per configuration:
  W      m x n fp32 Gaussian(0, sigma), PCG64(seed_W)
  mask   global magnitude pruning: exactly floor(S*m*n) entries of smallest |w| are
         pruned, ties broken by flat (row-major) index, lower index pruned first
  planes greedy residual binary coding of the kept weights, per row:
         alpha_p = mean |r| over the kept entries of the row, b_p = [r >= 0],
         r <- r - alpha_p*(2*b_p - 1); computed in fp64, alpha stored as fp32;
         a row without kept weights gets alpha_p = 0
  M      n_out x n_in iid Bernoulli(1/2), PCG64(seed_M), kept exactly as drawn
  X      n x B Gaussian(0, 1), PCG64(seed_X); for bf16 the fp32 draw is rounded to
         nearest-even and stored as the 16 high bits
Columns are padded with pruned (don't-care) columns up to a multiple of n_out so
that a slice never straddles two rows.
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np

from .configs import WorkloadConfig


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def draw_W(m: int, n: int, sigma: float, seed: int) -> np.ndarray:
    w = _rng(seed).standard_normal((m, n), dtype=np.float32)
    if sigma != 1.0:
        w *= np.float32(sigma)
    return w


def draw_M(n_out: int, n_in: int, seed: int) -> np.ndarray:
    """XOR-network connectivity, uint8 {0,1} of shape (n_out, n_in)."""
    return _rng(seed).integers(0, 2, size=(n_out, n_in), dtype=np.uint8)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def draw_X(n: int, B: int, dtype: str, seed: int):
    """Returns (stored, exact_f32): `stored` is fp32 values or uint16 bf16 patterns,
    `exact_f32` holds exactly the values the stored array represents."""
    x = _rng(seed).standard_normal((n, B), dtype=np.float32)
    if dtype == "f32":
        return x, x
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x)
        return bits, bf16_bits_to_f32(bits)
    raise ValueError(dtype)


def magnitude_mask(W: np.ndarray, S: float) -> np.ndarray:
    """Boolean keep-mask; exactly floor(S*size) entries pruned, stable tie-break."""
    a = np.abs(W).ravel()
    k = int(np.floor(S * a.size))
    keep = np.ones(a.size, dtype=bool)
    if k > 0:
        thr = np.partition(a, k - 1)[k - 1]
        below = a < thr
        keep[below] = False
        need = k - int(below.sum())
        if need > 0:
            ties = np.flatnonzero(a == thr)
            keep[ties[:need]] = False
    return keep.reshape(W.shape)


def greedy_binary_code(W: np.ndarray, keep: np.ndarray, q: int):
    """Returns (planes bool[q,m,n], alpha float32[q,m]); pruned positions get bit 0."""
    m, n = W.shape
    r = np.where(keep, W.astype(np.float64), 0.0)
    cnt = keep.sum(axis=1).astype(np.float64)
    planes = np.zeros((q, m, n), dtype=bool)
    alpha = np.zeros((q, m), dtype=np.float32)
    for p in range(q):
        s = np.abs(r).sum(axis=1)
        a = np.divide(s, cnt, out=np.zeros_like(s), where=cnt > 0)
        b = (r >= 0) & keep
        planes[p] = b
        alpha[p] = a.astype(np.float32)
        r = np.where(keep, r - a[:, None] * (2.0 * b - 1.0), 0.0)
    return planes, alpha


def pad_columns(a: np.ndarray, n_pad: int) -> np.ndarray:
    """Pad the last axis with zeros (False) up to n_pad columns."""
    n = a.shape[-1]
    if n == n_pad:
        return a
    pad = [(0, 0)] * (a.ndim - 1) + [(0, n_pad - n)]
    return np.pad(a, pad)


@dataclass
class Workload:
    cfg: WorkloadConfig
    m: int
    n: int
    n_pad: int
    keep: np.ndarray      # bool [m, n_pad]; padding columns False
    planes: np.ndarray    # bool [q, m, n_pad]; pruned/padding positions False
    alpha: np.ndarray     # float32 [q, m]
    M: np.ndarray         # uint8 [n_out, n_in]
    W: Optional[np.ndarray] = None  # the fp32 draw (kept only on request)

    def X(self, B: int, dtype: Optional[str] = None):
        return draw_X(self.n, B, dtype or self.cfg.x_dtype, self.cfg.seed_X + 1000 * B)


def make_workload(cfg: WorkloadConfig, m: Optional[int] = None, n: Optional[int] = None,
                  keep_W: bool = False) -> Workload:
    """Build a workload; `m`/`n` override the shape (same recipe, smaller matrix)."""
    m = cfg.m if m is None else m
    n = cfg.n if n is None else n
    W = draw_W(m, n, cfg.sigma, cfg.seed_W)
    keep = magnitude_mask(W, cfg.S)
    planes, alpha = greedy_binary_code(W, keep, cfg.q)
    n_pad = -(-n // cfg.n_out) * cfg.n_out
    return Workload(
        cfg=cfg, m=m, n=n, n_pad=n_pad,
        keep=pad_columns(keep, n_pad), planes=pad_columns(planes, n_pad), alpha=alpha,
        M=draw_M(cfg.n_out, cfg.n_in, cfg.seed_M), W=W if keep_W else None,
    )


def random_care_problem(n_elem: int, S: float, seed: int):
    """The paper's synthetic-data setting (Section 3.3): each element is a don't-care
    with probability S, otherwise a care bit that is 0 or 1 with equal probability.
    Returns (care bool[n_elem], bits bool[n_elem])."""
    g = _rng(seed)
    care = g.random(n_elem) >= S
    bits = g.integers(0, 2, size=n_elem).astype(bool) & care
    return care, bits
