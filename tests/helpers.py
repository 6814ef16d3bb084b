"""Glue used by the tests: oracle results <-> the arrays the library's binding takes."""
import dataclasses
import functools

import numpy as np

from oracle import encoder as oenc
from oracle import gf2
from synth_inputs import CONFIGS, make_workload


def paper_format_arrays(enc: "oenc.Encoded"):
    """Oracle `Encoded` -> (w_c uint32[q,l], keep uint64[m*spr] row-major 64-bit words, n_patch uint16[q,l],
    d_patch uint8[], M_rows uint32[n_out])."""
    w_c = gf2.bits_to_int(enc.w_c).astype(np.uint32)
    keep = gf2.bits_to_int(enc.keep.reshape(-1, 64)).astype(np.uint64)
    n_patch = enc.n_patch.astype(np.uint16)
    d_patch = np.concatenate([np.asarray(d, dtype=np.uint8) for d in enc.d_patch]) if enc.q else np.zeros(0, np.uint8)
    M_rows = gf2.bits_to_int(enc.M).astype(np.uint32)
    return w_c, keep, n_patch, d_patch, M_rows


def pack_encoded(enc: "oenc.Encoded"):
    import paper_1905_10138_amd as xe
    w_c, keep, n_patch, d_patch, M_rows = paper_format_arrays(enc)
    return xe.pack(enc.m, enc.n, enc.n_in, enc.q, w_c, keep, n_patch, d_patch, enc.alpha, M_rows, enc.n_out)


@functools.lru_cache(maxsize=8)
def encoded_workload(name: str, m=None, n=None, S=None, n_out=None, n_in=None, exhaustive=False):
    """(workload, oracle-encoded) for a config, cached for the test session.  `S` overrides the
    pruning rate (a low rate with a small n_in gives many patches per slice); `n_out` / `n_in`
    override the slice geometry (the paper's best ratios are at n_out near 200 with n_in = 20);
    `exhaustive` encodes with the 2^n_in search of Section 5.2 in place of Algorithm 1."""
    cfg = CONFIGS[name]
    over = {k: v for k, v in (("S", S), ("n_out", n_out), ("n_in", n_in)) if v is not None}
    if over:
        cfg = dataclasses.replace(cfg, **over)
    wl = make_workload(cfg, m=m, n=n)
    return wl, oenc.encode(wl.keep, wl.planes, wl.alpha, wl.M, wl.n, exhaustive=exhaustive)


def rel_fro(a, b) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
