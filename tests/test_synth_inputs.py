"""The seeded input generators: shapes, exact pruning counts, determinism, bf16 rounding."""
import numpy as np
import pytest

import synth_inputs as si


def test_magnitude_mask_exact_count_and_ties():
    W = np.array([[0.5, -0.5, 0.1, 0.5], [0.5, -2.0, 0.5, 0.0]], dtype=np.float32)
    keep = si.magnitude_mask(W, 0.5)                 # prune 4: 0.0, 0.1, then the first two 0.5 by index
    assert keep.astype(int).tolist() == [[0, 0, 0, 1], [1, 1, 1, 0]]
    rng = np.random.default_rng(0)
    W = rng.standard_normal((37, 53)).astype(np.float32)
    for S in (0.0, 0.8, 0.91, 0.999):
        keep = si.magnitude_mask(W, S)
        assert (~keep).sum() == int(np.floor(S * W.size))
        if keep.any() and (~keep).any():
            assert np.abs(W[keep]).min() >= np.abs(W[~keep]).max()


def test_greedy_binary_code_definition():
    W = np.array([[1.0, -3.0, 0.25, 0.0]], dtype=np.float32)
    keep = np.array([[True, True, False, True]])
    planes, alpha = si.greedy_binary_code(W, keep, 2)
    # kept: 1, -3, 0 -> alpha1 = 4/3, bits (1, 0, -, 1); residuals -1/3, -5/3, -4/3 -> alpha2 = 10/9, bits 0
    assert planes[0].astype(int).tolist() == [[1, 0, 0, 1]]
    assert planes[1].astype(int).tolist() == [[0, 0, 0, 0]]
    assert np.allclose(alpha[:, 0], [4 / 3, 10 / 9], rtol=1e-7)
    assert alpha.dtype == np.float32
    planes, alpha = si.greedy_binary_code(W, np.zeros_like(keep), 1)
    assert alpha[0, 0] == 0 and not planes.any()


@pytest.mark.parametrize("name", sorted(si.CONFIGS))
def test_workload_shapes_and_determinism(name):
    cfg = si.CONFIGS[name]
    m, n = min(cfg.m, 96), min(cfg.n, 200 if cfg.n % 64 else 192)
    a = si.make_workload(cfg, m=m, n=n)
    b = si.make_workload(cfg, m=m, n=n)
    assert a.n_pad % 64 == 0 and a.n_pad - n < 64
    assert a.keep.shape == (m, a.n_pad) and a.planes.shape == (cfg.q, m, a.n_pad)
    assert a.alpha.shape == (cfg.q, m) and a.M.shape == (64, cfg.n_in)
    assert not a.keep[:, n:].any() and not (a.planes & ~a.keep[None]).any()
    assert a.keep.sum() == m * n - int(np.floor(cfg.S * m * n))
    for f in ("keep", "planes", "alpha", "M"):
        assert np.array_equal(getattr(a, f), getattr(b, f))
    care_bits = a.planes[0][a.keep]
    assert 0.4 < care_bits.mean() < 0.6            # care bits are 0/1 with about equal probability
    assert 0.4 < a.M.mean() < 0.6
    B = cfg.batches[-1]
    xs, xe = a.X(B)
    assert xe.shape == (n, B) and xe.dtype == np.float32
    if cfg.x_dtype == "bf16":
        assert xs.dtype == np.uint16 and np.array_equal(si.bf16_bits_to_f32(xs), xe)


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.005, 65504.0], dtype=np.float32)
    b = si.f32_to_bf16_bits(x)
    assert b[:3].tolist() == [0x3F80, 0x3F80, 0x3F82]
    back = si.bf16_bits_to_f32(b)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
