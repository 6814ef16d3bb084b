"""Pins for the oracle's encoder: Algorithm 1, the exhaustive search, the rank-chain closed
form for the patch count, the paper's printed memory reduction, the lossless invariant."""
import math

import numpy as np
import pytest

from oracle import decoder, encoder, gf2, patch_search, ratio
from synth_inputs import CONFIGS, make_workload, random_care_problem


def _random_slice(rng, n_out, p_care):
    care = rng.random(n_out) < p_care
    bits = rng.integers(0, 2, size=n_out).astype(bool) & care
    return care, bits


def test_row_reduce_textbook_case():
    # x0 ^ x1 = 1, x1 ^ x2 = 0, x0 ^ x2 = 1 (dependent, consistent)
    mat = np.array([[1, 1, 0, 1], [0, 1, 1, 0], [1, 0, 1, 1]], dtype=np.uint8)
    r = patch_search.row_reduce(mat)
    assert r.tolist() == [[1, 0, 1, 1], [0, 1, 1, 0], [0, 0, 0, 0]]
    assert patch_search.has_solution(r)
    mat[2, 3] = 0                                   # now x0 ^ x2 = 0: contradiction
    assert not patch_search.has_solution(patch_search.row_reduce(mat))
    assert patch_search.solution_with_free_zero(r, 3).tolist() == [1, 0, 0]


def test_fig4_structure(golden):
    """Fig. 4 / Section 3.1: with care bits {3,4,5,7} of 8 the system keeps rows 3,4,5,7 of M."""
    n_in, n_out = int(golden["fig4_n_in"]), int(golden["fig4_n_out"])
    care1 = [int(t) for t in golden["fig4_care_1based"].split()]
    removed1 = [int(t) for t in golden["fig4_removed_rows_1based"].split()]
    assert sorted(care1 + removed1) == list(range(1, n_out + 1))
    rng = np.random.default_rng(4)
    M = rng.integers(0, 2, size=(n_out, n_in), dtype=np.uint8)
    care = np.zeros(n_out, bool)
    care[[c - 1 for c in care1]] = True
    x_true = rng.integers(0, 2, size=n_in, dtype=np.uint8)
    bits = gf2.xor_network(M, x_true).astype(bool)    # a solvable target
    n_patch, d_patch, w_c, dropped = patch_search.patch_search(care, bits, M)
    assert n_patch == 0 and dropped == []
    assert np.array_equal(gf2.xor_network(M, w_c)[care], bits[care])
    # changing a removed (don't-care) row of M cannot change the result
    M2 = M.copy()
    M2[[r - 1 for r in removed1]] ^= 1
    assert np.array_equal(patch_search.patch_search(care, bits, M2)[2], w_c)


@pytest.mark.parametrize("n_out,n_in,p_care,soft", [(8, 4, 0.5, True), (12, 5, 0.5, True), (16, 8, 0.45, True),
                                                     (16, 10, 0.7, False), (4, 3, 0.8, True)])
def test_algorithm1_against_exhaustive_search(n_out, n_in, p_care, soft, golden):
    rng = np.random.default_rng(n_out * 1000 + n_in)
    tot_greedy = tot_opt = 0
    for trial in range(120):
        M = rng.integers(0, 2, size=(n_out, n_in), dtype=np.uint8)
        care, bits = _random_slice(rng, n_out, p_care)
        n_patch, d_patch, w_c, dropped = patch_search.patch_search(care, bits, M)
        opt, x_opt = patch_search.exhaustive_min_patches(care, bits, M)
        assert d_patch == dropped                      # compare step returns the removed equations
        assert n_patch >= opt
        assert (n_patch == 0) == (opt == 0)            # solvable <=> no patches
        # flipping d_patch after decryption reproduces every care bit (lossless)
        w = gf2.xor_network(M, w_c).astype(bool)
        w[d_patch] ^= True
        assert np.array_equal(w[care], bits[care])
        tot_greedy += n_patch
        tot_opt += opt
    # Section 3.3: "up to 10 %" more replacements than exhaustive, in the regime the paper
    # works in (care bits per slice around n_in or fewer); sampling slack added.  The heavily
    # over-determined case only has to respect the hard bounds checked above.
    if soft:
        assert tot_greedy <= tot_opt * (1 + float(golden["alg1_excess_over_exhaustive"]) + 0.08) + 2


@pytest.mark.parametrize("n_out,n_in,p_care", [(8, 4, 0.5), (16, 6, 0.5), (64, 8, 0.05), (64, 16, 0.2), (24, 20, 0.9)])
def test_vectorised_encoder_equals_literal_algorithm(n_out, n_in, p_care):
    rng = np.random.default_rng(n_out + 7 * n_in)
    M = rng.integers(0, 2, size=(n_out, n_in), dtype=np.uint8)
    l = 150
    care = rng.random((l, n_out)) < p_care
    bits = rng.integers(0, 2, size=(l, n_out)).astype(bool) & care
    w_c, n_patch, d_patch = encoder.encode_plane(care, bits, M)
    off = 0
    for s in range(l):
        npch, dp, wc, _ = patch_search.patch_search(care[s], bits[s], M)
        assert npch == n_patch[s]
        assert dp == d_patch[off:off + npch].tolist()
        assert np.array_equal(wc, w_c[s])
        off += npch
    assert off == d_patch.size


def _expected_patches_rank_chain(k, n_in):
    """A fresh uniformly random equation lies in the span of r accepted independent ones with
    probability 2^(r - n_in); it then contradicts them with probability 1/2 (a patch), else is
    redundant; otherwise the rank grows by one."""
    dist = {0: 1.0}
    exp = 0.0
    for _ in range(k):
        new = {}
        for r, pr in dist.items():
            p_in = 2.0 ** (r - n_in)
            exp += pr * p_in * 0.5
            new[r] = new.get(r, 0.0) + pr * p_in
            if r < n_in:
                new[r + 1] = new.get(r + 1, 0.0) + pr * (1 - p_in)
        dist = new
    return exp


@pytest.mark.parametrize("n_in,S", [(8, 0.95), (8, 0.90), (12, 0.85)])
def test_patch_rate_matches_rank_chain_closed_form(n_in, S):
    n_out = 64
    pk = [math.comb(n_out, k) * (1 - S) ** k * S ** (n_out - k) for k in range(n_out + 1)]
    model = sum(pk[k] * _expected_patches_rank_chain(k, n_in) for k in range(n_out + 1))
    rng = np.random.default_rng(11 + n_in)
    tot = cnt = 0
    for trial in range(150):                         # fresh M every time: the model averages over M
        M = rng.integers(0, 2, size=(n_out, n_in), dtype=np.uint8)
        care = rng.random((600, n_out)) >= S
        bits = rng.integers(0, 2, size=(600, n_out)).astype(bool) & care
        _, n_patch, _ = encoder.encode_plane(care, bits, M)
        tot += int(n_patch.sum())
        cnt += 600
    assert model > 0.01
    assert abs(tot / cnt - model) / model < 0.10


def test_solvable_when_few_care_bits_and_explodes_when_many():
    """Section 3.1: about n_out (1 - S) independent equations need n_in >= that many inputs."""
    rng = np.random.default_rng(5)
    M = rng.integers(0, 2, size=(64, 16), dtype=np.uint8)
    for p_care, lo, hi in [(0.05, 0.0, 0.002), (0.6, 10.0, 64.0)]:
        care = rng.random((400, 64)) < p_care
        bits = rng.integers(0, 2, size=(400, 64)).astype(bool) & care
        _, n_patch, _ = encoder.encode_plane(care, bits, M)
        assert lo <= n_patch.mean() <= hi


def test_paper_synthetic_memory_reduction(golden):
    """Section 3.3 / Fig. 6: 10,000 random elements, S = 0.9, n_in = 20: memory reduction peaks
    at about 0.83 for n_out close to 200."""
    n_elem, S, n_in = int(golden["e2_elements"]), float(golden["e2_S"]), int(golden["e2_n_in"])
    target = float(golden["e2_best_memory_reduction"])
    sweep = [60, 120, 160, 200, 240, 320, 480]
    red = {n_out: [] for n_out in sweep}
    for seed in range(24):
        care, bits = random_care_problem(n_elem, S, 1000 + seed)
        M_full = np.random.default_rng(2000 + seed).integers(0, 2, size=(max(sweep), n_in), dtype=np.uint8)
        for n_out in sweep:
            l = n_elem // n_out                      # whole slices only
            c = care[:l * n_out].reshape(l, n_out)
            b = bits[:l * n_out].reshape(l, n_out)
            _, n_patch, _ = encoder.encode_plane(c, b, M_full[:n_out])
            red[n_out].append(ratio.memory_reduction(l * n_out, n_in, n_out, n_patch))
    mean = {k: float(np.mean(v)) for k, v in red.items()}
    best = max(mean, key=mean.get)
    assert 160 <= best <= 240
    assert abs(mean[best] - target) <= 0.03
    assert mean[best] < S                            # bounded by the share of don't-care bits
    assert mean[60] < mean[best] and mean[480] < mean[best]   # a real interior optimum (trade-off)


def test_more_inputs_mean_fewer_patches():
    """Section 3.3 / Fig. 7 trend: larger n_in needs fewer d_patch at the same n_out."""
    care, bits = random_care_problem(64 * 800, 0.8, 77)
    care, bits = care.reshape(-1, 64), bits.reshape(-1, 64)
    rng = np.random.default_rng(78)
    M = rng.integers(0, 2, size=(64, 32), dtype=np.uint8)
    counts = [int(encoder.encode_plane(care, bits, M[:, :n_in])[1].sum()) for n_in in (12, 16, 20, 24, 32)]
    assert all(a > b for a, b in zip(counts, counts[1:]))


@pytest.mark.parametrize("name,m,n", [("tiny", 256, 256), ("fig1", 96, 320), ("fc6", 64, 448),
                                      ("lstm", 70, 200), ("large_q1", 128, 512), ("large_q2", 128, 512)])
def test_lossless_roundtrip_on_config_recipes(name, m, n):
    """Section 3.2: decryption plus patches reproduces every care bit, for every plane."""
    wl = make_workload(CONFIGS[name], m=m, n=n)
    enc = encoder.encode(wl.keep, wl.planes, wl.alpha, wl.M, wl.n)
    dec = decoder.decrypt_planes(enc)
    assert dec.shape == wl.planes.shape
    assert np.array_equal(dec & wl.keep[None], wl.planes & wl.keep[None])
    assert not decoder.masked_planes(enc)[:, :, wl.n:].any()          # padding columns stay 0
    assert enc.l == m * wl.n_pad // 64
    # patches only ever sit on care positions
    for p in range(enc.q):
        sl = np.repeat(np.arange(enc.l), enc.n_patch[p])
        assert wl.keep.reshape(-1, 64)[sl, enc.d_patch[p]].all()


def test_flipping_is_an_involution():
    wl = make_workload(CONFIGS["large_q1"], m=64, n=256)
    enc = encoder.encode(wl.keep, wl.planes, wl.alpha, wl.M, wl.n)
    assert enc.n_patch.sum() > 0
    once = decoder.decrypt_planes(enc)
    twice = encoder.Encoded(**{**enc.__dict__, "n_patch": enc.n_patch * 0,
                               "d_patch": [np.zeros(0, np.int64)] * enc.q})
    raw = decoder.decrypt_planes(twice)
    diff = (once ^ raw).reshape(enc.q, enc.l, 64)
    assert np.array_equal(diff.sum(axis=2), enc.n_patch)             # exactly the listed bits differ
    # a row with no kept weight: w^c = 0 and no patches
    keep = wl.keep.copy(); keep[3] = False
    planes = wl.planes & keep[None]
    e2 = encoder.encode(keep, planes, wl.alpha, wl.M, wl.n)
    spr = wl.n_pad // 64
    assert not e2.w_c[:, 3 * spr:(3 + 1) * spr].any()
    assert not e2.n_patch[:, 3 * spr:(3 + 1) * spr].any()


@pytest.mark.parametrize("n_out,n_in,p_care", [(64, 8, 0.1), (64, 8, 0.3), (128, 10, 0.08), (192, 12, 0.06)])
def test_vectorised_exhaustive_search_against_the_per_slice_listing(n_out, n_in, p_care):
    """`encode_plane_exhaustive` (all slices at once, distances through a matrix product) against
    `patch_search.exhaustive_min_patches` (one slice, mismatches counted directly): same minimum, same
    input (both take the first minimum in integer order), never more patches than Algorithm 1, and the
    patched output reproduces every care bit."""
    rng = np.random.default_rng(7 * n_out + n_in)
    M = rng.integers(0, 2, size=(n_out, n_in), dtype=np.uint8)
    l = 60
    care = rng.random((l, n_out)) < p_care
    bits = rng.integers(0, 2, size=(l, n_out)).astype(bool) & care
    w_c, n_patch, d_patch = encoder.encode_plane_exhaustive(care, bits, M)
    _, n_g, _ = encoder.encode_plane(care, bits, M)
    assert np.all(n_patch <= n_g)
    pos = np.split(d_patch, np.cumsum(n_patch)[:-1])
    for s in range(l):
        opt, x_opt = patch_search.exhaustive_min_patches(care[s], bits[s], M)
        assert n_patch[s] == opt
        assert np.array_equal(w_c[s], x_opt)
        y = gf2.xor_network(M, w_c[s][None])[0].astype(bool)
        y[pos[s]] ^= True
        assert np.array_equal(y & care[s], bits[s])


@pytest.mark.parametrize("n_out,n_in,part_bits,p_care", [(64, 10, 4, 0.15), (128, 12, 7, 0.1), (64, 9, 16, 0.3),
                                                         (192, 11, 1, 0.05)])
def test_exhaustive_listing_in_parts_equals_the_one_part_listing(n_out, n_in, part_bits, p_care):
    """The listing taken 2^part_bits inputs at a time (Section 5.2 for wider inputs) returns the same minimum and
    the same smallest input as the listing taken at once, whatever the part size."""
    rng = np.random.default_rng(100 * n_out + n_in)
    M = rng.integers(0, 2, size=(n_out, n_in), dtype=np.uint8)
    for _ in range(12):
        care = rng.random(n_out) < p_care
        bits = rng.integers(0, 2, size=n_out).astype(np.uint8) & care
        d0, x0 = patch_search.exhaustive_min_patches(care, bits, M)
        d1, x1 = patch_search.exhaustive_min_patches_in_parts(care, bits, M, part_bits)
        assert d0 == d1
        assert np.array_equal(x0, x1)


def test_exhaustive_listing_in_parts_on_planted_inputs_of_18_bits():
    """n_in = 18, where the one-part listing is already heavy.  The outputs of a planted input with up to two care
    bits turned over: the minimum is at most the number turned over; the network has full column rank on the
    care set, so with nothing turned over the planted input is the only one with zero mismatches and is returned;
    and ties go to the smallest integer: with a zero column in M the bit of that column comes back 0."""
    rng = np.random.default_rng(18)
    n_out, n_in = 64, 18
    M = rng.integers(0, 2, size=(n_out, n_in), dtype=np.uint8)
    care = np.ones(n_out, dtype=bool)                              # 64 equations, 18 unknowns
    reduced = patch_search.row_reduce(np.concatenate([M, np.zeros((n_out, 1), np.uint8)], axis=1))
    assert int(reduced[:, :-1].any(axis=1).sum()) == n_in          # full column rank over GF(2): one solution at most
    x = rng.integers(0, 2, size=n_in, dtype=np.uint8)
    y = gf2.xor_network(M, x[None])[0]
    d, xb = patch_search.exhaustive_min_patches_in_parts(care, y, M, 14)
    assert d == 0 and np.array_equal(xb, x)
    y2 = y.copy(); y2[[5, 40]] ^= 1
    d2, xb2 = patch_search.exhaustive_min_patches_in_parts(care, y2, M, 14)
    assert d2 <= 2
    assert int((gf2.xor_network(M, xb2[None])[0] != y2).sum()) == d2
    M0 = M.copy(); M0[:, 17] = 0                                   # input bit 17 changes nothing
    x17 = x.copy(); x17[17] = 1
    y0 = gf2.xor_network(M0, x17[None])[0]
    d3, xb3 = patch_search.exhaustive_min_patches_in_parts(care, y0, M0, 14)
    assert d3 == 0 and xb3[17] == 0
