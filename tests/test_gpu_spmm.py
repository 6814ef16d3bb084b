"""GPU parity of the fused decode + product (xorenc_spmm) against the fp64 oracle.

Tolerances (relative Frobenius error against fp64): 2e-3 for bf16 X, 1e-5 for fp32 X.  The
kernel multiplies exact +-2/0 operands with exact bf16 terms and accumulates in fp32, so the
observed error is far below both; the bounds are the contract, not the expectation."""
import numpy as np
import pytest

from helpers import encoded_workload, pack_encoded, rel_fro
from oracle import decoder
from synth_inputs import draw_X

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-3, "f32": 1e-5}
# Element-wise bound on top of the contract: every product of the kernel is exact (+-2 or 0 times a bf16 value,
# scaled in fp32) and sums are fp32, so |Y - Y_64| <= n_terms * 2^-24 * sum_c |W[r,c]| |X[c,b]|; at most a few
# hundred kept weights per row keep that below 1e-5 of the sum of magnitudes, while one wrong weight bit moves
# an output by 2 alpha |x|, a thousand times more.
ELEMENT_TOL = 1e-5


def few_column_allowance(enc, exact):
    """Extra room for bf16 X with few columns (at most two, or up to eight on layers of several rounds; granted to every
    bf16 call of at most four columns and to the tall-layer cases).  That path carries X as two FP8 terms and multiplies on
    the block-scaled matrix instruction, which aligns the (up to 16) products of one operand run to the largest
    of them and keeps 14 bits below its leading bit: a product more than 2^10 times smaller than the largest
    product of its run loses low bits, less than 2^-13 of the largest.  A run = the columns 4j + d (j = 0..7)
    of one 32-column half-word with d in {0, 1} or in {2, 3}.  Only kept weights produce non-zero products, so
    the allowance of an output is the sum over its runs of 2^-12 * (largest kept |x| of the run) per kept value
    below 2^-9 of that largest (a factor two of margin on both); it is zero for almost every output."""
    X = np.abs(np.asarray(exact, dtype=np.float64))
    n, B = X.shape
    n_pad = enc.keep.shape[1]
    Xp = np.zeros((n_pad, B))
    Xp[:n] = X
    cols = np.arange(n_pad)
    run = (cols // 32) * 2 + ((cols % 4) >> 1)
    pos = ((cols % 4) & 1) * 8 + (cols % 32) // 4
    order = np.argsort(run * 16 + pos, kind="stable")          # column of (run, position)
    keep = np.asarray(enc.keep)[:, order].reshape(enc.keep.shape[0], n_pad // 16, 16)
    Xr = Xp[order].reshape(n_pad // 16, 16, B)
    alpha = enc.alpha.astype(np.float64).sum(axis=0)
    out = np.zeros((keep.shape[0], B))
    for r0 in range(0, keep.shape[0], 2048):
        k = keep[r0:r0 + 2048]
        top = np.zeros((k.shape[0], k.shape[1], B))
        for t in range(16):
            top = np.maximum(top, k[:, :, t, None] * Xr[None, :, t, :])
        extra = np.zeros_like(top)
        for t in range(16):
            small = k[:, :, t, None] & (Xr[None, :, t, :] < top * 2.0 ** -9)
            extra += small * top * 2.0 ** -12
        out[r0:r0 + 2048] = alpha[r0:r0 + 2048, None] * extra.sum(axis=1)
    return out


def assert_every_output_close(got, want, enc, exact, few_columns=False):
    """|got - want| <= ELEMENT_TOL * (|W| |X|) for every row and column (|W| = keep * sum_p alpha_p)."""
    absW = np.where(enc.keep, enc.alpha.astype(np.float64).sum(axis=0)[:, None], 0.0)[:, :enc.n]
    bound = ELEMENT_TOL * (absW @ np.abs(np.asarray(exact, dtype=np.float64)))
    if few_columns:
        bound = bound + few_column_allowance(enc, exact)
    diff = np.abs(np.asarray(got, dtype=np.float64) - want)
    bad = np.argwhere(diff > bound + 1e-30)
    assert bad.size == 0, f"{len(bad)} outputs off, first (row, col) = {bad[0].tolist()}"


def _run(name, m, n, B, dtype, ldx_pad=0, S=None, n_out=None, n_in=None, every_output=False, few_columns=None):
    """few_columns: whether the call may take the kernel whose X travels as two FP8 terms (then the element-wise
    bound carries that kernel's allowance): by default bf16 X with at most four columns; layers of many rounds take
    it up to eight columns, and the tests of such layers say so."""
    import torch
    import paper_1905_10138_amd as xe
    wl, enc = encoded_workload(name, m, n, S, n_out, n_in)
    L = pack_encoded(enc).to(torch.device("cuda:0"))
    stored, exact = draw_X(wl.n, B, dtype, wl.cfg.seed_X + 1000 * B)
    if dtype == "bf16":
        xt = torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16)
    else:
        xt = torch.from_numpy(stored)
    if ldx_pad:
        buf = torch.zeros((wl.n, B + ldx_pad), dtype=xt.dtype)
        buf[:, :B] = xt
        xg = buf.to("cuda:0")[:, :B]
    else:
        xg = xt.to("cuda:0")
    Y = xe.spmm(L, xg)
    torch.cuda.synchronize()
    want = decoder.spmm_f64(enc, exact)
    if every_output:
        if few_columns is None:
            few_columns = dtype == "bf16" and B <= 4
        assert_every_output_close(Y.cpu().numpy(), want, enc, exact, few_columns=few_columns)
    return Y.cpu().numpy(), want


SMALL_CASES = [
    ("tiny", 256, 256, 8, "f32"), ("tiny", 256, 256, 8, "bf16"), ("tiny", 70, 200, 1, "f32"),
    ("tiny", 70, 200, 33, "f32"), ("tiny", 33, 70, 5, "bf16"),
    ("fig1", 200, 448, 64, "bf16"), ("fig1", 200, 448, 63, "bf16"), ("fig1", 64, 2048, 1, "bf16"),
    ("fc6", 97, 640, 1, "bf16"), ("fc6", 97, 640, 64, "bf16"), ("fc6", 97, 640, 100, "bf16"), ("fc6", 97, 640, 4, "f32"),
    ("lstm", 130, 3000, 1, "bf16"), ("lstm", 130, 3000, 32, "bf16"), ("lstm", 130, 3000, 40, "f32"),
    ("large_q1", 320, 1024, 1, "bf16"), ("large_q1", 320, 1024, 8, "bf16"), ("large_q1", 320, 1024, 64, "bf16"),
    ("large_q1", 320, 1024, 256, "bf16"), ("large_q1", 320, 1024, 130, "bf16"), ("large_q1", 320, 1024, 7, "bf16"),
    ("lstm", 130, 3000, 3, "bf16"), ("fc6", 97, 640, 8, "bf16"),
    ("large_q2", 96, 4096, 8, "bf16"), ("large_q2", 96, 4096, 256, "bf16"), ("large_q2", 96, 4096, 16, "f32"),
]


EDGE_CASES = [
    ("tiny", 1, 1, 1, "f32"), ("tiny", 1, 1, 1, "bf16"), ("tiny", 1, 1, 8, "bf16"), ("tiny", 31, 63, 2, "bf16"),
    ("fig1", 40, 130, 1000, "bf16"), ("fig1", 40, 130, 1024, "bf16"), ("large_q1", 4100, 64, 512, "bf16"),
    ("large_q2", 4100, 64, 512, "bf16"), ("lstm", 70, 64, 264, "f32"), ("fc6", 2, 9216, 8, "bf16"),
]


@pytest.mark.parametrize("name,m,n,B,dtype", EDGE_CASES)
def test_spmm_degenerate_and_extreme_shapes(name, m, n, B, dtype):
    """One weight; fewer rows than a row block and fewer columns than a slice; many more columns of X than a
    workgroup covers; a single slice (most waves of a workgroup get nothing); two rows with a long reduction."""
    got, want = _run(name, m, n, B, dtype)
    assert got.shape == want.shape == (m, B)
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= TOL[dtype]


@pytest.mark.parametrize("name,m,n,B,dtype", SMALL_CASES)
def test_spmm_matches_fp64_oracle(name, m, n, B, dtype):
    got, want = _run(name, m, n, B, dtype)
    assert got.shape == want.shape
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= TOL[dtype]


FULL_CASES = [("fig1", 64), ("fc6", 1), ("fc6", 64), ("lstm", 1), ("lstm", 32), ("large_q1", 1), ("large_q1", 8),
              ("large_q1", 64), ("large_q1", 256), ("large_q2", 1), ("large_q2", 8), ("large_q2", 64), ("large_q2", 256),
              ("large_q1", 4), ("large_q2", 3), ("fc6", 2), ("lstm", 4)]


@pytest.mark.parametrize("name,B", FULL_CASES)
def test_spmm_full_size_configs(name, B):
    got, want = _run(name, None, None, B, "bf16", every_output=True)  # every row and column, element by element
    err = rel_fro(got, want)
    assert err <= TOL["bf16"], err


@pytest.mark.parametrize("name,m,n,B,n_in,S", [
    ("large_q1", 16384, 256, 256, 8, None), ("large_q1", 16390, 200, 248, 8, None), ("large_q1", 12288, 320, 384, 16, None),
    ("large_q1", 12290, 256, 376, 24, None), ("large_q1", 16384, 192, 256, 8, 0.8),
    ("large_q2", 16390, 200, 136, 16, None), ("large_q2", 12810, 320, 64, 8, None), ("large_q2", 8200, 256, 256, 24, 0.85),
    ("large_q1", 8192, 256, 256, 8, None), ("large_q1", 8200, 200, 328, 16, None), ("large_q2", 8200, 320, 136, 8, None),
    # more than 256 tiles of 64 rows at 8, 16 and 32 aligned columns: four-wave workgroups, several per CU
    ("large_q1", 20000, 512, 8, 8, None), ("large_q1", 40010, 200, 8, 16, 0.8), ("large_q1", 20000, 384, 16, 8, None),
    ("large_q1", 18000, 320, 32, 16, None), ("large_q2", 17000, 256, 8, 8, None), ("large_q1", 33000, 130, 24, 8, 0.8)])
def test_tall_matrix_many_columns(name, m, n, B, n_in, S):
    """Enough tiles to fill the chip once or twice: the launches with 128-row tiles (one plane) or 64-row tiles
    (two planes), with eight waves per workgroup up to 256 tiles and four waves, two workgroups per CU, above
    (n_in <= 16).  Ragged rows, columns and batch; a short reduction (3 to 5 slices over 4 or 8 waves:
    some waves get none)."""
    got, want = _run(name, m, n, B, "bf16", S=S, n_in=n_in, every_output=True)
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= TOL["bf16"]


@pytest.mark.parametrize("name,m,n,B,n_in,S", [
    ("large_q1", 40000, 512, 4, 8, None), ("large_q1", 33000, 448, 1, 8, None), ("large_q1", 20010, 1000, 3, 16, None),
    ("large_q2", 36000, 256, 3, 8, None), ("lstm", 24000, 320, 2, 24, None), ("large_q1", 17000, 2048, 4, 8, 0.8),
    # three rounds (an odd count), one and two planes; four, six and seven rounds, where five to seven columns take
    # the same kernel
    ("large_q1", 70000, 256, 2, 8, None), ("large_q2", 90000, 128, 1, 8, None),
    ("large_q1", 170000, 256, 6, 8, None), ("large_q1", 200000, 128, 7, 8, None), ("large_q1", 115000, 256, 5, 8, 0.8)])
def test_tall_matrix_few_columns(name, m, n, B, n_in, S):
    """More 16-row pieces than one round of workgroups takes: every wave of the few-column kernel walks over
    several of them with the next piece's words requested while the current one is multiplied.  Ragged rows
    and columns, one to three planes, dense patch lists in two cases."""
    got, want = _run(name, m, n, B, "bf16", S=S, n_in=n_in, every_output=True, few_columns=True)
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= TOL["bf16"]


@pytest.mark.parametrize("B,dtype", [(1, "bf16"), (8, "bf16"), (64, "bf16"), (200, "bf16"), (16, "f32")])
def test_many_patches_per_unit(B, dtype):
    """Pruning rate 0.75 with n_in = 8: about 16 care bits per slice against 8 encrypted bits, so most
    slices carry several patches and a wave's range holds more patch entries than its registers prefetch."""
    wl, enc = encoded_workload("large_q1", 160, 1024, 0.75)
    assert enc.n_patch.sum() > 3 * enc.n_patch.size
    got, want = _run("large_q1", 160, 1024, B, dtype, S=0.75)
    assert rel_fro(got, want) <= TOL[dtype]


@pytest.mark.parametrize("B", [8, 64])
def test_patch_counts_from_none_to_a_dozen_per_unit(B):
    """Pruning rate 0.93: units without patches next to units with up to a dozen."""
    got, want = _run("large_q1", 320, 1024, B, "bf16", S=0.93)
    assert rel_fro(got, want) <= TOL["bf16"]


WIDE_CASES = [
    ("lstm", 130, 3000, 192, 24, 1, "bf16"), ("lstm", 130, 3000, 192, 24, 32, "bf16"), ("lstm", 130, 3000, 192, 24, 40, "f32"),
    ("large_q1", 320, 1024, 128, 8, 8, "bf16"), ("large_q1", 320, 1024, 128, 8, 64, "bf16"),
    ("large_q1", 320, 1024, 128, 8, 256, "bf16"), ("large_q1", 320, 1024, 128, 8, 5, "bf16"),
    ("large_q2", 96, 4096, 256, 16, 8, "bf16"), ("large_q2", 96, 4096, 256, 16, 200, "bf16"),
    ("fig1", 200, 448, 256, 32, 64, "bf16"), ("fig1", 200, 448, 256, 32, 63, "bf16"), ("tiny", 33, 70, 128, 16, 8, "f32"),
]


# n_in that is not a whole number of bytes: 20 and 17 (one or two dwords per lane, specialised kernels),
# 4 (several slices per byte), and widths that take the general kernel (13, 27, 31, 9)
ANY_N_IN_CASES = [
    ("lstm", 130, 3000, 192, 20, 32, "bf16"), ("lstm", 130, 3000, 192, 20, 1, "bf16"), ("lstm", 130, 3000, 192, 20, 40, "f32"),
    ("lstm", 130, 3000, 64, 17, 8, "bf16"), ("lstm", 130, 3000, 64, 17, 3, "bf16"), ("lstm", 130, 3000, 64, 20, 7, "bf16"),
    ("large_q1", 320, 1024, 64, 4, 64, "bf16"), ("large_q1", 320, 1024, 64, 4, 5, "bf16"),
    ("large_q1", 320, 1024, 64, 20, 256, "bf16"), ("large_q1", 320, 1024, 64, 20, 64, "bf16"),
    ("tiny", 256, 256, 64, 13, 8, "f32"), ("tiny", 256, 256, 64, 13, 64, "bf16"), ("fc6", 97, 640, 128, 27, 64, "bf16"),
    ("fc6", 97, 640, 128, 27, 1, "bf16"), ("large_q2", 96, 4096, 128, 31, 72, "bf16"), ("fig1", 200, 448, 64, 9, 6, "bf16"),
    ("large_q2", 96, 4096, 64, 20, 64, "bf16"),
]


@pytest.mark.parametrize("name,m,n,n_out,n_in,B,dtype", ANY_N_IN_CASES)
def test_spmm_with_bit_packed_encrypted_vectors(name, m, n, n_out, n_in, B, dtype):
    got, want = _run(name, m, n, B, dtype, n_out=n_out, n_in=n_in)
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= TOL[dtype]


@pytest.mark.parametrize("name,m,n,n_out,n_in,B,dtype", WIDE_CASES)
def test_spmm_with_slices_of_several_words(name, m, n, n_out, n_in, B, dtype):
    """n_out = 128, 192, 256: one encrypted vector feeds two to four 64-bit words of a row."""
    got, want = _run(name, m, n, B, dtype, n_out=n_out, n_in=n_in)
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= TOL[dtype]


def test_paper_region_full_size():
    """The paper's best compression is near n_out = 200 with n_in = 20: the LSTM-shaped layer at
    n_out = 192 with n_in = 24 and with n_in = 20, full size, fused product at B = 32."""
    got, want = _run("lstm", None, None, 32, "bf16", n_out=192, n_in=24)
    assert rel_fro(got, want) <= TOL["bf16"]
    got, want = _run("lstm", None, None, 32, "bf16", n_out=192, n_in=20)
    assert rel_fro(got, want) <= TOL["bf16"]


def test_tiny_config_fp32_full():
    got, want = _run("tiny", None, None, 8, "f32")
    assert rel_fro(got, want) <= TOL["f32"]


def test_odd_leading_dimension_and_unaligned_rows():
    got, want = _run("fig1", 200, 448, 64, "bf16", ldx_pad=3)     # ldx = 67: the 16-bit load path
    assert rel_fro(got, want) <= TOL["bf16"]
    got, want = _run("fig1", 200, 448, 8, "bf16", ldx_pad=3)      # few columns, rows not 16-byte aligned
    assert rel_fro(got, want) <= TOL["bf16"]
    got, want = _run("fig1", 200, 448, 2, "bf16", ldx_pad=1)
    assert rel_fro(got, want) <= TOL["bf16"]
    got, want = _run("fig1", 200, 448, 6, "f32", ldx_pad=1)
    assert rel_fro(got, want) <= TOL["f32"]


@pytest.mark.parametrize("name,m,n,B,dtype,pad", [
    # compact X whose rows do not start on 16-byte boundaries: copied to a padded staging area first
    ("large_q1", 320, 1024, 33, "bf16", 0), ("large_q1", 320, 1024, 65, "bf16", 0), ("lstm", 130, 3000, 9, "bf16", 0),
    ("large_q2", 96, 4096, 100, "bf16", 3), ("fc6", 97, 640, 7, "bf16", 0), ("fig1", 200, 448, 5, "bf16", 2),
    ("tiny", 256, 256, 9, "f32", 0), ("tiny", 33, 70, 13, "f32", 2), ("lstm", 130, 3000, 21, "f32", 0),
    # aligned rows, a last 16-byte piece with fewer columns (fetched whole; the extent of X ends inside a dword)
    ("large_q1", 320, 1024, 33, "bf16", 7), ("large_q1", 320, 1024, 5, "bf16", 3), ("fig1", 200, 448, 71, "bf16", 1),
    ("tiny", 33, 70, 5, "f32", 3), ("lstm", 130, 3000, 3, "bf16", 5),
    # too large for the staging area (4 MiB with padded rows): the element-wise kernels
    ("large_q2", 96, 4096, 530, "bf16", 0)])
def test_rows_of_X_that_do_not_start_on_16_byte_boundaries(name, m, n, B, dtype, pad):
    got, want = _run(name, m, n, B, dtype, ldx_pad=pad, every_output=(dtype == "bf16"))
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= TOL[dtype]


def test_identity_X_reproduces_decoded_weights():
    """Y = W I = W: the fused path against the decode path, no oracle involved in the comparison."""
    import torch
    import paper_1905_10138_amd as xe
    wl, enc = encoded_workload("fc6", 97, 640)
    L = pack_encoded(enc).to(torch.device("cuda:0"))
    X = torch.eye(wl.n, dtype=torch.float32, device="cuda:0")
    Y = xe.spmm(L, X).cpu().numpy()
    W = xe.decode(L, xe.OUT_F32).cpu().numpy()
    assert np.allclose(Y, W, rtol=1e-6, atol=1e-9)
    assert np.allclose(W, decoder.dequantize_f64(enc), rtol=1e-6, atol=0)


def test_output_leading_dimension_and_overwrite():
    import torch
    import paper_1905_10138_amd as xe
    wl, enc = encoded_workload("fig1", 200, 448)
    L = pack_encoded(enc).to(torch.device("cuda:0"))
    stored, exact = draw_X(wl.n, 64, "bf16", 99)
    xg = torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16).to("cuda:0")
    buf = torch.full((200, 80), 3.0, dtype=torch.float32, device="cuda:0")
    xe.spmm(L, xg, Y=buf[:, :64])
    got = buf.cpu().numpy()
    assert rel_fro(got[:, :64], decoder.spmm_f64(enc, exact)) <= TOL["bf16"]
    assert np.all(got[:, 64:] == 3.0)


def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    names = ["tiny", "fig1", "fc6", "lstm", "large_q1", "large_q2"]
    cases = []
    for _ in range(count):
        name = names[int(rng.integers(len(names)))]
        n_out = int(rng.choice([64, 64, 64, 128, 192, 256]))
        n_in = int(rng.integers(4, 33))
        m = int(rng.integers(1, 300))
        n = int(rng.integers(1, 1500))
        B = int(rng.choice([1, 2, 3, 7, 8, 16, 24, 31, 32, 33, 40, 64, 65, 96, 128, 200, 256, 300]))
        dtype = "f32" if rng.random() < 0.25 else "bf16"
        pad = int(rng.choice([0, 0, 0, 1, 8]))
        cases.append((name, m, n, n_out, n_in, B, dtype, pad))
    return cases


@pytest.mark.parametrize("name,m,n,n_out,n_in,B,dtype,pad", _random_cases(48, 20240611))
def test_spmm_random_shapes(name, m, n, n_out, n_in, B, dtype, pad):
    """Seeded random geometry: every slice width, any n_in, ragged m / n / B, padded leading dimension."""
    got, want = _run(name, m, n, B, dtype, ldx_pad=pad, n_out=n_out, n_in=n_in)
    assert got.shape == want.shape == (m, B)
    assert np.isfinite(got).all()
    assert rel_fro(got, want) <= TOL[dtype]


@pytest.mark.parametrize("name,m,n,B,dtype", [
    ("fc6", 4096, 9216, 1, "bf16"), ("lstm", 6000, 3000, 1, "bf16"), ("fig1", 2048, 2048, 64, "bf16"),
    ("lstm", 6000, 3000, 32, "bf16"), ("tiny", 256, 256, 8, "f32"), ("fc6", 97, 640, 3, "bf16")])
def test_split_reduction_is_deterministic_and_one_launch(name, m, n, B, dtype):
    """Layers with fewer output tiles than CUs split the reduction dimension over several workgroups per tile.
    Their partial sums meet in the library's scratch area and are added in a fixed order: the same bits on
    every call, also when calls on other layers come in between (the scratch slots are taken in turn and the
    arrival counters must be back at zero after every launch), and Y needs no clearing beforehand."""
    import torch
    import paper_1905_10138_amd as xe
    wl, enc = encoded_workload(name, m, n)
    L = pack_encoded(enc).to(torch.device("cuda:0"))
    other_wl, other_enc = encoded_workload("fc6", 97, 640)
    other = pack_encoded(other_enc).to(torch.device("cuda:0"))
    stored, exact = draw_X(wl.n, B, dtype, wl.cfg.seed_X + 1000 * B)
    xg = (torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16) if dtype == "bf16" else torch.from_numpy(stored)).to("cuda:0")
    xo = torch.from_numpy(draw_X(other_wl.n, 5, "bf16", 3)[0].view(np.int16)).view(torch.bfloat16).to("cuda:0")
    Y = torch.full((wl.m, B), float("nan"), dtype=torch.float32, device="cuda:0")   # stale content must not matter
    xe.spmm(L, xg, Y=Y)
    first = Y.clone()
    assert rel_fro(first.cpu().numpy(), decoder.spmm_f64(enc, exact)) <= TOL[dtype]
    assert_every_output_close(first.cpu().numpy(), decoder.spmm_f64(enc, exact), enc, exact) if dtype == "bf16" else None
    for i in range(12):
        if i % 3 == 1:
            xe.spmm(other, xo)                  # another split launch in between: takes the next slot
        Y.fill_(float(i))
        xe.spmm(L, xg, Y=Y)
        assert torch.equal(Y, first), f"call {i} differs"
