"""CPU-side tests of libxorenc.so: exported symbols, sizes, pack/unpack round trip, content
checker, argument validation (every check happens before any GPU call)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1905_10138_amd as xe
from paper_1905_10138_amd import binding
from helpers import encoded_workload, pack_encoded, paper_format_arrays

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = xe.load_library()
    text = open(os.path.join(ROOT, "include", "xorenc.h")).read()
    names = set(re.findall(r"XORENC_API[^;(]*?\b(xorenc_\w+)\s*\(", text))
    assert {"xorenc_decode", "xorenc_spmm", "xorenc_pack", "xorenc_unpack", "xorenc_get_sizes",
            "xorenc_encode", "xorenc_encode_exhaustive", "xorenc_encode_static", "xorenc_paper_sizes", "xorenc_paper_export", "xorenc_paper_import",
            "xorenc_check_packed", "xorenc_version", "xorenc_strerror",
            "xorenc_last_hip_error"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert xe.version() >> 16 == 2
    assert "align" in xe.strerror(-3)


def test_sizes():
    s = xe.get_sizes(6000, 3000, 24, 3)
    assert (s["n_pad"], s["m_pad"], s["spr"]) == (3008, 6016, 47)
    assert s["n_slots"] == 6016 * 47 and s["n_units"] == 188 * 47
    assert s["enc_bytes"] == 3 * s["n_slots"] * 3 and s["patch_off_words"] == 3 * s["n_units"] + 1
    s = xe.get_sizes(6000, 3000, 24, 3, 192)                     # slices of three 64-bit words
    assert (s["n_pad"], s["spr"], s["espr"]) == (3072, 48, 16)
    assert s["n_eslots"] == 6016 * 16 and s["enc_bytes"] == 3 * s["n_eslots"] * 3
    for bad in [(8, 8, 8, 1, 96), (8, 8, 8, 1, 320), (8, 8, 8, 1, 0)]:
        with pytest.raises(xe.XorencError) as e:
            xe.get_sizes(*bad)
        assert e.value.code == -2
    for bad in [(0, 8, 8, 1), (8, 0, 8, 1)]:
        with pytest.raises(xe.XorencError) as e:
            xe.get_sizes(*bad)
        assert e.value.code == -1
    s = xe.get_sizes(6000, 3000, 20, 3, 192)                     # 20 encrypted bits: 20 dwords per 32 slices
    assert s["enc_bytes"] == 3 * (s["n_eslots"] // 32) * 20 * 4
    for bad in [(8, 8, 3, 1), (8, 8, 8, 5), (8, 8, 40, 1)]:
        with pytest.raises(xe.XorencError) as e:
            xe.get_sizes(*bad)
        assert e.value.code == -2


@pytest.mark.parametrize("name,m,n,n_out,n_in", [
    ("tiny", 70, 256, 64, None), ("lstm", 45, 200, 64, None), ("large_q2", 64, 512, 64, None),
    ("fc6", 33, 130, 64, None), ("lstm", 45, 200, 192, None), ("large_q2", 64, 500, 128, None),
    ("fig1", 40, 700, 256, None), ("lstm", 45, 200, 192, 20), ("tiny", 70, 256, 64, 13), ("fc6", 33, 130, 128, 27),
    ("large_q1", 64, 512, 64, 4), ("large_q2", 64, 500, 128, 31)])
def test_pack_unpack_roundtrip(name, m, n, n_out, n_in):
    wl, enc = encoded_workload(name, m, n, n_out=n_out, n_in=n_in)
    w_c, keep, n_patch, d_patch, M_rows = paper_format_arrays(enc)
    L = pack_encoded(enc)
    assert xe.check_packed(L) == 0
    w2, k2, np2, dp2 = xe.unpack(L)
    assert np.array_equal(w2, w_c) and np.array_equal(k2, keep)
    assert np.array_equal(np2, n_patch) and np.array_equal(dp2, d_patch)
    # layout spot checks straight from the documented slot formulas
    J = n_out // 64
    spr = wl.n_pad // 64
    espr = wl.n_pad // n_out
    n_eslots = L.mask.size // J
    stream = np.unpackbits(L.enc, bitorder="little")              # bit k of the stream
    rng = np.random.default_rng(0)
    for _ in range(50):
        r, s, p = rng.integers(m), rng.integers(spr), rng.integers(enc.q)
        slot = ((r // 32) * spr + s) * 32 + r % 32
        assert L.mask[slot] == keep[r * spr + s]
        eslot = ((r // 32) * espr + s // J) * 32 + r % 32
        field = stream[(p * n_eslots + eslot) * enc.n_in:(p * n_eslots + eslot + 1) * enc.n_in]
        assert int((field.astype(np.uint64) << np.arange(enc.n_in, dtype=np.uint64)).sum()) == w_c[p, r * espr + s // J]
    assert int(L.patch_off[-1]) == d_patch.size
    assert np.all(np.diff(L.patch_off.astype(np.int64)) >= 0)


def test_pack_rejects_malformed_patch_data():
    wl, enc = encoded_workload("large_q1", 64, 512)
    w_c, keep, n_patch, d_patch, M_rows = paper_format_arrays(enc)
    assert d_patch.size > 2
    with pytest.raises(xe.XorencError) as e:        # one entry short
        xe.pack(enc.m, enc.n, enc.n_in, enc.q, w_c, keep, n_patch, d_patch[:-1], enc.alpha, M_rows)
    assert e.value.code == -5
    bad = d_patch.copy(); bad[0] = 64
    with pytest.raises(xe.XorencError):
        xe.pack(enc.m, enc.n, enc.n_in, enc.q, w_c, keep, n_patch, bad, enc.alpha, M_rows)
    wbad = w_c.copy(); wbad[0, 0] |= 1 << 8        # bit beyond n_in = 8
    with pytest.raises(xe.XorencError):
        xe.pack(enc.m, enc.n, enc.n_in, enc.q, wbad, keep, n_patch, d_patch, enc.alpha, M_rows)


def test_check_packed_finds_planted_damage():
    wl, enc = encoded_workload("large_q1", 64, 512)
    L = pack_encoded(enc)
    assert xe.check_packed(L) == 0
    off = L.patch_off.copy()
    i = int(np.flatnonzero(np.diff(off.astype(np.int64)) > 0)[0])
    L.patch_off = off.copy(); L.patch_off[i + 1] = off[i] - 1 if off[i] > 0 else off[i + 2] + 5
    assert xe.check_packed(L) == -5
    L.patch_off = off
    p = L.patch.copy(); p[0] = (p[0] & ~np.uint16(63)) | np.uint16(int(np.flatnonzero(
        [(int(L.mask[i * 32 + (int(p[0]) >> 6)]) >> b) & 1 == 0 for b in range(64)])[0]))
    L.patch = p                                      # patch moved onto a pruned position
    assert xe.check_packed(L) == -5


def test_gpu_entry_points_validate_before_touching_the_gpu():
    lib = xe.load_library()
    wl, enc = encoded_workload("tiny", 70, 256)
    L = pack_encoded(enc)
    st = L.c_struct()                                # host pointers: fine for validation-only calls
    out = np.zeros(8, np.uint64)
    assert lib.xorenc_decode(None, 0, out.ctypes.data, 0, None) == -1
    assert lib.xorenc_decode(ctypes.byref(st), 0, None, 0, None) == -1
    assert lib.xorenc_decode(ctypes.byref(st), 7, out.ctypes.data, 0, None) == -2
    assert lib.xorenc_decode(ctypes.byref(st), 1, out.ctypes.data, 10, None) == -1        # ld < n
    assert lib.xorenc_decode(ctypes.byref(st), 0, out.ctypes.data + 4, 0, None) == -3
    bad = L.c_struct(); bad.struct_size = 8
    assert lib.xorenc_decode(ctypes.byref(bad), 0, out.ctypes.data, 0, None) == -1
    bad = L.c_struct(); bad.n_out = 96
    assert lib.xorenc_decode(ctypes.byref(bad), 0, out.ctypes.data, 0, None) == -2
    bad = L.c_struct(); bad.q = 9
    assert lib.xorenc_spmm(ctypes.byref(bad), out.ctypes.data, 1, 8, 8, out.ctypes.data, 8, None) == -2
    bad = L.c_struct(); bad.mask = (bad.mask or 0) + 4
    assert lib.xorenc_spmm(ctypes.byref(bad), out.ctypes.data, 1, 8, 8, out.ctypes.data, 8, None) == -3
    assert lib.xorenc_spmm(ctypes.byref(st), None, 1, 8, 8, out.ctypes.data, 8, None) == -1
    assert lib.xorenc_spmm(ctypes.byref(st), out.ctypes.data, 1, 4, 8, out.ctypes.data, 8, None) == -1   # ldx < B
    assert lib.xorenc_spmm(ctypes.byref(st), out.ctypes.data, 1, 8, 0, out.ctypes.data, 8, None) == -1   # B = 0
    assert lib.xorenc_spmm(ctypes.byref(st), out.ctypes.data, 5, 8, 8, out.ctypes.data, 8, None) == -2
    assert lib.xorenc_spmm(ctypes.byref(st), out.ctypes.data + 1, 1, 8, 8, out.ctypes.data, 8, None) == -3


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "library_path", lambda: "/nonexistent/libxorenc.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library()


@pytest.mark.parametrize("name,m,n,n_out,n_in,S", [("large_q1", 64, 512, 64, 8, None), ("lstm", 45, 200, 192, 20, None),
                                                  ("fc6", 33, 130, 128, 16, 0.7), ("tiny", 70, 256, 64, 13, None)])
def test_paper_format_stream_matches_oracle(name, m, n, n_out, n_in, S):
    """The library's bit stream of Section 3.2's format with blocked n_patch widths (Section 5.2) against the
    oracle's writer, byte for byte, starting from the packed layer; and its reader against the arrays."""
    from oracle import gf2, paper_format
    wl, enc = encoded_workload(name, m, n, S=S, n_out=n_out, n_in=n_in)
    L = pack_encoded(enc)
    w_c, keep, n_patch, d_patch = xe.unpack(L)
    for blk in (enc.l, 32, 7):
        want_sizes = paper_format.sizes(enc.n_in, enc.n_out, enc.n_patch, blk)
        got_sizes = xe.paper_sizes(enc.m, enc.n, enc.n_in, enc.q, n_patch, blk, enc.n_out)
        assert got_sizes == {"wc_bits": want_sizes.wc_bits, "n_patch_bits": want_sizes.n_patch_bits,
                             "d_patch_bits": want_sizes.d_patch_bits, "header_bits": want_sizes.header_bits,
                             "total_bits": want_sizes.total_bits}
        stream = xe.paper_export(enc.m, enc.n, enc.n_in, enc.q, w_c, n_patch, d_patch, blk, enc.n_out)
        want = paper_format.write_stream(enc.n_in, enc.n_out, gf2.bits_to_int(enc.w_c), enc.n_patch, enc.d_patch, blk)
        assert stream.tobytes() == want
        w2, np2, dp2 = xe.paper_import(enc.m, enc.n, enc.n_in, enc.q, stream, blk, enc.n_out)
        assert np.array_equal(w2, w_c) and np.array_equal(np2, n_patch) and np.array_equal(dp2, d_patch)
    # damaged streams are rejected, not read out of bounds
    with pytest.raises(xe.XorencError):
        xe.paper_import(enc.m, enc.n, enc.n_in, enc.q, stream[:len(stream) // 2], 7, enc.n_out)
    with pytest.raises(xe.XorencError):
        xe.paper_sizes(enc.m, enc.n, enc.n_in, enc.q, n_patch, 0, enc.n_out)


def _random_host_cases(count, seed):
    rng = np.random.default_rng(seed)
    names = ["tiny", "fig1", "fc6", "lstm", "large_q1", "large_q2"]
    return [(names[int(rng.integers(len(names)))], int(rng.integers(1, 120)), int(rng.integers(1, 700)),
             int(rng.choice([64, 128, 192, 256])), int(rng.integers(4, 33)), float(rng.choice([0.6, 0.8, 0.95])))
            for _ in range(count)]


@pytest.mark.parametrize("name,m,n,n_out,n_in,S", _random_host_cases(20, 11))
def test_random_geometries_pack_unpack_export_import(name, m, n, n_out, n_in, S):
    """Seeded random geometries through every host-side transformation: paper arrays -> packed layout -> paper
    arrays -> bit stream -> paper arrays; the content checker accepts the packed layer; the stream's parts add
    up to the oracle's accounting."""
    from oracle import paper_format
    wl, enc = encoded_workload(name, m, n, S=S, n_out=n_out, n_in=n_in)
    w_c, keep, n_patch, d_patch, M_rows = paper_format_arrays(enc)
    L = pack_encoded(enc)
    assert xe.check_packed(L) == 0
    w2, k2, np2, dp2 = xe.unpack(L)
    assert np.array_equal(w2, w_c) and np.array_equal(k2, keep)
    assert np.array_equal(np2, n_patch) and np.array_equal(dp2, d_patch)
    blk = int(np.random.default_rng(m * n).integers(1, 2 * enc.l + 1))
    stream = xe.paper_export(enc.m, enc.n, enc.n_in, enc.q, w2, np2, dp2, blk, enc.n_out)
    want = paper_format.sizes(enc.n_in, enc.n_out, enc.n_patch, blk)
    assert stream.size == (want.total_bits + 7) // 8
    w3, np3, dp3 = xe.paper_import(enc.m, enc.n, enc.n_in, enc.q, stream, blk, enc.n_out)
    assert np.array_equal(w3, w_c) and np.array_equal(np3, n_patch) and np.array_equal(dp3, d_patch)
