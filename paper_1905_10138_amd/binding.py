"""ctypes binding of libxorenc.so: same names as the C ABI, argument marshalling only.

Host-side calls (sizes, pack, unpack, check) take NumPy arrays.  GPU calls take torch tensors that
live on the GPU; torch is used for device memory and the current stream, nothing else.  There is
no CPU fallback: if the library is missing every call raises.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

OUT_PLANES, OUT_F32, OUT_BF16 = 0, 1, 2
X_F32, X_BF16 = 0, 1

_LIB = None


class XorencError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = strerror(code) if _LIB is not None else str(code)
        extra = ""
        if code == -4 and _LIB is not None:
            extra = f" (hipError_t {_LIB.xorenc_last_hip_error()})"
        super().__init__(f"{where}: xorenc status {code}: {msg}{extra}")


class _Layer(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32), ("m", ctypes.c_int32), ("n", ctypes.c_int32),
        ("n_out", ctypes.c_int32), ("n_in", ctypes.c_int32), ("q", ctypes.c_int32),
        ("M_rows", ctypes.c_void_p), ("enc", ctypes.c_void_p), ("mask", ctypes.c_void_p),
        ("patch_off", ctypes.c_void_p), ("patch", ctypes.c_void_p), ("alpha", ctypes.c_void_p),
    ]


class _Sizes(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int64) for k in
                ("n_pad", "m_pad", "spr", "n_slots", "n_units", "enc_bytes", "mask_words", "patch_off_words",
                 "espr", "n_eslots")]


def library_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libxorenc.so")


def load_library():
    """Load libxorenc.so from the package directory (built by `python -m paper_1905_10138_amd.build`)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_1905_10138_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.xorenc_version.restype = ctypes.c_uint32
    lib.xorenc_version.argtypes = []
    lib.xorenc_strerror.restype = ctypes.c_char_p
    lib.xorenc_strerror.argtypes = [i32]
    lib.xorenc_last_hip_error.restype = i32
    lib.xorenc_last_hip_error.argtypes = []
    lib.xorenc_get_sizes.restype = i32
    lib.xorenc_get_sizes.argtypes = [i32, i32, i32, i32, i32, ctypes.POINTER(_Sizes)]
    lib.xorenc_pack.restype = i32
    lib.xorenc_pack.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.xorenc_unpack.restype = i32
    lib.xorenc_unpack.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.xorenc_check_packed.restype = i32
    lib.xorenc_check_packed.argtypes = [ctypes.POINTER(_Layer)]
    lib.xorenc_pack_bits.restype = i32
    lib.xorenc_pack_bits.argtypes = [i32, i32, i32, vp, i64, vp]
    lib.xorenc_encode.restype = i32
    lib.xorenc_encode.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, i64, vp, i64, vp]
    lib.xorenc_paper_sizes.restype = i32
    lib.xorenc_paper_sizes.argtypes = [i32, i32, i32, i32, i32, vp, i64, vp]
    lib.xorenc_paper_export.restype = i32
    lib.xorenc_paper_export.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, i64, i64, vp, i64]
    lib.xorenc_paper_import.restype = i32
    lib.xorenc_paper_import.argtypes = [i32, i32, i32, i32, i32, i64, vp, i64, vp, vp, vp, i64, vp]
    lib.xorenc_encode_exhaustive.restype = i32
    lib.xorenc_encode_exhaustive.argtypes = lib.xorenc_encode.argtypes
    lib.xorenc_encode_static.restype = i32
    lib.xorenc_encode_static.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.xorenc_decode.restype = i32
    lib.xorenc_decode.argtypes = [ctypes.POINTER(_Layer), i32, vp, i64, vp]
    lib.xorenc_spmm.restype = i32
    lib.xorenc_spmm.argtypes = [ctypes.POINTER(_Layer), vp, i32, i64, i32, vp, i64, vp]
    _LIB = lib
    return lib


def version() -> int:
    return int(load_library().xorenc_version())


def strerror(code: int) -> str:
    return load_library().xorenc_strerror(int(code)).decode()


def _check(code: int, where: str):
    if code != 0:
        raise XorencError(int(code), where)


def get_sizes(m: int, n: int, n_in: int, q: int, n_out: int = 64) -> dict:
    s = _Sizes()
    _check(load_library().xorenc_get_sizes(m, n, n_in, q, n_out, ctypes.byref(s)), "xorenc_get_sizes")
    return {k: int(getattr(s, k)) for k, _ in _Sizes._fields_}


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _as(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


@dataclass
class PackedLayer:
    """One encrypted matrix in the packed layout; buffers are NumPy (host) or torch (device)."""
    m: int
    n: int
    n_in: int
    q: int
    M_rows: np.ndarray            # uint32[64], always host
    enc: object
    mask: object
    patch_off: object
    patch: object
    alpha: object
    n_out: int = 64               # bits per slice: 64, 128, 192 or 256

    @property
    def on_device(self) -> bool:
        return not isinstance(self.enc, np.ndarray)

    def _ptr(self, buf):
        if buf is None:
            return None
        if isinstance(buf, np.ndarray):
            return buf.ctypes.data if buf.size else None
        return buf.data_ptr() if buf.numel() else None

    def c_struct(self) -> _Layer:
        return _Layer(ctypes.sizeof(_Layer), self.m, self.n, self.n_out, self.n_in, self.q,
                      self.M_rows.ctypes.data, self._ptr(self.enc), self._ptr(self.mask),
                      self._ptr(self.patch_off), self._ptr(self.patch), self._ptr(self.alpha))

    def to(self, device) -> "PackedLayer":
        import torch
        def mv(a, view=None):
            t = torch.from_numpy(a.view(view) if view is not None else a)
            return t.to(device)
        # torch has no uint64/uint32/uint16 arithmetic needs here: move raw bytes with signed views
        return PackedLayer(self.m, self.n, self.n_in, self.q, self.M_rows,
                           mv(self.enc), mv(self.mask, np.int64), mv(self.patch_off, np.int32),
                           mv(self.patch, np.int16), mv(self.alpha), self.n_out)

    def to_host(self) -> "PackedLayer":
        def mv(t, dt):
            return t.detach().cpu().contiguous().numpy().view(dt)
        return PackedLayer(self.m, self.n, self.n_in, self.q, self.M_rows, mv(self.enc, np.uint8),
                           mv(self.mask, np.uint64), mv(self.patch_off, np.uint32), mv(self.patch, np.uint16),
                           mv(self.alpha, np.float32), self.n_out)

    def compressed_bytes(self) -> int:
        """Bytes of every device buffer a kernel reads for this layer."""
        def nb(b):
            return b.nbytes if isinstance(b, np.ndarray) else b.numel() * b.element_size()
        return sum(nb(b) for b in (self.enc, self.mask, self.patch_off, self.patch, self.alpha))


def pack(m, n, n_in, q, w_c, keep, n_patch, d_patch, alpha, M_rows, n_out: int = 64) -> PackedLayer:
    """xorenc_pack: paper format (host NumPy arrays) -> packed layout (host NumPy arrays).
    w_c, n_patch: one entry per n_out-bit slice; keep: uint64 words, row-major (m, spr)."""
    lib = load_library()
    sz = get_sizes(m, n, n_in, q, n_out)
    l = m * sz["espr"]
    w_c = _as(w_c, np.uint32).reshape(q, l)
    keep = _as(keep, np.uint64).reshape(m * sz["spr"])
    n_patch = _as(n_patch, np.uint16).reshape(q, l)
    d_patch = _as(d_patch, np.uint8).reshape(-1)
    alpha = _as(alpha, np.float32).reshape(q, m)
    M_rows = _as(M_rows, np.uint32).reshape(n_out)
    enc = np.empty(sz["enc_bytes"], np.uint8)
    mask = np.empty(sz["mask_words"], np.uint64)
    patch_off = np.empty(sz["patch_off_words"], np.uint32)
    patch = np.empty(d_patch.size, np.uint16)
    _check(lib.xorenc_pack(m, n, n_in, q, n_out, _np_ptr(w_c), _np_ptr(keep), _np_ptr(n_patch),
                           _np_ptr(d_patch) if d_patch.size else None, d_patch.size, _np_ptr(enc), _np_ptr(mask),
                           _np_ptr(patch_off), _np_ptr(patch) if patch.size else None), "xorenc_pack")
    return PackedLayer(m, n, n_in, q, M_rows, enc, mask, patch_off, patch, alpha, n_out)


def unpack(layer: PackedLayer):
    """xorenc_unpack on a host layer: returns (w_c uint32[q,l], keep uint64[m*spr], n_patch uint16[q,l],
    d_patch uint8[]) with l = m * espr slices per plane."""
    if layer.on_device:
        raise ValueError("unpack needs host buffers")
    lib = load_library()
    sz = get_sizes(layer.m, layer.n, layer.n_in, layer.q, layer.n_out)
    l = layer.m * sz["espr"]
    w_c = np.empty((layer.q, l), np.uint32)
    keep = np.empty(layer.m * sz["spr"], np.uint64)
    n_patch = np.empty((layer.q, l), np.uint16)
    d_patch = np.empty(int(layer.patch_off[-1]), np.uint8)
    _check(lib.xorenc_unpack(layer.m, layer.n, layer.n_in, layer.q, layer.n_out, _np_ptr(layer.enc),
                             _np_ptr(layer.mask), _np_ptr(layer.patch_off),
                             _np_ptr(layer.patch) if layer.patch.size else None,
                             _np_ptr(w_c), _np_ptr(keep), _np_ptr(n_patch),
                             _np_ptr(d_patch) if d_patch.size else None), "xorenc_unpack")
    return w_c, keep, n_patch, d_patch


class _PaperBits(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int64) for k in ("wc_bits", "n_patch_bits", "d_patch_bits", "header_bits", "total_bits")]


def paper_sizes(m, n, n_in, q, n_patch, block_slices, n_out: int = 64) -> dict:
    """xorenc_paper_sizes: bits of the parts of the paper-format stream (n_patch: uint16 [q, l])."""
    n_patch = _as(n_patch, np.uint16)
    out = _PaperBits()
    _check(load_library().xorenc_paper_sizes(m, n, n_in, q, n_out, _np_ptr(n_patch), int(block_slices),
                                             ctypes.byref(out)), "xorenc_paper_sizes")
    return {k: int(getattr(out, k)) for k, _ in _PaperBits._fields_}


def paper_export(m, n, n_in, q, w_c, n_patch, d_patch, block_slices, n_out: int = 64) -> np.ndarray:
    """xorenc_paper_export: the arrays of `unpack` -> the bit stream (uint8 array)."""
    w_c, n_patch, d_patch = _as(w_c, np.uint32), _as(n_patch, np.uint16), _as(d_patch, np.uint8)
    nbytes = (paper_sizes(m, n, n_in, q, n_patch, block_slices, n_out)["total_bits"] + 7) // 8
    out = np.empty(nbytes, np.uint8)
    _check(load_library().xorenc_paper_export(m, n, n_in, q, n_out, _np_ptr(w_c), _np_ptr(n_patch),
                                              _np_ptr(d_patch) if d_patch.size else None, d_patch.size,
                                              int(block_slices), _np_ptr(out) if nbytes else None, nbytes),
           "xorenc_paper_export")
    return out


def paper_import(m, n, n_in, q, stream, block_slices, n_out: int = 64):
    """xorenc_paper_import: the bit stream -> (w_c uint32[q,l], n_patch uint16[q,l], d_patch uint8[])."""
    stream = _as(stream, np.uint8)
    l = m * get_sizes(m, n, n_in, q, n_out)["espr"]
    w_c = np.empty((q, l), np.uint32)
    n_patch = np.empty((q, l), np.uint16)
    total = ctypes.c_int64(0)
    cap = max(16, stream.size)
    while True:
        d_patch = np.empty(cap, np.uint8)
        rc = load_library().xorenc_paper_import(m, n, n_in, q, n_out, int(block_slices), _np_ptr(stream), stream.size,
                                                _np_ptr(w_c), _np_ptr(n_patch), _np_ptr(d_patch), cap,
                                                ctypes.byref(total))
        if rc == -1 and total.value > cap:
            cap = int(total.value)
            continue
        _check(rc, "xorenc_paper_import")
        return w_c, n_patch, d_patch[:total.value].copy()


def pack_bits(a: np.ndarray, n_out: int = 64) -> np.ndarray:
    """xorenc_pack_bits: dense 0/1 matrix (m, n) -> unit-major uint64 words (host), columns padded to n_out."""
    a = np.ascontiguousarray(a).view(np.uint8) if a.dtype == np.bool_ else _as(a, np.uint8)
    m, n = a.shape
    spr, nrb = -(-n // n_out) * (n_out // 64), (m + 31) // 32
    out = np.empty(nrb * 32 * spr, np.uint64)
    _check(load_library().xorenc_pack_bits(m, n, n_out, _np_ptr(a), a.strides[0], _np_ptr(out)), "xorenc_pack_bits")
    return out


def encode(m, n, n_in, q, M_rows, mask, planes, alpha, patch_capacity: Optional[int] = None,
           n_out: int = 64, _entry: str = "xorenc_encode") -> PackedLayer:
    """xorenc_encode on the current stream.  mask: int64 GPU tensor [n_slots] (unit-major words),
    planes: int64 GPU tensor [q, n_slots], alpha: float32 GPU tensor [q, m].  Returns a device
    PackedLayer that shares `mask` and `alpha`.  Synchronises once to read the patch total (the
    C call itself does not) and retries with a larger patch buffer if the first was too small."""
    import torch
    lib = load_library()
    sz = get_sizes(m, n, n_in, q, n_out)
    dev = mask.device
    M_rows = _as(M_rows, np.uint32).reshape(n_out)
    if mask.numel() != sz["n_slots"] or planes.numel() != q * sz["n_slots"]:
        raise ValueError("mask/planes do not have n_slots words per plane")
    enc = torch.zeros(sz["enc_bytes"], dtype=torch.uint8, device=dev)
    patch_off = torch.empty(sz["patch_off_words"], dtype=torch.int32, device=dev)
    ws_bytes = q * sz["n_slots"] * 8 + q * sz["n_units"] * 4
    ws = torch.empty((ws_bytes + 7) // 8, dtype=torch.int64, device=dev)
    cap = int(patch_capacity) if patch_capacity is not None else max(1024, q * sz["n_slots"] // 8)
    while True:
        patch = torch.empty(cap, dtype=torch.int16, device=dev)
        _check(getattr(lib, _entry)(m, n, n_in, q, n_out, _np_ptr(M_rows), ctypes.c_void_p(mask.data_ptr()),
                                    ctypes.c_void_p(planes.data_ptr()), ctypes.c_void_p(enc.data_ptr()),
                                    ctypes.c_void_p(patch_off.data_ptr()), ctypes.c_void_p(patch.data_ptr()), cap,
                                    ctypes.c_void_p(ws.data_ptr()), ws.numel() * 8, _stream_ptr()), _entry)
        total = int(patch_off[-1].item())
        if total <= cap:
            break
        cap = total
    return PackedLayer(m, n, n_in, q, M_rows, enc, mask, patch_off, patch[:total], alpha, n_out)


def encode_exhaustive(m, n, n_in, q, M_rows, mask, planes, alpha, patch_capacity: Optional[int] = None,
                      n_out: int = 64) -> PackedLayer:
    """xorenc_encode_exhaustive on the current stream; arguments and result as `encode`."""
    return encode(m, n, n_in, q, M_rows, mask, planes, alpha, patch_capacity, n_out,
                  _entry="xorenc_encode_exhaustive")


STATIC_SCRATCH_BYTES = 24 * 1024 * 1024


def encode_static(m, n, n_in, q, M_rows, mask, planes, enc_out, patch_off_out, patch_out, n_out: int = 64) -> None:
    """xorenc_encode_static on the current stream: like xorenc_encode, but the scratch memory is the library's
    own static area, and every output buffer is the caller's (GPU tensors: enc_out uint8[enc_bytes],
    patch_off_out int32[q*n_units + 1], patch_out int16[capacity]).  Nothing is allocated and nothing
    synchronises; read patch_off_out[-1] afterwards to learn the patch total."""
    M_rows = _as(M_rows, np.uint32).reshape(n_out)
    _check(load_library().xorenc_encode_static(
        m, n, n_in, q, n_out, _np_ptr(M_rows), ctypes.c_void_p(mask.data_ptr()), ctypes.c_void_p(planes.data_ptr()),
        ctypes.c_void_p(enc_out.data_ptr()), ctypes.c_void_p(patch_off_out.data_ptr()),
        ctypes.c_void_p(patch_out.data_ptr()) if patch_out.numel() else None, patch_out.numel(), _stream_ptr()),
        "xorenc_encode_static")


def check_packed(layer: PackedLayer) -> int:
    """xorenc_check_packed on a host layer; returns the status code (0 = well formed)."""
    if layer.on_device:
        raise ValueError("check_packed needs host buffers")
    st = layer.c_struct()
    return int(load_library().xorenc_check_packed(ctypes.byref(st)))


def _stream_ptr():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def decode(layer: PackedLayer, out_kind: int = OUT_PLANES, out=None):
    """xorenc_decode on the current stream.  Returns the output tensor (int64 words for planes,
    float32, or int16 bf16 patterns)."""
    import torch
    if not layer.on_device:
        raise ValueError("decode needs a layer whose buffers are on the GPU")
    dev = layer.enc.device
    spr = -(-layer.n // layer.n_out) * (layer.n_out // 64)
    if out is None:
        if out_kind == OUT_PLANES:
            out = torch.empty((layer.q, layer.m * spr), dtype=torch.int64, device=dev)
        elif out_kind == OUT_F32:
            out = torch.empty((layer.m, layer.n), dtype=torch.float32, device=dev)
        else:
            out = torch.empty((layer.m, layer.n), dtype=torch.bfloat16, device=dev)
    ld = out.stride(0) if out_kind != OUT_PLANES else 0
    st = layer.c_struct()
    _check(load_library().xorenc_decode(ctypes.byref(st), out_kind, ctypes.c_void_p(out.data_ptr()), ld,
                                        _stream_ptr()), "xorenc_decode")
    return out


def spmm(layer: PackedLayer, X, Y=None):
    """xorenc_spmm on the current stream: Y = W X with X (n, B) float32 or bfloat16, row-major."""
    import torch
    if not layer.on_device:
        raise ValueError("spmm needs a layer whose buffers are on the GPU")
    if X.dim() != 2 or X.shape[0] != layer.n or X.stride(1) != 1:
        raise ValueError("X must be (n, B) with contiguous columns")
    if X.dtype == torch.float32:
        xd = X_F32
    elif X.dtype == torch.bfloat16:
        xd = X_BF16
    else:
        raise ValueError("X must be float32 or bfloat16")
    B = X.shape[1]
    if Y is None:
        Y = torch.empty((layer.m, B), dtype=torch.float32, device=X.device)
    st = layer.c_struct()
    _check(load_library().xorenc_spmm(ctypes.byref(st), ctypes.c_void_p(X.data_ptr()), xd, X.stride(0), B,
                                      ctypes.c_void_p(Y.data_ptr()), Y.stride(0), _stream_ptr()), "xorenc_spmm")
    return Y
