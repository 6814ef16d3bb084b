"""MI355X (gfx950) library for XOR-gate-encrypted sparse quantized weights (arXiv 1905.10138):
decode and fused decode + W X.  All arithmetic runs in the HIP kernels of libxorenc.so; this
package is the argument-marshalling layer over its C ABI (include/xorenc.h)."""
from .binding import (
    OUT_BF16,
    OUT_F32,
    OUT_PLANES,
    STATIC_SCRATCH_BYTES,
    PackedLayer,
    XorencError,
    check_packed,
    decode,
    encode,
    encode_exhaustive,
    encode_static,
    get_sizes,
    library_path,
    load_library,
    pack,
    pack_bits,
    paper_export,
    paper_import,
    paper_sizes,
    spmm,
    strerror,
    unpack,
    version,
)

__all__ = [
    "OUT_BF16", "OUT_F32", "OUT_PLANES", "PackedLayer", "XorencError", "check_packed", "decode", "encode", "encode_exhaustive", "encode_static", "STATIC_SCRATCH_BYTES",
    "pack_bits",
    "paper_export", "paper_import", "paper_sizes", "get_sizes", "library_path", "load_library", "pack", "spmm", "strerror", "unpack", "version",
]
