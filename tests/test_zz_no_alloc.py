"""xorenc_encode_static (the entry point for callers that cannot allocate: scratch in a static device array)
against xorenc_encode (scratch in a caller-provided workspace): the two enqueue the same kernels, so every
output must be identical bit for bit.  Two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared scratch area would show; then the size limit and the error text."""
import ctypes

import numpy as np
import pytest

from synth_inputs import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _inputs(name, m, n):
    import torch
    import paper_1905_10138_amd as xe
    dev = torch.device("cuda:0")
    wl = make_workload(CONFIGS[name], m=m, n=n)
    n_out = wl.cfg.n_out
    mask = torch.from_numpy(xe.pack_bits(wl.keep[:, :wl.n], n_out).view(np.int64)).to(dev)
    planes = torch.from_numpy(
        np.stack([xe.pack_bits(wl.planes[p][:, :wl.n], n_out) for p in range(wl.cfg.q)]).view(np.int64)).to(dev)
    alpha = torch.from_numpy(wl.alpha).to(dev)
    M_rows = (wl.M.astype(np.uint64) << np.arange(wl.cfg.n_in, dtype=np.uint64)).sum(axis=1).astype(np.uint32)
    return wl, mask, planes, alpha, M_rows


def _both_ways(name, m, n):
    import torch
    import paper_1905_10138_amd as xe
    wl, mask, planes, alpha, M_rows = _inputs(name, m, n)
    cfg = wl.cfg
    ref = xe.encode(wl.m, wl.n, cfg.n_in, cfg.q, M_rows, mask, planes, alpha, n_out=cfg.n_out)   # workspace version
    torch.cuda.synchronize()
    sz = xe.get_sizes(wl.m, wl.n, cfg.n_in, cfg.q, cfg.n_out)
    dev = mask.device
    # outputs are the caller's: allocated here, before the call, and pre-filled so that stale content would show
    enc = torch.zeros(sz["enc_bytes"], dtype=torch.uint8, device=dev)
    patch_off = torch.full((sz["patch_off_words"],), -1, dtype=torch.int32, device=dev)
    patch = torch.full((max(1, ref.patch.numel()),), -1, dtype=torch.int16, device=dev)
    before = torch.cuda.memory_allocated()
    xe.encode_static(wl.m, wl.n, cfg.n_in, cfg.q, M_rows, mask, planes, enc, patch_off, patch, n_out=cfg.n_out)
    assert torch.cuda.memory_allocated() == before          # nothing went through torch's allocator either
    torch.cuda.synchronize()
    total = int(patch_off[-1].item())
    assert total == ref.patch.numel()
    assert torch.equal(enc, ref.enc)
    assert torch.equal(patch_off, ref.patch_off)
    assert torch.equal(patch[:total], ref.patch)
    return total


def test_static_scratch_encoder_equals_workspace_encoder_twice_in_a_row():
    big = _both_ways("large_q2", 4096, 4096)          # 2 planes, 4.2 MB of the scratch area
    small = _both_ways("lstm", 130, 3000)             # then a smaller, differently shaped input
    assert big > 0 and small >= 0
    again = _both_ways("large_q2", 4096, 4096)        # and the first once more
    assert again == big


def test_static_scratch_limit_is_an_error_not_a_fault():
    import torch
    import paper_1905_10138_amd as xe
    lib = xe.load_library()
    # 3 planes of 16384 x 4096: 3 * 1 Mi words * 8 bytes alone exceed the area
    m, n, n_in, q = 16384, 4096, 8, 3
    sz = xe.get_sizes(m, n, n_in, q)
    assert q * sz["n_slots"] * 8 + q * sz["n_units"] * 4 > xe.STATIC_SCRATCH_BYTES
    dummy = torch.zeros(16, dtype=torch.int64, device="cuda:0")     # never touched: the sizes are checked first
    M_rows = np.zeros(64, np.uint32)
    rc = lib.xorenc_encode_static(m, n, n_in, q, 64, ctypes.c_void_p(M_rows.ctypes.data), ctypes.c_void_p(dummy.data_ptr()),
                                  ctypes.c_void_p(dummy.data_ptr()), ctypes.c_void_p(dummy.data_ptr()),
                                  ctypes.c_void_p(dummy.data_ptr()), ctypes.c_void_p(dummy.data_ptr()), 0, None)
    assert rc == -6
    assert "capacity" in xe.strerror(rc)
