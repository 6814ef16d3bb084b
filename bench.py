#!/usr/bin/env python3
"""Benchmark of the fused decode + W X path on one MI355X.

A step is one xorenc_spmm call: the whole hot path (stream-in, GF(2) decode, patch flips, mask,
dequantise, contraction) over one batch X of the workload.  Inputs are synthetic (seeded, see
synth_inputs), encoded on the GPU by xorenc_encode before timing, and resident in HBM.  To keep
the timed reads cold (the layers are far smaller than the 256 MB last-level cache) the steps walk
round-robin over R replicas of the compressed layer, X and Y with R * bytes >= 1 GiB.  Steps are
issued back to back on one stream from a captured HIP graph so that host launch cost does not
pace the GPU.

Prints ONE JSON line.  Headline (`value`, `roofline`): the large one-bit matrix at B = 64.  `sweep`: the other
batch sizes of that matrix.  `configs`: every configuration of the benchmark contract at each of its batch sizes,
with its own roofline object.  `marginal`: the same recipe four times as tall, to separate what a launch costs
from what a row of W costs.  `decode`, `fig1`, `n_out_192*`, `storage`, `encoder`: see the functions below.
"""
import argparse
import ctypes
import hashlib
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
LAUNCH_BOUND_US = 4.0           # below about this many microseconds of roofline time a kernel is mostly fixed cost


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="large_q1", help="one of synth_inputs.CONFIGS")
    ap.add_argument("--batch", type=int, default=64, help="columns of X (B)")
    ap.add_argument("--sweep", default="1,8,64,256", help="other batch sizes reported under 'sweep' ('' = none)")
    ap.add_argument("--sweep-steps", type=int, default=400)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of from a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of W in the CPU-oracle sample (0 = auto)")
    ap.add_argument("--replica-bytes", type=float, default=float(1 << 30))
    ap.add_argument("--no-wide", action="store_true", help="skip the n_out=192 / n_in=24 extra on the same matrix")
    ap.add_argument("--no-decode", action="store_true", help="skip the timing of xorenc_decode on the workload")
    ap.add_argument("--no-encoder", action="store_true", help="skip the timing of the two GPU encoders")
    ap.add_argument("--no-fig1", action="store_true", help="skip the Fig. 1-shaped extra (decode-only and fused, B=64)")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration table")
    ap.add_argument("--no-marginal", action="store_true", help="skip the four-times-taller matrix")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region run one 256 MiB device copy (reference dispatch for rocprofv3 --pmc)")
    return ap.parse_args()


def encoder_inputs(wl, xe, torch, dev):
    """Unit-major mask and bit-planes of the workload on the GPU, alpha, and the rows of M as integers."""
    n_out = wl.cfg.n_out
    mask = torch.from_numpy(xe.pack_bits(wl.keep[:, :wl.n], n_out).view(np.int64)).to(dev)
    planes = torch.from_numpy(
        np.stack([xe.pack_bits(wl.planes[p][:, :wl.n], n_out) for p in range(wl.cfg.q)]).view(np.int64)).to(dev)
    alpha = torch.from_numpy(wl.alpha).to(dev)
    M_rows = (wl.M.astype(np.uint64) << np.arange(wl.cfg.n_in, dtype=np.uint64)).sum(axis=1).astype(np.uint32)
    return mask, planes, alpha, M_rows


def build_layer(wl, xe, torch, dev):
    """Encode the workload on the GPU (xorenc_encode) and return the device layer."""
    mask, planes, alpha, M_rows = encoder_inputs(wl, xe, torch, dev)
    return xe.encode(wl.m, wl.n, wl.cfg.n_in, wl.cfg.q, M_rows, mask, planes, alpha, n_out=wl.cfg.n_out)


def clone_layer(L, xe):
    return xe.PackedLayer(L.m, L.n, L.n_in, L.q, L.M_rows, L.enc.clone(), L.mask.clone(), L.patch_off.clone(),
                          L.patch.clone(), L.alpha.clone(), L.n_out)


def tile_rows(L, times, xe, torch):
    """The layer repeated `times` times downwards (m a multiple of 32): pure re-arrangement of the packed
    buffers on the GPU.  Gives a taller matrix of the same recipe without encoding one."""
    assert L.m % 32 == 0
    q = L.q
    U = (L.patch_off.numel() - 1) // q                       # units per plane
    off = L.patch_off.to(torch.int64)
    enc = L.enc.view(q, -1).repeat(1, times).reshape(-1)
    mask = L.mask.repeat(times)
    alpha = L.alpha.repeat(1, times)
    new_off, new_patch, base = [], [], 0
    for p in range(q):
        lo, hi = int(off[p * U]), int(off[(p + 1) * U])
        rel = off[p * U:(p + 1) * U] - lo
        for _ in range(times):
            new_off.append(rel + base)
            new_patch.append(L.patch[lo:hi])
            base += hi - lo
    new_off.append(torch.tensor([base], dtype=torch.int64, device=off.device))
    patch_off = torch.cat(new_off).to(torch.int32)
    patch = torch.cat(new_patch) if base else L.patch[:0]
    return xe.PackedLayer(L.m * times, L.n, L.n_in, q, L.M_rows, enc.contiguous(), mask.contiguous(), patch_off,
                          patch.contiguous(), alpha.contiguous(), L.n_out)


class GraphRunner:
    """Pre-marshalled C-ABI calls over R replicas, issued from a captured HIP graph of min(R, steps) calls
    (so that a replay happens even for few steps) plus an eager remainder.  No Python work per call beyond
    the ctypes call itself."""

    def __init__(self, torch, fn, calls, what):
        self.torch, self.fn, self.calls, self.what = torch, fn, calls, what
        self.R = len(calls)
        self.pos = 0
        self.graph = None
        self.graph_len = 0
        self.replays = 0

    def launch(self, count):
        stream = ctypes.c_void_p(self.torch.cuda.current_stream().cuda_stream)
        for _ in range(count):
            rc = self.fn(*self.calls[self.pos], stream)
            if rc != 0:
                raise RuntimeError(f"{self.what} failed with status {rc}")
            self.pos = (self.pos + 1) % self.R

    def capture(self, steps):
        torch = self.torch
        self.graph_len = max(1, min(self.R, steps))
        self.pos = 0
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            self.launch(self.R)  # warm the code objects before capture
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        self.pos = 0
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            self.launch(self.graph_len)
        self.graph = g

    def run(self, steps, count_replays=False):
        if self.graph is not None:
            n = steps // self.graph_len
            for _ in range(n):
                self.graph.replay()
            if count_replays:
                self.replays += n
            self.pos = 0
            self.launch(steps % self.graph_len)
        else:
            self.launch(steps)

    def time(self, steps, warmup):
        """(wall seconds, HIP-event seconds) of exactly `steps` calls on the current stream."""
        torch = self.torch
        self.run(warmup)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        self.run(steps, count_replays=True)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, e0.elapsed_time(e1) * 1e-3


def replica_count(replica_bytes, step_bytes):
    return int(min(256, max(2, np.ceil(replica_bytes / step_bytes))))


def spmm_runner(xe, torch, layer, x_dev, B, replica_bytes):
    lib = xe.load_library()
    xbytes = x_dev.numel() * x_dev.element_size()
    comp = layer.compressed_bytes()
    step_bytes = comp + xbytes + layer.m * B * 4
    R = replica_count(replica_bytes, step_bytes)
    layers = [layer] + [clone_layer(layer, xe) for _ in range(R - 1)]
    xs = [x_dev] + [x_dev.clone() for _ in range(R - 1)]
    ys = [torch.empty((layer.m, B), dtype=torch.float32, device=x_dev.device) for _ in range(R)]
    structs = [l.c_struct() for l in layers]
    xd = 0 if x_dev.dtype == torch.float32 else 1
    calls = [(ctypes.byref(st), ctypes.c_void_p(x.data_ptr()), xd, x.stride(0), B, ctypes.c_void_p(y.data_ptr()), y.stride(0))
             for st, x, y in zip(structs, xs, ys)]
    runner = GraphRunner(torch, lib.xorenc_spmm, calls, "xorenc_spmm")
    runner.keep = (layers, xs, ys, structs)  # the buffers live as long as the runner
    runner.ys, runner.comp_bytes, runner.step_bytes = ys, comp, step_bytes
    return runner


def decode_runner(xe, torch, layer, kind, replica_bytes):
    lib = xe.load_library()
    out0 = xe.decode(layer, kind)
    out_bytes = out0.numel() * out0.element_size()
    R = min(64, replica_count(replica_bytes, layer.compressed_bytes() + out_bytes))
    layers = [layer] + [clone_layer(layer, xe) for _ in range(R - 1)]
    outs = [out0] + [torch.empty_like(out0) for _ in range(R - 1)]
    structs = [l.c_struct() for l in layers]
    ld = out0.stride(0) if kind != xe.OUT_PLANES else 0
    calls = [(ctypes.byref(st), kind, ctypes.c_void_p(o.data_ptr()), ld) for st, o in zip(structs, outs)]
    runner = GraphRunner(torch, lib.xorenc_decode, calls, "xorenc_decode")
    runner.keep = (layers, outs, structs)
    runner.bytes = layer.compressed_bytes() + out_bytes
    return runner


def kernel_source_digest():
    """Digest of the kernel sources: a traffic profile applies only to the sources it was taken with."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_1905_10138_amd", "csrc")
    for name in ("xorenc_spmm_kernel.h", "xorenc_spmm_small.h", "xorenc_spmm_f4.h", "xorenc_spmm.hip", "xorenc_device.h"):
        with open(os.path.join(src, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_from_profile(workload, B):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload (FETCH_SIZE and
    WRITE_SIZE, scaled by what the same counters read for a copy of known size), or None when there is no
    summary, no row for this B, or the summary was taken with other kernel sources."""
    path = os.path.join(ROOT, "profiles", f"spmm_{workload}_hbm_traffic.md")
    if not os.path.exists(path):
        return None
    text = open(path).read()
    m = re.search(r"kernel sources digest: ([0-9a-f]+)", text)
    if not m or m.group(1) != kernel_source_digest():
        return None
    for line in text.splitlines():
        r = re.match(r"\|[^|]*\(B=(\d+)\)\s*\|\s*[\d.]+\s*\|\s*([\d.]+)\s*\|\s*[\d.]+\s*\|\s*([\d.]+)\s*\|", line)
        if r and int(r.group(1)) == B:
            return {"read_bytes": float(r.group(2)) * 1e6, "write_bytes": float(r.group(3)) * 1e6,
                    "source": os.path.relpath(path, ROOT)}
    return None


def roofline_entry(flops, comp_bytes, total_bytes, sec_per_launch, B, workload=None):
    if B >= 32:
        ach = flops / sec_per_launch / 1e12
        ent = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
               "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
        ideal_us = flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e6
    else:
        ach = comp_bytes / sec_per_launch / 1e9
        ent = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
               "traffic": None, "total_bytes_gbs": total_bytes / sec_per_launch / 1e9}
        ideal_us = comp_bytes / (HBM_PEAK_GBS * 1e9) * 1e6
    ent["roofline_us"] = ideal_us
    ent["launch_bound"] = bool(ideal_us < LAUNCH_BOUND_US)   # the roofline time is below what any launch costs here
    tr = traffic_from_profile(workload, B) if workload else None
    if tr is not None:
        ent["traffic"] = tr["read_bytes"] + tr["write_bytes"]
        ent["traffic_read_bytes"], ent["traffic_write_bytes"], ent["traffic_source"] = tr["read_bytes"], tr["write_bytes"], tr["source"]
    return ent


def x_tensor(torch, wl, B, dev):
    stored, exact = wl.X(B)
    if wl.cfg.x_dtype == "bf16":
        return torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16).to(dev), exact
    return torch.from_numpy(stored).to(dev), exact


def measure_spmm(xe, torch, layer, xg, B, m, n, args, steps, warmup, workload=None):
    runner = spmm_runner(xe, torch, layer, xg, B, args.replica_bytes)
    if not args.no_graph:
        runner.capture(steps)
    wall, ev = runner.time(steps, warmup)
    flops = 2.0 * m * n * B
    res = {"B": B, "ms_per_step": wall * 1e3 / steps, "us_per_launch_events": ev * 1e6 / steps,
           "tflops": flops * steps / wall / 1e12, "compressed_gbs": runner.comp_bytes * steps / wall / 1e9,
           "replicas": runner.R, "graph_replays": runner.replays, "step_bytes": runner.step_bytes,
           "compressed_bytes": runner.comp_bytes,
           "roofline": roofline_entry(flops, runner.comp_bytes, runner.step_bytes, ev / steps, B, workload)}
    return res, runner


def cpu_baseline(wl, B, x_exact, y_gpu_rows, rows):
    """Time the CPU oracle (decode + fp64 product) on the first `rows` rows of the same workload."""
    from oracle import decoder, encoder
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    enc = encoder.encode(wl.keep[:rows], wl.planes[:, :rows], wl.alpha[:, :rows], wl.M, wl.n)  # not timed (offline step)
    times = []
    y = None
    for _ in range(5):
        t0 = time.perf_counter()
        y = decoder.spmm_f64(enc, x_exact)
        times.append(time.perf_counter() - t0)
    t = float(np.median(times))
    err = float(np.linalg.norm(y_gpu_rows - y) / max(np.linalg.norm(y), 1e-300))
    flops = 2.0 * rows * wl.n * B
    return {"value": flops / t / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {rows} of {wl.m} rows of the same W, X and B; median of 5 runs; oracle decode + fp64 W X "
                      "(the oracle's encoder runs before, untimed)",
            "seconds": t, "gpu_vs_oracle_rel_fro": err}


def decode_times(xe, torch, layer, args, kinds=None, steps=200):
    """xorenc_decode on a layer: bit-planes, dense bf16 and dense fp32, over cold replicas from a HIP graph.
    Bytes = compressed bytes read + output bytes written; the fraction is against 8 TB/s."""
    res = {}
    for kind, name in kinds or ((xe.OUT_PLANES, "planes"), (xe.OUT_BF16, "bf16"), (xe.OUT_F32, "f32")):
        runner = decode_runner(xe, torch, layer, kind, args.replica_bytes)
        if not args.no_graph:
            runner.capture(steps)
        wall, ev = runner.time(steps, 20)
        us = ev * 1e6 / steps
        res[name] = {"us": us, "bytes": runner.bytes, "gbs": runner.bytes / (us * 1e-6) / 1e9,
                     "hbm_frac": runner.bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "replicas": runner.R}
        del runner
    return res


def config_table(xe, torch, dev, args, done):
    """Every configuration of the benchmark contract at each of its batch sizes (the headline matrix's
    entries are the ones already measured).  Per entry: microseconds per launch, dense-equivalent TFLOP/s,
    GB/s on the compressed bytes, and the roofline object of its bound."""
    from synth_inputs import CONFIGS, make_workload
    table = {}
    for name, cfg in CONFIGS.items():
        if name in done:
            table[name] = done[name]
            continue
        wl = make_workload(cfg)
        layer = build_layer(wl, xe, torch, dev)
        weights = float(cfg.m) * cfg.n
        ent = {"workload": f"W {cfg.m}x{cfg.n} S={cfg.S} q={cfg.q} n_in={cfg.n_in} n_out={cfg.n_out}, X {cfg.x_dtype}",
               "compressed_bytes": layer.compressed_bytes(), "patches": int(layer.patch.numel()),
               "patches_per_slice": float(layer.patch.numel()) / (cfg.q * cfg.m * -(-cfg.n // cfg.n_out)),
               "stored_bits_per_weight": 8.0 * layer.compressed_bytes() / weights,
               "encrypted_bits_per_weight": 8.0 * layer.enc.numel() / weights, "batches": {}}
        for B in cfg.batches:
            xg, _ = x_tensor(torch, wl, B, dev)
            steps = max(100, args.sweep_steps // 2)
            r, runner = measure_spmm(xe, torch, layer, xg, B, cfg.m, cfg.n, args, steps, 20, workload=name)
            ent["batches"][f"B{B}"] = {k: r[k] for k in ("us_per_launch_events", "tflops", "compressed_gbs", "replicas",
                                                        "graph_replays", "roofline")}
            del runner
        if name == "fig1":      # this configuration asks for decode-only next to the fused product
            ent["decode"] = decode_times(xe, torch, layer, args, ((xe.OUT_PLANES, "planes"), (xe.OUT_BF16, "bf16")))
        table[name] = ent
        del layer
        torch.cuda.empty_cache()
    return table


def marginal_rates(xe, torch, dev, args, wl, layer, base):
    """The headline matrix repeated four times downwards (65536 x 4096, same recipe): time per launch at both
    heights gives the cost of a row of W without the fixed cost of a launch: the slope, as TFLOP/s and GB/s of
    compressed bytes, with the roofline fraction of each."""
    tall = tile_rows(layer, 4, xe, torch)
    res = {"workload": f"{wl.cfg.name} x4 rows: W {4 * wl.m}x{wl.n}", "batches": {}}
    for B in (1, 8, 64, 256):
        if B not in base:
            continue
        xg, _ = x_tensor(torch, wl, B, dev)
        r, runner = measure_spmm(xe, torch, tall, xg, B, 4 * wl.m, wl.n, args, max(100, args.sweep_steps // 2), 20)
        y_tall = runner.ys[0]
        t1, t4 = base[B]["us_per_launch_events"], r["us_per_launch_events"]
        dt = max(t4 - t1, 1e-9) * 1e-6
        ent = {"us_m": t1, "us_4m": t4, "tflops_4m": r["tflops"], "compressed_gbs_4m": r["compressed_gbs"],
               "marginal_tflops": 2.0 * 3 * wl.m * wl.n * B / dt / 1e12,
               "marginal_gbs": 3.0 * base[B]["compressed_bytes"] / dt / 1e9}
        ent["marginal_frac"] = (ent["marginal_tflops"] / MFMA_BF16_PEAK_TFLOPS if B >= 32
                                else ent["marginal_gbs"] / HBM_PEAK_GBS)
        ent["marginal_bound"] = "mfma" if B >= 32 else "hbm"
        ent["rows_repeat_bit_exactly"] = bool(torch.equal(y_tall[:wl.m], y_tall[wl.m:2 * wl.m]))
        res["batches"][f"B{B}"] = ent
        del runner
    del tall
    torch.cuda.empty_cache()
    return res


def wide_extra(xe, torch, dev, args, base_cfg, n_in=24):
    """The default workload re-encoded with slices of 192 bits and n_in = 24 or 20 (the region where the
    paper reports its best ratios, Section 3.3): same or fewer bits per weight for the encrypted stream,
    fewer patches."""
    import dataclasses

    from synth_inputs import make_workload
    cfg = dataclasses.replace(base_cfg, n_out=192, n_in=n_in)
    wl = make_workload(cfg)
    layer = build_layer(wl, xe, torch, dev)
    res = {"workload": f"{cfg.name}: W {cfg.m}x{cfg.n} S={cfg.S} q={cfg.q} n_in={n_in} n_out=192 bf16",
           "compressed_bytes": layer.compressed_bytes(), "patches": int(layer.patch.numel())}
    for B in (8, 64):
        xg, _ = x_tensor(torch, wl, B, dev)
        r, runner = measure_spmm(xe, torch, layer, xg, B, cfg.m, cfg.n, args, max(200, args.sweep_steps), 50)
        res[f"B{B}_us_per_launch"] = r["us_per_launch_events"]
        res[f"B{B}_tflops"] = r["tflops"]
        res[f"B{B}_compressed_gbs"] = r["compressed_gbs"]
        del runner
    if not args.no_decode:
        res["decode"] = decode_times(xe, torch, layer, args)
    return res


def storage_extra(xe, layer):
    """Bits per weight of the quantised stream (everything but the mask and alpha): this library's packed
    layout (enc + patch entries of 16 bits + one 32-bit offset per unit) next to the paper's format as a bit
    stream (Section 3.2) with one n_patch width per plane and per block of 1024 and 32 slices (Section 5.2)."""
    host = layer.to_host()
    w_c, keep, n_patch, d_patch = xe.unpack(host)
    weights = float(host.m) * host.n
    res = {"packed_bits_per_weight": 8.0 * (host.enc.nbytes + host.patch.nbytes + host.patch_off.nbytes) / weights,
           "mask_bits_per_weight": 8.0 * host.mask.nbytes / weights, "patches": int(d_patch.size)}
    for name, blk in (("plane", n_patch.shape[1]), ("1024", 1024), ("32", 32)):
        sz = xe.paper_sizes(host.m, host.n, host.n_in, host.q, n_patch, blk, host.n_out)
        res[f"paper_bits_per_weight_block_{name}"] = (sz["total_bits"] - sz["header_bits"]) / weights
        res[f"paper_header_bits_per_weight_block_{name}"] = sz["header_bits"] / weights
    return res


def encoder_extra(xe, torch, dev, base_cfg):
    """Both GPU encoders (Algorithm 1; the 2^n_in search of Section 5.2) on the default matrix, at its own
    slice geometry, at n_out = 128 / n_in = 16 and at the paper's preferred n_out = 192 / n_in = 20 (Section 3.3:
    2^20 inputs per slice).  Times are host wall-clock around the binding call
    (buffer allocation, the kernels, one synchronisation to read the patch total), best of three."""
    import dataclasses

    from synth_inputs import make_workload
    res = []
    for n_out, n_in in ((base_cfg.n_out, base_cfg.n_in), (128, 16), (192, 20)):
        cfg = dataclasses.replace(base_cfg, n_out=n_out, n_in=n_in)
        if n_in > 24:
            continue
        wl = make_workload(cfg)
        mask, planes, alpha, M_rows = encoder_inputs(wl, xe, torch, dev)
        slices = cfg.q * wl.m * (-(-wl.n // n_out))
        ent = {"n_out": n_out, "n_in": n_in, "slices": slices}
        for key, fn in (("algorithm1", xe.encode), ("exhaustive", xe.encode_exhaustive)):
            best = float("inf")
            for _ in range(4):      # the first call warms up
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                L = fn(wl.m, wl.n, n_in, cfg.q, M_rows, mask, planes, alpha, n_out=n_out)
                torch.cuda.synchronize()
                best = min(best, time.perf_counter() - t0)
            ent[key] = {"ms": best * 1e3, "patches": int(L.patch.numel())}
        ent["exhaustive"]["inputs_tried_per_s"] = slices * float(1 << n_in) / (ent["exhaustive"]["ms"] * 1e-3)
        res.append(ent)
    return res


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_1905_10138_amd as xe
    from synth_inputs import CONFIGS, make_workload

    xe.load_library()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    cfg = CONFIGS[args.workload]
    t_gen = time.perf_counter()
    wl = make_workload(cfg)
    layer = build_layer(wl, xe, torch, dev)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    xg, xexact = x_tensor(torch, wl, args.batch, dev)
    main_res, runner = measure_spmm(xe, torch, layer, xg, args.batch, wl.m, wl.n, args, args.steps, args.warmup,
                                    workload=cfg.name)
    y0 = runner.ys[0].cpu().numpy()
    del runner

    by_batch = {args.batch: main_res}
    sweep = []
    for tok in [t for t in args.sweep.split(",") if t.strip()]:
        B = int(tok)
        if B == args.batch or B not in cfg.batches:
            continue
        xs, _ = x_tensor(torch, wl, B, dev)
        r, rn = measure_spmm(xe, torch, layer, xs, B, wl.m, wl.n, args, args.sweep_steps,
                             max(10, args.sweep_steps // 10), workload=cfg.name)
        del rn
        sweep.append(r)
        by_batch[B] = r

    weights = float(cfg.m) * cfg.n
    out = {
        "metric": "fused decode+SpMM TFLOP/s & compressed-HBM GB/s (% roofline) at 1 MI355X",
        "value": main_res["tflops"], "unit": "TFLOP/s (dense-equivalent 2*m*n*B per step)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.x_dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: W {cfg.m}x{cfg.n} S={cfg.S} q={cfg.q} n_in={cfg.n_in} n_out=64, "
                               f"X {cfg.n}x{args.batch} {cfg.x_dtype}",
                   "B": args.batch, "replicas": main_res["replicas"],
                   "graph": bool(main_res["graph_replays"] > 0), "graph_replays": main_res["graph_replays"],
                   "patches": int(layer.patch.numel()), "compressed_bytes": main_res["compressed_bytes"],
                   "setup_seconds": t_gen, "kernel_sources_digest": kernel_source_digest()},
        "compressed_hbm_gbs": main_res["compressed_gbs"],
        "us_per_launch": main_res["us_per_launch_events"],
        "roofline": main_res["roofline"],
        "sweep": sweep,
    }
    extra = {}
    if not args.no_configs:
        mine = {"workload": f"W {cfg.m}x{cfg.n} S={cfg.S} q={cfg.q} n_in={cfg.n_in} n_out={cfg.n_out}, X {cfg.x_dtype}",
                "compressed_bytes": layer.compressed_bytes(), "patches": int(layer.patch.numel()),
                "patches_per_slice": float(layer.patch.numel()) / (cfg.q * cfg.m * -(-cfg.n // cfg.n_out)),
                "stored_bits_per_weight": 8.0 * layer.compressed_bytes() / weights,
                "encrypted_bits_per_weight": 8.0 * layer.enc.numel() / weights,
                "batches": {f"B{B}": {k: r[k] for k in ("us_per_launch_events", "tflops", "compressed_gbs", "replicas",
                                                        "graph_replays", "roofline")}
                            for B, r in sorted(by_batch.items())}}
        extra["configs"] = config_table(xe, torch, dev, args, {cfg.name: mine})
    if not args.no_marginal and cfg.m % 32 == 0 and cfg.m * 4 * cfg.n <= (1 << 29):
        extra["marginal"] = marginal_rates(xe, torch, dev, args, wl, layer, by_batch)
    if not args.no_fig1 and cfg.name != "fig1" and args.no_configs:
        from synth_inputs import make_workload as mk
        f1 = mk(CONFIGS["fig1"])
        l1 = build_layer(f1, xe, torch, dev)
        extra["fig1"] = {"decode": decode_times(xe, torch, l1, args, ((xe.OUT_PLANES, "planes"), (xe.OUT_BF16, "bf16")))}
    if not args.no_wide and cfg.n_out == 64:
        extra["n_out_192"] = wide_extra(xe, torch, dev, args, cfg)
        extra["n_out_192_n_in_20"] = wide_extra(xe, torch, dev, args, cfg, n_in=20)
    extra["storage"] = storage_extra(xe, layer)
    if not args.no_decode:
        extra["decode"] = decode_times(xe, torch, layer, args)
    if not args.no_encoder:
        extra["encoder"] = encoder_extra(xe, torch, dev, cfg)
    if args.copy_calibration:
        a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        extra["copy_calibration_bytes"] = int(a.numel())
    out.update(extra)
    if not args.no_cpu_baseline:
        rows = args.cpu_rows or wl.m
        out["cpu_baseline"] = cpu_baseline(wl, args.batch, xexact, y0[:rows].astype(np.float64), rows)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
