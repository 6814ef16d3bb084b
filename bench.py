#!/usr/bin/env python3
"""Benchmark of the fused decode + W X path on one MI355X.

A step is one xorenc_spmm call: the whole hot path (stream-in, GF(2) decode, patch flips, mask,
dequantise, contraction) over one batch X of the workload.  Inputs are synthetic (seeded, see
synth_inputs), encoded on the GPU by xorenc_encode before timing, and resident in HBM.  To keep
the timed reads cold (the layers are far smaller than the 256 MB last-level cache) the steps walk
round-robin over R replicas of the compressed layer, X and Y with R * bytes >= 1 GiB.  Steps are
issued back to back on one stream from a captured HIP graph so that host launch cost does not
pace the GPU.

Prints ONE JSON line (see README for the fields).
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


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
    ap.add_argument("--decode-only", action="store_true", help="also time xorenc_decode (planes) on the workload")
    ap.add_argument("--no-wide", action="store_true", help="skip the n_out=192 / n_in=24 extra on the same matrix")
    ap.add_argument("--no-decode", action="store_true", help="skip the timing of xorenc_decode on the workload")
    ap.add_argument("--no-encoder", action="store_true", help="skip the timing of the two GPU encoders")
    ap.add_argument("--no-fig1", action="store_true", help="skip the Fig. 1-shaped extra (decode-only and fused, B=64)")
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


class SpmmRunner:
    """Pre-marshalled xorenc_spmm calls over R replicas (no Python work per step beyond the ctypes call)."""

    def __init__(self, xe, torch, layer, x_dev, B, replica_bytes):
        self.torch = torch
        self.lib = xe.load_library()
        self.B = B
        xbytes = x_dev.numel() * x_dev.element_size()
        ybytes = layer.m * B * 4
        self.comp_bytes = layer.compressed_bytes()
        self.step_bytes = self.comp_bytes + xbytes + ybytes
        R = int(min(256, max(2, np.ceil(replica_bytes / self.step_bytes))))
        self.layers = [layer] + [clone_layer(layer, xe) for _ in range(R - 1)]
        self.xs = [x_dev] + [x_dev.clone() for _ in range(R - 1)]
        self.ys = [torch.empty((layer.m, B), dtype=torch.float32, device=x_dev.device) for _ in range(R)]
        self.structs = [l.c_struct() for l in self.layers]
        xd = 0 if x_dev.dtype == torch.float32 else 1
        self.calls = []
        for st, x, y in zip(self.structs, self.xs, self.ys):
            self.calls.append((ctypes.byref(st), ctypes.c_void_p(x.data_ptr()), xd, x.stride(0), B,
                               ctypes.c_void_p(y.data_ptr()), y.stride(0)))
        self.R = R
        self.pos = 0
        self.graph = None

    def launch(self, count):
        fn = self.lib.xorenc_spmm
        stream = ctypes.c_void_p(self.torch.cuda.current_stream().cuda_stream)
        for _ in range(count):
            rc = fn(*self.calls[self.pos], stream)
            if rc != 0:
                raise RuntimeError(f"xorenc_spmm failed with status {rc}")
            self.pos = (self.pos + 1) % self.R

    def capture(self):
        """Capture one rotation (R steps) into a HIP graph."""
        torch = self.torch
        self.pos = 0
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            self.launch(self.R)  # warm the code objects before capture
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            self.launch(self.R)
        self.graph = g

    def run(self, steps):
        """Issue exactly `steps` steps (graph replays of R steps + an eager remainder)."""
        if self.graph is not None:
            for _ in range(steps // self.R):
                self.graph.replay()
            self.pos = 0
            self.launch(steps % self.R)
        else:
            self.launch(steps)

    def time(self, steps, warmup):
        torch = self.torch
        self.run(warmup)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        self.run(steps)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, e0.elapsed_time(e1) * 1e-3


def roofline_entry(flops, comp_bytes, total_bytes, sec_per_launch, B):
    if B >= 32:
        ach = flops / sec_per_launch / 1e12
        return {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
    ach = comp_bytes / sec_per_launch / 1e9
    return {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "traffic": None, "total_bytes_gbs": total_bytes / sec_per_launch / 1e9}


# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), scaled by
# what the same counters read for a 256 MiB device copy in the same run; see profiles/.
# Filled in from the committed profile of this exact command; None = not measured.
MEASURED_TRAFFIC = {
    # profiles/spmm_large_q1_hbm_traffic.md: bytes read + written per launch
    "large_q1:B1": {"read_bytes": 9.98e6, "write_bytes": 0.07e6},
    "large_q1:B8": {"read_bytes": 10.48e6, "write_bytes": 0.52e6},
    "large_q1:B64": {"read_bytes": 14.16e6, "write_bytes": 4.19e6},
    "large_q1:B256": {"read_bytes": 26.75e6, "write_bytes": 16.78e6},
}


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


def fig1_extra(xe, torch, dev, args):
    """The Fig. 1-shaped configuration: decode-only (planes and dense bf16) and the fused product at B = 64."""
    from synth_inputs import CONFIGS, make_workload
    cfg = CONFIGS["fig1"]
    wl = make_workload(cfg)
    layer = build_layer(wl, xe, torch, dev)
    stored, _ = wl.X(64)
    xg = torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16).to(dev)
    runner = SpmmRunner(xe, torch, layer, xg, 64, args.replica_bytes)
    if not args.no_graph:
        runner.capture()
    steps = max(200, args.sweep_steps)
    wall, ev = runner.time(steps, 50)
    res = {"workload": f"fig1: W {cfg.m}x{cfg.n} S={cfg.S} q=1 n_in=16, X {cfg.n}x64 bf16",
           "fused_us_per_launch": ev * 1e6 / steps, "fused_tflops": 2.0 * cfg.m * cfg.n * 64 * steps / wall / 1e12,
           "compressed_bytes": runner.comp_bytes, "replicas": runner.R}
    for kind, name, width in ((xe.OUT_PLANES, "decode_planes", 8 * ((cfg.n + 63) // 64) / cfg.n),
                              (xe.OUT_BF16, "decode_bf16", 2.0)):
        out = xe.decode(layer, kind)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(200):
            xe.decode(layer, kind, out=out)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 200
        res[name + "_us"] = us
        res[name + "_gbs"] = (layer.compressed_bytes() + cfg.m * cfg.n * width) / (us * 1e-6) / 1e9
    return res


def decode_extra(xe, torch, layer, reps=50):
    """xorenc_decode on the main workload's layer: bit-planes, dense bf16 and dense fp32.  Bytes = compressed
    bytes read + output bytes written; the fraction is against 8 TB/s."""
    res = {}
    for kind, name in ((xe.OUT_PLANES, "planes"), (xe.OUT_BF16, "bf16"), (xe.OUT_F32, "f32")):
        out = xe.decode(layer, kind)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            xe.decode(layer, kind, out=out)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        nbytes = layer.compressed_bytes() + out.numel() * out.element_size()
        res[name] = {"us": us, "bytes": nbytes, "gbs": nbytes / (us * 1e-6) / 1e9,
                     "hbm_frac": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}
        del out
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
        stored, _ = wl.X(B)
        xg = torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16).to(dev)
        runner = SpmmRunner(xe, torch, layer, xg, B, args.replica_bytes)
        if not args.no_graph:
            runner.capture()
        steps = max(200, args.sweep_steps)
        wall, ev = runner.time(steps, 50)
        res[f"B{B}_us_per_launch"] = ev * 1e6 / steps
        res[f"B{B}_tflops"] = 2.0 * cfg.m * cfg.n * B * steps / wall / 1e12
        res[f"B{B}_compressed_gbs"] = runner.comp_bytes * steps / wall / 1e9
        del runner
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
    slice geometry and at n_out = 128 / n_in = 16.  Times are host wall-clock around the binding call
    (buffer allocation, three kernels, one synchronisation to read the patch total), best of three."""
    import dataclasses

    from synth_inputs import make_workload
    res = []
    for n_out, n_in in ((base_cfg.n_out, base_cfg.n_in), (128, 16)):
        cfg = dataclasses.replace(base_cfg, n_out=n_out, n_in=n_in)
        if n_in > 16:
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

    def x_for(B):
        stored, exact = wl.X(B)
        if cfg.x_dtype == "bf16":
            return torch.from_numpy(stored.view(np.int16)).view(torch.bfloat16).to(dev), exact
        return torch.from_numpy(stored).to(dev), exact

    def measure(B, steps, warmup):
        xg, xexact = x_for(B)
        runner = SpmmRunner(xe, torch, layer, xg, B, args.replica_bytes)
        if not args.no_graph:
            runner.capture()
        wall, ev = runner.time(steps, warmup)
        flops = 2.0 * wl.m * wl.n * B
        res = {"B": B, "ms_per_step": wall * 1e3 / steps, "us_per_launch_events": ev * 1e6 / steps,
               "tflops": flops * steps / wall / 1e12, "compressed_gbs": runner.comp_bytes * steps / wall / 1e9,
               "replicas": runner.R, "step_bytes": runner.step_bytes, "compressed_bytes": runner.comp_bytes,
               "roofline": roofline_entry(flops, runner.comp_bytes, runner.step_bytes, ev / steps, B)}
        tr = MEASURED_TRAFFIC.get(f"{cfg.name}:B{B}")
        if tr is not None:      # HBM bytes per launch (read + written), rocprofv3 counters scaled by a known copy
            res["roofline"]["traffic"] = tr["read_bytes"] + tr["write_bytes"]
            res["roofline"]["traffic_read_bytes"] = tr["read_bytes"]
            res["roofline"]["traffic_write_bytes"] = tr["write_bytes"]
        return res, runner, xexact

    main_res, runner, xexact = measure(args.batch, args.steps, args.warmup)
    y0 = runner.ys[0].cpu().numpy()

    sweep = []
    for tok in [t for t in args.sweep.split(",") if t.strip()]:
        B = int(tok)
        if B == args.batch or B not in cfg.batches:
            continue
        r, _, _ = measure(B, args.sweep_steps, max(10, args.sweep_steps // 10))
        sweep.append(r)

    extra = {}
    if args.decode_only:
        out = xe.decode(layer, xe.OUT_PLANES)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(200):
            xe.decode(layer, xe.OUT_PLANES, out=out)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 200
        extra["decode_planes_us"] = us
        extra["decode_planes_gbs"] = (layer.compressed_bytes() + out.numel() * 8) / (us * 1e-6) / 1e9

    out = {
        "metric": "fused decode+SpMM TFLOP/s & compressed-HBM GB/s (% roofline) at 1 MI355X",
        "value": main_res["tflops"], "unit": "TFLOP/s (dense-equivalent 2*m*n*B per step)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.x_dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: W {cfg.m}x{cfg.n} S={cfg.S} q={cfg.q} n_in={cfg.n_in} n_out=64, "
                               f"X {cfg.n}x{args.batch} {cfg.x_dtype}",
                   "B": args.batch, "replicas": main_res["replicas"], "graph": not args.no_graph,
                   "patches": int(layer.patch.numel()), "compressed_bytes": main_res["compressed_bytes"],
                   "setup_seconds": t_gen},
        "compressed_hbm_gbs": main_res["compressed_gbs"],
        "us_per_launch": main_res["us_per_launch_events"],
        "roofline": main_res["roofline"],
        "sweep": sweep,
    }
    if not args.no_fig1 and cfg.name != "fig1":
        extra["fig1"] = fig1_extra(xe, torch, dev, args)
    if not args.no_wide and cfg.n_out == 64:
        extra["n_out_192"] = wide_extra(xe, torch, dev, args, cfg)
        extra["n_out_192_n_in_20"] = wide_extra(xe, torch, dev, args, cfg, n_in=20)
    extra["storage"] = storage_extra(xe, layer)
    if not args.no_decode:
        extra["decode"] = decode_extra(xe, torch, layer)
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
