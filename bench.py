#!/usr/bin/env python3
"""Benchmark of the generalized sparse convolution hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch that is already resident in HBM:
  sp_coords_build (hash + merge duplicates) -> sp_kmap_build (3x3x3, stride 1) -> sp_conv_fwd
  -> sp_conv_bwd_data -> sp_conv_bwd_weight.
Workload: benchmark configs[1] (8 clouds x 20k surface points on a 128^3 grid, Cin=32, Cout=64, fp32).

Prints ONE JSON line.  `value` is the effective TFLOP/s of the step: the active multiply-adds of
fwd + dgrad + wgrad (2 * 3 * pairs * Cin * Cout flops) divided by the time of the WHOLE step, map
building included.  Per-stage figures, the kernel-map rate, the roofline of the dominant kernel and the
CPU oracle's rate on the same workload ride along in the same line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_F32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix-core peak
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

# HBM-side bytes per launch of the forward gather kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each
# scaled by what the counter reads for a plain copy of known size (see the files under profiles/).
MEASURED_TRAFFIC_BYTES = {
    "cfg1_k3s1_c32x64_f32": 92.6e6,   # profiles/step_cfg1_k3s1_c32x64_f32.txt: 66.8 MB read + 25.8 MB written
}

WORKLOADS = {
    # name: (config index, kernel, stride, dilation, cin, cout, bf16)
    "cfg1_k3s1_c32x64_f32": (1, 3, 1, 1, 32, 64, False),
    "cfg0_k3s1_c16x16_f32": (0, 3, 1, 1, 16, 16, False),
    "cfg3_k3s1_c64x64_bf16": (3, 3, 1, 1, 64, 64, True),
    "cfg4_k3s1_c64x64_bf16": (4, 3, 1, 1, 64, 64, True),
    "cfg4_k3s1d2_c64x64_bf16": (4, 3, 1, 2, 64, 64, True),
    "cfg2_k2s2_c64x128_bf16": (2, 2, 2, 1, 64, 128, True),
}


def cpu_baseline(raw, K, stride, dil, cin, cout, bf16, seed):
    """The CPU oracle, as it stands, on the full workload once (single thread)."""
    import oracle
    from paper_2012_13846_amd import spgen
    oracle.build()
    t0 = time.perf_counter()
    c_in, _ = oracle.unique_coords(raw)
    c_out, _, _ = oracle.strided_coords(c_in, 1, stride)
    pin, pout, counts = oracle.kernel_map(c_in, c_out, K, dil)
    t_map = time.perf_counter() - t0
    X = spgen.features(seed, len(c_in), cin, bf16)
    dY = spgen.features(seed + 1, len(c_out), cout, bf16)
    W = spgen.weights(seed + 2, K ** 3, cin, cout, bf16)
    t1 = time.perf_counter()
    oracle.conv_fwd(pin, pout, counts, X, W, len(c_out))
    oracle.conv_bwd_data(pin, pout, counts, dY, W, len(c_in))
    oracle.conv_bwd_weight(pin, pout, counts, X, dY)
    t_conv = time.perf_counter() - t1
    flops = 2.0 * 3.0 * float(counts.sum()) * cin * cout
    total = t_map + t_conv
    return {"value": flops / total / 1e12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "sample": "full workload, one pass (coords + kernel map + fwd + dgrad + wgrad), gcc -O2 scalar fp64",
            "seconds": round(total, 3), "map_seconds": round(t_map, 3),
            "kmap_mvoxels_per_s": len(c_in) / t_map / 1e6}


STACK_CHANNELS = [32, 32, 64, 64, 128, 128, 256, 256, 256]  # input features, then the 8 convs' outputs
STACK_STRIDES = [1, 1, 1, 2, 1, 2, 1, 1]                     # two stride-2 downsamples
STACK_CLASSES = 40


def run_stack(args, sp, spgen, torch):
    """Config 3: one training step (forward, loss, backward) of the 8-conv sparse ResNet-style stack on a
    micro-batch of 4 clouds, bf16 features and weights with fp32 accumulation.  A step is: coordinate hashing,
    the 5 kernel maps of the hierarchy, 8 x (conv, BN+ReLU), per-cloud average pool, linear, softmax
    cross-entropy, and every layer's backward (BN, data gradient, weight gradient)."""
    cfg = 3
    raw_np = spgen.coords_config(cfg)
    raw = torch.from_numpy(raw_np).cuda()
    bf = torch.bfloat16
    nb = int(raw_np[:, 0].max()) + 1
    rng = np.random.default_rng(spgen.seed_for(cfg, 0, stream=2))
    W = [torch.from_numpy(spgen.weights(spgen.seed_for(cfg, l, stream=3), 27, STACK_CHANNELS[l], STACK_CHANNELS[l + 1],
                                        True)).cuda().to(bf) for l in range(8)]
    gamma = [torch.ones(c, device="cuda") for c in STACK_CHANNELS[1:]]
    beta = [torch.zeros(c, device="cuda") for c in STACK_CHANNELS[1:]]
    w_fc = torch.from_numpy((rng.standard_normal((STACK_CLASSES, 256)) / 16).astype(np.float32)).cuda()
    b_fc = torch.zeros(STACK_CLASSES, device="cuda")
    labels = torch.from_numpy(rng.integers(0, STACK_CLASSES, nb).astype(np.int32)).cuda()

    info = {}

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        c0 = sp.sp_coords_build(raw, 1)
        maps, by_key, cur, level, handles = [], {}, c0, 0, [c0]
        for st in STACK_STRIDES:                      # layers on one level with one stride share their map
            if (level, st) not in by_key:
                km, co = sp.sp_kmap_build(cur, 3, st, 1)
                by_key[(level, st)] = (km, co)
                handles += [km, co]
            km, co = by_key[(level, st)]
            maps.append(km)
            if st > 1:
                cur, level = co, level + 1
        mark(1)
        if "x0" not in info:                          # input features: fixed after the first step (same coordinates)
            info["x0"] = torch.from_numpy(spgen.features(spgen.seed_for(cfg, 0, stream=1), c0.n, 32, True)).cuda().to(bf)
            info["pairs"] = [m.total for m in maps]
            info["rows"] = [c0.n] + [m.n_out for m in maps]
        x = info["x0"]
        saved = []
        for l in range(8):
            z = sp.sp_conv_fwd(maps[l], x, W[l])
            y, mean, rstd = sp.sp_bn_relu_fwd(z, gamma[l], beta[l])
            saved.append((x, z, y, mean, rstd))
            x = y
        coords_last = cur.coords()
        pooled, counts = sp.sp_pool_avg_fwd(coords_last, x, nb)
        logits = sp.sp_linear_fwd(pooled, w_fc, b_fc)
        loss, dlogits = sp.sp_softmax_ce(logits, labels)
        mark(2)
        dpooled, dw_fc, db_fc = sp.sp_linear_bwd(pooled, w_fc, dlogits)
        g = sp.sp_pool_avg_bwd(coords_last, dpooled, counts, x.shape[0], bf)
        for l in reversed(range(8)):
            xin, z, y, mean, rstd = saved[l]
            dz, dgamma, dbeta = sp.sp_bn_relu_bwd(z, y, g, gamma[l], mean, rstd)
            dw = sp.sp_conv_bwd_weight(maps[l], xin, dz)
            g = sp.sp_conv_bwd_data(maps[l], dz, W[l])
        mark(3)
        info["loss"] = loss
        for h in handles:
            h.close()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(ev[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    names = ["coords_and_maps", "forward", "backward"]
    stage_ms = {n: float(np.mean([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(args.steps)]))
                for j, n in enumerate(names)}
    flops_layer = [2.0 * info["pairs"][l] * STACK_CHANNELS[l] * STACK_CHANNELS[l + 1] for l in range(8)]
    flops_step = 3.0 * sum(flops_layer)

    # dominant kernel: the forward convolution of the widest layer (256 -> 256 on the twice-downsampled level)
    c0 = sp.sp_coords_build(raw, 1)
    cur, hs = c0, [c0]
    for _ in range(2):
        km, co = sp.sp_kmap_build(cur, 3, 2, 1)
        hs += [km, co]
        cur = co
    km, co = sp.sp_kmap_build(cur, 3, 1, 1)
    hs += [km, co]
    x = torch.randn(km.n_in, 256, device="cuda").to(bf)
    y = torch.empty(km.n_out, 256, device="cuda", dtype=bf)
    for _ in range(3):
        sp.sp_conv_fwd(km, x, W[7], out=y)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for _ in range(reps):
        sp.sp_conv_fwd(km, x, W[7], out=y)
    e1.record()
    torch.cuda.synchronize()
    conv_s = e0.elapsed_time(e1) / reps * 1e-3
    fl = 2.0 * km.total * 256 * 256
    for h in hs:
        h.close()
    out = {
        "metric": "sparse-conv effective TFLOP/s (active MACs) + kernel-map Mvoxels/s, 1 GPU",
        "value": flops_step / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "clouds": nb, "n_raw": int(raw.shape[0]), "rows_per_level": info["rows"],
                   "pairs_per_layer": info["pairs"], "channels": STACK_CHANNELS, "strides": STACK_STRIDES,
                   "step": "coords + 5 kernel maps + 8x(conv, BN+ReLU) + pool + linear + CE + full backward"},
        "stages": {n: {"ms": round(stage_ms[n], 4)} for n in names},
        "conv_gflop_per_step": round(flops_step / 1e9, 1),
        "loss": float(info["loss"].item()),
        "roofline": {"bound": "mfma", "kernel": "gather_dense_kernel<256,256> (sp_conv_fwd, layer 7/8)",
                     "achieved": fl / conv_s / 1e12, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": fl / conv_s / 1e12 / PEAK_BF16_MFMA_TFLOPS, "traffic": None,
                     "launch_us": round(conv_s * 1e6, 2), "flops_per_launch": fl},
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg1_k3s1_c32x64_f32", choices=sorted(WORKLOADS) + ["cfg3_stack_bf16"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of known size (256 MiB read + 256 MiB written per launch): "
                         "the reference the FETCH_SIZE / WRITE_SIZE counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2012_13846_amd import binding as sp
    from paper_2012_13846_amd import spgen
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sp.lib()
    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_launch": src.numel() * 4,
                          "bytes_written_per_launch": src.numel() * 4, "launches": 10}))
        return

    if args.workload == "cfg3_stack_bf16":
        run_stack(args, sp, spgen, torch)
        return
    cfg, K, stride, dil, cin, cout, bf16 = WORKLOADS[args.workload]
    seed = spgen.seed_for(cfg, 0, stream=1)
    raw_np = spgen.coords_config(cfg)
    raw = torch.from_numpy(raw_np).cuda()
    tdt = torch.bfloat16 if bf16 else torch.float32

    # sizes of this workload (also the first warm-up of the pool)
    c = sp.sp_coords_build(raw, 1)
    km, co = sp.sp_kmap_build(c, K, stride, dil)
    n_in, n_out, pairs = km.n_in, km.n_out, km.total
    x = torch.from_numpy(spgen.features(seed, n_in, cin, bf16)).cuda().to(tdt)
    dy = torch.from_numpy(spgen.features(seed + 1, n_out, cout, bf16)).cuda().to(tdt)
    w = torch.from_numpy(spgen.weights(seed + 2, K ** 3, cin, cout, bf16)).cuda().to(tdt)
    y = torch.empty((n_out, cout), dtype=tdt, device="cuda")
    dx = torch.empty((n_in, cin), dtype=tdt, device="cuda")
    dw = torch.empty((K ** 3, cout, cin), dtype=torch.float32, device="cuda")
    del km, co, c

    names = ["coords_build", "kmap_build", "conv_fwd", "conv_bwd_data", "conv_bwd_weight"]

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record()          # torch's current stream = the stream the library launches on
        mark(0)
        c = sp.sp_coords_build(raw, 1)
        mark(1)
        km, co = sp.sp_kmap_build(c, K, stride, dil)
        mark(2)
        sp.sp_conv_fwd(km, x, w, out=y)
        mark(3)
        sp.sp_conv_bwd_data(km, dy, w, out=dx)
        mark(4)
        sp.sp_conv_bwd_weight(km, x, dy, out=dw)
        mark(5)
        km.close(), co.close(), c.close()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(ev[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    stage_ms = {n: float(np.mean([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(args.steps)]))
                for j, n in enumerate(names)}
    ms_per_step = elapsed / args.steps * 1e3
    flops_conv = 2.0 * pairs * cin * cout
    value = 3.0 * flops_conv / (ms_per_step * 1e-3) / 1e12
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS

    # Dominant kernel: the gather-GEMM kernel of sp_conv_fwd (the same kernel serves the data gradient).
    # Timed live with events on the launch stream over a run of back-to-back calls on the last step's map;
    # each call is that kernel plus the ~3 us fragment-major weight copy that precedes it.
    c = sp.sp_coords_build(raw, 1)
    km, co = sp.sp_kmap_build(c, K, stride, dil)
    reps = 30
    for _ in range(3):
        sp.sp_conv_fwd(km, x, w, out=y)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        sp.sp_conv_fwd(km, x, w, out=y)
    e1.record()
    torch.cuda.synchronize()
    fwd_s = e0.elapsed_time(e1) / reps * 1e-3
    km.close(), co.close(), c.close()
    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload)
    # which of the library's gather kernels sp_conv_fwd picks for this shape (same rule as csrc/sp_conv.hip)
    fill = pairs / float(n_out * K ** 3)
    dense = bf16 and cin in (64, 128, 256) and cout % 64 == 0 and fill >= (0.25 if cin == 64 else 0.06)
    kernel_name = "gather_dense_kernel" if dense else "gather_wave_kernel"
    roofline = {"bound": "mfma", "kernel": kernel_name + " (sp_conv_fwd)",
                "achieved": flops_conv / fwd_s / 1e12, "peak": peak, "unit": "TFLOP/s",
                "frac": flops_conv / fwd_s / 1e12 / peak, "traffic": traffic,
                "launch_us": round(fwd_s * 1e6, 2), "flops_per_launch": flops_conv}
    esz = 2 if bf16 else 4
    compulsory = n_in * cin * esz + n_out * cout * esz + pairs * 6 + K ** 3 * cin * cout * esz
    stages = {n: {"ms": round(stage_ms[n], 4)} for n in names}
    for n in ("conv_fwd", "conv_bwd_data", "conv_bwd_weight"):
        stages[n]["tflops"] = round(flops_conv / (stage_ms[n] * 1e-3) / 1e12, 3)
        stages[n]["frac_mfma_peak"] = round(flops_conv / (stage_ms[n] * 1e-3) / 1e12 / peak, 4)
    stages["conv_fwd"]["compulsory_GBps"] = round(compulsory / fwd_s / 1e9, 1)
    map_ms = stage_ms["coords_build"] + stage_ms["kmap_build"]

    out = {
        "metric": "sparse-conv effective TFLOP/s (active MACs) + kernel-map Mvoxels/s, 1 GPU",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "n_raw": int(raw.shape[0]), "n_in": n_in, "n_out": n_out,
                   "pairs": pairs, "kernel": K, "stride": stride, "dilation": dil, "cin": cin, "cout": cout,
                   "step": "coords_build + kmap_build + fwd + dgrad + wgrad"},
        "kmap_mvoxels_per_s": n_in / (stage_ms["kmap_build"] * 1e-3) / 1e6,
        "coords_mpoints_per_s": int(raw.shape[0]) / (stage_ms["coords_build"] * 1e-3) / 1e6,
        "map_build_ms": round(map_ms, 4),
        "stages": stages,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(raw_np, K, stride, dil, cin, cout, bf16, seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
