#!/usr/bin/env python3
"""Benchmark of the generalized sparse convolution hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch that is already resident in HBM:
  sp_coords_build (hash + merge duplicates) -> sp_kmap_build -> sp_conv_fwd -> sp_conv_bwd_data
  -> sp_conv_bwd_weight.
Headline workload: benchmark configs[1] (8 clouds x 20k surface points on a 128^3 grid, 3x3x3 stride 1,
Cin=32, Cout=64, fp32).

Prints ONE JSON line.  `value` is the effective TFLOP/s of the headline step: the active multiply-adds of
fwd + dgrad + wgrad (2 * 3 * pairs * Cin * Cout flops) divided by the time of the WHOLE step, map building
included.  The same line carries
  - `roofline`: the dominant kernel of the headline step, timed live with events on the launch stream;
  - `cpu_baseline`: the CPU oracle on the headline workload, one thread and all cores (one process per cloud);
  - `configs`: every other BASELINE config and the paper's sparsity-sweep batches, each with per-stage times,
    the roof that binds each stage (matrix cores or HBM) and the achieved fraction of it; for the two
    map-building stages the algorithmic bytes, achieved GB/s and the fraction of the HBM peak.
`--workload NAME` makes another workload the headline; `--only-headline` skips `configs` (profiling runs).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_F32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix-core peak
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
METRIC = "sparse-conv effective TFLOP/s (active MACs) + kernel-map Mvoxels/s, 1 GPU"

WORKLOADS = {
    # name: (coords source, kernel, stride, dilation, cin, cout, bf16)
    "cfg0_k3s1_c16x16_f32": (("cfg", 0), 3, 1, 1, 16, 16, False),
    "cfg1_k3s1_c32x64_f32": (("cfg", 1), 3, 1, 1, 32, 64, False),
    "cfg2_k2s2_c64x128_bf16": (("cfg", 2), 2, 2, 1, 64, 128, True),
    "cfg3_k3s1_c64x64_bf16": (("cfg", 3), 3, 1, 1, 64, 64, True),
    "cfg4_k3s1_c64x64_bf16": (("cfg", 4), 3, 1, 1, 64, 64, True),
    "cfg4_k3s1d2_c64x64_bf16": (("cfg", 4), 3, 1, 2, 64, 64, True),
    # literal readings of two configs whose text contradicts its own voxel count (latency datapoints)
    "cfg2lit_2048pt_k2s2_c64x128_bf16": (("literal", "cfg2_2048pt"), 2, 2, 1, 64, 128, True),
    "cfg4lit_5cm_k3s1_c64x64_bf16": (("literal", "cfg4_5cm"), 3, 1, 1, 64, 64, True),
}
# the paper's sparsity sweep (Sec. IV-C, Table II): grid, p, clouds per batch (the batch sizes of Table II)
for _g, _p, _b in ((32, 1.0, 256), (32, 0.5, 256), (32, 0.25, 512), (50, 1.0, 128), (50, 0.5, 128), (50, 0.25, 256)):
    WORKLOADS[f"sweep{_g}_p{_p:g}_b{_b}_k3s1_c64x64_f32"] = (("sweep", _g, _p, _b), 3, 1, 1, 64, 64, False)
DEFAULT_EXTRA = [n for n in WORKLOADS if n != "cfg1_k3s1_c32x64_f32"] + ["cfg3_stack_bf16"]


def raw_coords(spgen, src):
    if src[0] == "cfg":
        return spgen.coords_config(src[1])
    if src[0] == "literal":
        return spgen.coords_literal(src[1])
    return spgen.coords_sweep(src[1], src[2], src[3])


# ---------------------------------------------------------------------------------------------------------
# roofs
# ---------------------------------------------------------------------------------------------------------
def conv_roofs(stage, n_in, n_out, pairs, kvol, cin, cout, bf16):
    """T_mfma = 2 * active MACs / matrix-core peak of the dtype; T_hbm = compulsory bytes / HBM peak (every
    feature row once, the neighbour table or the pair lists once, the weights once)."""
    e = 2 if bf16 else 4
    flops = 2.0 * pairs * cin * cout
    if stage == "conv_fwd":
        byts = n_in * cin * e + n_out * cout * e + n_out * kvol * 4 + kvol * cin * cout * e
    elif stage == "conv_bwd_data":
        byts = n_out * cout * e + n_in * cin * e + n_in * kvol * 4 + kvol * cin * cout * e
    else:
        byts = n_in * cin * e + n_out * cout * e + pairs * 8 + kvol * cin * cout * 4
    t_mfma = flops / ((PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS) * 1e12)
    t_hbm = byts / (PEAK_HBM_GBS * 1e9)
    return flops, byts, t_mfma, t_hbm


def conv_stage_entry(stage, ms, n_in, n_out, pairs, kvol, cin, cout, bf16):
    flops, byts, t_mfma, t_hbm = conv_roofs(stage, n_in, n_out, pairs, kvol, cin, cout, bf16)
    t = ms * 1e-3
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS
    return {"ms": round(ms, 4), "tflops": round(flops / t / 1e12, 3), "frac_mfma_peak": round(flops / t / 1e12 / peak, 4),
            "T_mfma_us": round(t_mfma * 1e6, 2), "T_hbm_us": round(t_hbm * 1e6, 2),
            "bound": "mfma" if t_mfma >= t_hbm else "hbm", "frac": round(max(t_mfma, t_hbm) / t, 4)}


def coords_alg_bytes(n_raw, n):
    """Per raw row: 16 B read, one 16-B table slot written, 4 + 4 B slot number written and read, 4 B inverse written;
    per distinct row 16 B of coordinates written."""
    return 44 * n_raw + 16 * n


def kmap_alg_bytes(n_in, n_out, pairs, kvol, K, stride):
    """Output coordinates read (16 B), one 16-B table slot per search, both neighbour tables written once, the
    pair lists (8 B) and one tile list per direction (6 B) per link.  Stride 1 with an odd kernel searches only
    the offsets below the centre and stores one table and one tile list for both directions; a strided map's
    coarse coordinates add the hashing of n_in rows."""
    symmetric = stride == 1 and K % 2 == 1
    if symmetric:
        return n_out * (16 + (kvol // 2) * 16 + kvol * 4) + pairs * 14
    b = n_out * (16 + kvol * 16) + (n_out + n_in) * kvol * 4 + pairs * 20
    if stride > 1:
        b += coords_alg_bytes(n_in, n_out)
    return b


def map_stage_entries(stage_ms, n_raw, n_in, n_out, pairs, kvol, K, stride):
    cb, kb = coords_alg_bytes(n_raw, n_in), kmap_alg_bytes(n_in, n_out, pairs, kvol, K, stride)
    tc, tk = stage_ms["coords_build"] * 1e-3, stage_ms["kmap_build"] * 1e-3
    return {
        "coords_build": {"ms": round(stage_ms["coords_build"], 4), "alg_bytes": cb, "GBps": round(cb / tc / 1e9, 1),
                         "frac_hbm": round(cb / tc / 1e9 / PEAK_HBM_GBS, 4), "mpoints_per_s": round(n_raw / tc / 1e6, 1)},
        "kmap_build": {"ms": round(stage_ms["kmap_build"], 4), "alg_bytes": kb, "GBps": round(kb / tk / 1e9, 1),
                       "frac_hbm": round(kb / tk / 1e9 / PEAK_HBM_GBS, 4), "mvoxels_per_s": round(n_in / tk / 1e6, 1)},
    }


# ---------------------------------------------------------------------------------------------------------
# the CPU oracle beside it
# ---------------------------------------------------------------------------------------------------------
def cpu_info():
    model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return model, os.cpu_count() or 1, usable


def _oracle_pass(args):
    """One pass of the oracle over `raw` (coords + kernel map + fwd + dgrad + wgrad); returns (t_map, t_conv, pairs)."""
    raw, K, stride, dil, cin, cout, bf16, seed = args
    import oracle
    from paper_2012_13846_amd import spgen
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
    return t_map, time.perf_counter() - t1, int(counts.sum())


def cpu_baseline(raw, K, stride, dil, cin, cout, bf16, seed, all_cores=True):
    """The CPU oracle, as it stands, on the full workload: one pass on one thread, and (clouds are independent, no
    link crosses them) one pass with the clouds dealt to one oracle process per usable core."""
    import oracle
    oracle.build()
    model, nproc, usable = cpu_info()
    t_map, t_conv, pairs = _oracle_pass((raw, K, stride, dil, cin, cout, bf16, seed))
    flops = 2.0 * 3.0 * pairs * cin * cout
    total = t_map + t_conv
    out = {"value": flops / total / 1e12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
           "sample": "full workload, one pass (coords + kernel map + fwd + dgrad + wgrad), gcc -O2 scalar fp64",
           "seconds": round(total, 3), "map_seconds": round(t_map, 3),
           "kmap_mvoxels_per_s": round(len(np.unique(raw, axis=0)) / t_map / 1e6, 4),
           "cpu_model": model, "nproc": nproc, "usable_cores": usable}
    clouds = np.unique(raw[:, 0])
    workers = max(1, min(usable, len(clouds), 16))      # a one-GPU machine offers 16 cores, whatever nproc says
    if all_cores and workers > 1:
        import multiprocessing as mp
        shards = [[] for _ in range(workers)]
        for i, b in enumerate(clouds):
            shards[i % workers].append(b)
        jobs = [(np.ascontiguousarray(raw[np.isin(raw[:, 0], s)]), K, stride, dil, cin, cout, bf16, seed) for s in shards]
        with mp.get_context("spawn").Pool(workers) as pool:
            pool.map(_oracle_pass, jobs[:1])                 # processes up, library loaded
            t0 = time.perf_counter()
            res = pool.map(_oracle_pass, jobs, chunksize=1)
            wall = time.perf_counter() - t0
        out["all_cores"] = {"value": 2.0 * 3.0 * sum(r[2] for r in res) * cin * cout / wall / 1e12, "unit": "TFLOP/s",
                            "cores": workers, "seconds": round(wall, 3),
                            "sample": "same workload, clouds dealt to one single-threaded oracle process per core"}
    return out


# ---------------------------------------------------------------------------------------------------------
# one layer: coords + map + fwd + dgrad + wgrad
# ---------------------------------------------------------------------------------------------------------
def measured_roofs(sp, torch):
    """What this GPU reaches on the two roofs' own microbenchmarks (the fractions in this file are against the
    published peaks, these are for context): a plain 256 MiB device copy, and a register-resident MFMA loop."""
    src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    return {"hbm_copy_GBps": round(copy_gbs, 1), "hbm_peak_GBps": PEAK_HBM_GBS,
            "mfma_f32_TFLOPs": round(sp.sp_measure_mfma_peak(torch.float32), 1), "mfma_f32_peak_TFLOPs": PEAK_F32_MFMA_TFLOPS,
            "mfma_bf16_TFLOPs": round(sp.sp_measure_mfma_peak(torch.bfloat16), 1), "mfma_bf16_peak_TFLOPs": PEAK_BF16_MFMA_TFLOPS,
            "note": "copy counts bytes read + written; MFMA loop: 2 wavefronts per SIMD, operands in registers"}


def profile_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 summary of this workload, if it has one: a line
    `roofline_traffic_bytes <kernel name> <bytes>` in profiles/step_<workload>.txt."""
    path = os.path.join(ROOT, "profiles", f"step_{workload}.txt")
    try:
        for line in open(path):
            m = re.match(r"\s*roofline_traffic_bytes\s+(\S+)\s+([0-9.eE+]+)", line)
            if m and m.group(1) == kernel:
                return float(m.group(2)), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def run_layer(name, steps, warmup, sp, spgen, torch, with_roofline):
    src, K, stride, dil, cin, cout, bf16 = WORKLOADS[name]
    seed = spgen.seed_for(src[1] if src[0] == "cfg" else 5, 0, stream=1)
    raw_np = raw_coords(spgen, src)
    raw = torch.from_numpy(raw_np).cuda()
    tdt = torch.bfloat16 if bf16 else torch.float32
    kvol = K ** 3

    c = sp.sp_coords_build(raw, 1)                       # sizes of this workload (also warms the pool)
    km, co = sp.sp_kmap_build(c, K, stride, dil)
    n_in, n_out, pairs = km.n_in, km.n_out, km.total
    x = torch.from_numpy(spgen.features(seed, n_in, cin, bf16)).cuda().to(tdt)
    dy = torch.from_numpy(spgen.features(seed + 1, n_out, cout, bf16)).cuda().to(tdt)
    w = torch.from_numpy(spgen.weights(seed + 2, kvol, cin, cout, bf16)).cuda().to(tdt)
    y = torch.empty((n_out, cout), dtype=tdt, device="cuda")
    dx = torch.empty((n_in, cin), dtype=tdt, device="cuda")
    dw = torch.empty((kvol, cout, cin), dtype=torch.float32, device="cuda")
    up = stride > 1                                      # also time the matching transposed (upsampling) layer
    if up:
        w_up = torch.from_numpy(spgen.weights(seed + 3, kvol, cout, cin, bf16)).cuda().to(tdt)   # cout -> cin channels
        z = torch.empty((n_in, cin), dtype=tdt, device="cuda")
    km.close(), co.close(), c.close()

    names = ["coords_build", "kmap_build", "conv_fwd", "conv_bwd_data", "conv_bwd_weight"] + (["up_fwd"] if up else [])

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
        if up:
            kt = sp.sp_kmap_transpose(km)
            sp.sp_conv_fwd(kt, y, w_up, out=z)
            mark(6)
            kt.close()
        km.close(), co.close(), c.close()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(ev[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_step = {n: [ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(steps)] for j, n in enumerate(names)}
    stage_ms = {n: float(np.mean(v)) for n, v in per_step.items()}
    ms_per_step = elapsed / steps * 1e3
    flops_conv = 2.0 * pairs * cin * cout
    n_conv = 4 if up else 3
    value = n_conv * flops_conv / (ms_per_step * 1e-3) / 1e12

    stages = map_stage_entries(stage_ms, int(raw.shape[0]), n_in, n_out, pairs, kvol, K, stride)
    for n in ("conv_fwd", "conv_bwd_data", "conv_bwd_weight"):
        stages[n] = conv_stage_entry(n, stage_ms[n], n_in, n_out, pairs, kvol, cin, cout, bf16)
    if up:   # transposed layer: sources = coarse rows (n_out), destinations = fine rows (n_in), cout -> cin channels
        stages["up_fwd"] = conv_stage_entry("conv_fwd", stage_ms["up_fwd"], n_out, n_in, pairs, kvol, cout, cin, bf16)
    for n, v in per_step.items():   # "ms" above is the mean over the timed steps
        stages[n]["median_ms"] = round(float(np.median(v)), 4)
        stages[n]["min_ms"] = round(float(np.min(v)), 4)
    entry = {
        "workload": name, "dtype": "bf16" if bf16 else "f32", "n_raw": int(raw.shape[0]), "n_in": n_in, "n_out": n_out,
        "pairs": pairs, "kernel": K, "stride": stride, "dilation": dil, "cin": cin, "cout": cout,
        "steps": steps, "ms_per_step": round(ms_per_step, 4), "tflops_step": round(value, 3),
        "map_build_ms": round(stage_ms["coords_build"] + stage_ms["kmap_build"], 4),
        "map_build_share_of_step": round((stage_ms["coords_build"] + stage_ms["kmap_build"]) / ms_per_step, 3),
        "stages": stages,
    }
    roofline = None
    if with_roofline:
        # Dominant kernel: the gather-GEMM kernel of sp_conv_fwd (the same kernel serves the data gradient), timed
        # live with events on the launch stream over back-to-back calls; each call is that kernel plus, for the
        # link-list kernel, the ~3 us fragment-major weight copy that precedes it.
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
        kernel = sp.sp_conv_kernel_name(km, cin, cout, tdt, 0)
        km.close(), co.close(), c.close()
        flops, byts, t_mfma, t_hbm = conv_roofs("conv_fwd", n_in, n_out, pairs, kvol, cin, cout, bf16)
        traffic, traffic_from = profile_traffic(name, kernel)
        if t_mfma >= t_hbm:
            peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS
            roofline = {"bound": "mfma", "kernel": kernel + " (sp_conv_fwd)", "achieved": flops / fwd_s / 1e12, "peak": peak,
                        "unit": "TFLOP/s", "frac": flops / fwd_s / 1e12 / peak, "flops_per_launch": flops}
        else:
            roofline = {"bound": "hbm", "kernel": kernel + " (sp_conv_fwd)", "achieved": byts / fwd_s / 1e9,
                        "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": byts / fwd_s / 1e9 / PEAK_HBM_GBS,
                        "bytes_per_launch": byts}
        roofline.update({"traffic": traffic, "traffic_from": traffic_from, "launch_us": round(fwd_s * 1e6, 2),
                         "T_mfma_us": round(t_mfma * 1e6, 2), "T_hbm_us": round(t_hbm * 1e6, 2)})
    return entry, roofline, (raw_np, K, stride, dil, cin, cout, bf16, seed)


# ---------------------------------------------------------------------------------------------------------
# the 8-conv stack of BASELINE config 3
# ---------------------------------------------------------------------------------------------------------
STACK_CHANNELS = [32, 32, 64, 64, 128, 128, 256, 256, 256]  # input features, then the 8 convs' outputs
STACK_STRIDES = [1, 1, 1, 2, 1, 2, 1, 1]                     # two stride-2 downsamples
STACK_CLASSES = 40


def run_stack(steps, warmup, sp, spgen, torch):
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
            info["rows"] = [(m.n_in, m.n_out) for m in maps]
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

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(ev[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / steps * 1e3
    names = ["coords_and_maps", "forward", "backward"]
    stage_ms = {n: float(np.mean([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(steps)]))
                for j, n in enumerate(names)}
    flops_layer = [2.0 * info["pairs"][l] * STACK_CHANNELS[l] * STACK_CHANNELS[l + 1] for l in range(8)]
    flops_step = 3.0 * sum(flops_layer)
    # what the roofs allow for the 24 convolution launches of a step (each layer's binding roof, summed)
    roof_fwd = roof_bwd = 0.0
    layers = []
    for l in range(8):
        n_in, n_out = info["rows"][l]
        per = {}
        for st in ("conv_fwd", "conv_bwd_data", "conv_bwd_weight"):
            _, _, t_mfma, t_hbm = conv_roofs(st, n_in, n_out, info["pairs"][l], 27, STACK_CHANNELS[l], STACK_CHANNELS[l + 1], True)
            per[st] = max(t_mfma, t_hbm)
        roof_fwd += per["conv_fwd"]
        roof_bwd += per["conv_bwd_data"] + per["conv_bwd_weight"]
        layers.append({"cin": STACK_CHANNELS[l], "cout": STACK_CHANNELS[l + 1], "stride": STACK_STRIDES[l], "n_in": n_in,
                       "n_out": n_out, "pairs": info["pairs"][l],
                       "roof_us": {k: round(v * 1e6, 1) for k, v in per.items()}})

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
    kernel = sp.sp_conv_kernel_name(km, 256, 256, bf, 0)
    for h in hs:
        h.close()
    traffic, traffic_from = profile_traffic("cfg3_stack_bf16", kernel)
    entry = {
        "workload": "cfg3_stack_bf16", "dtype": "bf16", "clouds": nb, "n_raw": int(raw.shape[0]),
        "channels": STACK_CHANNELS, "strides": STACK_STRIDES, "layers": layers, "steps": steps,
        "step": "coords + 5 kernel maps + 8x(conv, BN+ReLU) + pool + linear + CE + full backward",
        "ms_per_step": round(ms_per_step, 4), "tflops_step": round(flops_step / (ms_per_step * 1e-3) / 1e12, 3),
        "conv_gflop_per_step": round(flops_step / 1e9, 1),
        "stages": {n: {"ms": round(stage_ms[n], 4)} for n in names},
        "conv_roof_sum_us": {"forward": round(roof_fwd * 1e6, 1), "backward": round(roof_bwd * 1e6, 1)},
        "frac_of_conv_roofs": {"forward": round(roof_fwd * 1e3 / stage_ms["forward"], 4),
                               "backward": round(roof_bwd * 1e3 / stage_ms["backward"], 4),
                               "note": "stage times include BN+ReLU, pooling, linear and loss"},
        "map_build_share_of_step": round(stage_ms["coords_and_maps"] / ms_per_step, 3),
        "loss": float(info["loss"].item()),
    }
    roofline = {"bound": "mfma", "kernel": f"{kernel}<256,256> (sp_conv_fwd, layers 7 and 8)",
                "achieved": fl / conv_s / 1e12, "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": fl / conv_s / 1e12 / PEAK_BF16_MFMA_TFLOPS, "traffic": traffic, "traffic_from": traffic_from,
                "launch_us": round(conv_s * 1e6, 2), "flops_per_launch": fl}
    return entry, roofline


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg1_k3s1_c32x64_f32", choices=sorted(WORKLOADS) + ["cfg3_stack_bf16"],
                    help="the headline workload (value, ms_per_step, roofline, cpu_baseline)")
    ap.add_argument("--only-headline", action="store_true", help="skip the other workloads (`configs`)")
    ap.add_argument("--extra-steps", type=int, default=10, help="timed steps of each workload in `configs`")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of known size (256 MiB read + 256 MiB written per launch): "
                         "the reference the FETCH_SIZE / WRITE_SIZE counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    from paper_2012_13846_amd import spgen
    # The CPU oracle runs first, before this process touches the GPU: its all-cores leg starts worker processes.
    cpu = None
    if not args.no_cpu_baseline and not args.copy_calibration:
        import oracle
        oracle.build()
        if args.workload in WORKLOADS:
            src, K, stride, dil, cin, cout, bf16 = WORKLOADS[args.workload]
            seed = spgen.seed_for(src[1] if src[0] == "cfg" else 5, 0, stream=1)
            cpu = cpu_baseline(raw_coords(spgen, src), K, stride, dil, cin, cout, bf16, seed)

    import torch
    from paper_2012_13846_amd import binding as sp
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

    measured = measured_roofs(sp, torch)
    out = {"metric": METRIC, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic"}
    if args.workload == "cfg3_stack_bf16":
        entry, roofline = run_stack(args.steps, args.warmup, sp, spgen, torch)
        out["config"] = {k: entry[k] for k in ("workload", "clouds", "n_raw", "channels", "strides", "step")}
    else:
        entry, roofline, _ = run_layer(args.workload, args.steps, args.warmup, sp, spgen, torch, True)
        out["config"] = {k: entry[k] for k in ("workload", "n_raw", "n_in", "n_out", "pairs", "kernel", "stride", "dilation",
                                               "cin", "cout")}
        out["config"]["step"] = "coords_build + kmap_build + fwd + dgrad + wgrad"
        out["kmap_mvoxels_per_s"] = entry["stages"]["kmap_build"]["mvoxels_per_s"]
        out["coords_mpoints_per_s"] = entry["stages"]["coords_build"]["mpoints_per_s"]
        out["map_build_ms"] = entry["map_build_ms"]
    out.update({"value": entry["tflops_step"], "ms_per_step": entry["ms_per_step"], "dtype": entry["dtype"],
                "stages": entry["stages"], "roofline": roofline, "measured_roofs": measured})
    if not args.only_headline:
        configs = []
        for name in DEFAULT_EXTRA:
            if name == args.workload:
                continue
            t0 = time.perf_counter()
            if name == "cfg3_stack_bf16":
                e, r = run_stack(args.extra_steps, 3, sp, spgen, torch)
            else:
                e, r, oa = run_layer(name, args.extra_steps, 3, sp, spgen, torch, True)
                if not args.no_cpu_baseline and name in ("cfg0_k3s1_c16x16_f32", "cfg2_k2s2_c64x128_bf16"):
                    b = cpu_baseline(*oa, all_cores=False)      # the oracle in full on the two other small configs
                    e["cpu_oracle"] = {k: b[k] for k in ("value", "unit", "cores", "seconds", "map_seconds", "kmap_mvoxels_per_s")}
            e["roofline"] = r
            e["bench_seconds"] = round(time.perf_counter() - t0, 1)
            configs.append(e)
            sp.sp_pool_trim()
            torch.cuda.empty_cache()
        out["configs"] = configs
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out))


if __name__ == "__main__":
    main()
