"""SmartProfile (Sec. III-C): per-layer compute time, activation size and parameter size of a sparse layer stack
on the GPU at hand, dumped to a text file that partition.py reads.

As the paper describes it: a warm-up stage of 50 training iterations that keeps the GPU busy, then a profile stage
of 100 iterations that records, for every layer, the total computation time (forward + backward), the activation
size and the weight-parameter size.  The stack profiled here is the library's own: the 8-convolution
ResNet-style stack (3x3x3 sparse convolutions with two stride-2 downsamples, BatchNorm + ReLU after each,
per-cloud average pooling, linear classifier, softmax cross-entropy), bf16 features with fp32 accumulation.
A layer = one convolution with its BatchNorm + ReLU; pooling, classifier and loss are one layer each.
The activation of a sparse layer is a sparse tensor: its coordinate matrix (16 bytes a row) travels with the
feature matrix (Sec. III-B), so both count.

Run on the GPU machine:  python -m paper_2012_13846_amd.smartprofile out.txt [--scale 1.0] [--warmup 50] [--iters 100]
"""
from __future__ import annotations

import argparse
from typing import List

import numpy as np

from . import partition, spgen

CHANNELS = [32, 32, 64, 64, 128, 128, 256, 256, 256]
STRIDES = [1, 1, 1, 2, 1, 2, 1, 1]
CLASSES = 40


def profile_stack(scale: float = 1.0, warmup: int = 50, iters: int = 100, clouds_cfg: int = 3) -> List[partition.LayerRecord]:
    import torch

    from . import binding as sp

    bf = torch.bfloat16
    raw_np = spgen.coords_config(clouds_cfg, scale)
    raw = torch.from_numpy(raw_np).cuda()
    nb = int(raw_np[:, 0].max()) + 1
    rng = np.random.default_rng(spgen.seed_for(clouds_cfg, 0, stream=2))
    W = [torch.from_numpy(spgen.weights(spgen.seed_for(clouds_cfg, l, stream=3), 27, CHANNELS[l], CHANNELS[l + 1], True)).cuda().to(bf)
         for l in range(8)]
    gamma = [torch.ones(c, device="cuda") for c in CHANNELS[1:]]
    beta = [torch.zeros(c, device="cuda") for c in CHANNELS[1:]]
    w_fc = torch.from_numpy((rng.standard_normal((CLASSES, 256)) / 16).astype(np.float32)).cuda()
    b_fc = torch.zeros(CLASSES, device="cuda")
    labels = torch.from_numpy(rng.integers(0, CLASSES, nb).astype(np.int32)).cuda()

    # the coordinate hierarchy and its maps are built once: the profile is of the layers
    c0 = sp.sp_coords_build(raw, 1)
    maps, by_key, cur, level, keep = [], {}, c0, 0, [c0]
    for st in STRIDES:
        if (level, st) not in by_key:
            by_key[(level, st)] = sp.sp_kmap_build(cur, 3, st, 1)
            keep += list(by_key[(level, st)])
        km, co = by_key[(level, st)]
        maps.append(km)
        if st > 1:
            cur, level = co, level + 1
    x0 = torch.from_numpy(spgen.features(spgen.seed_for(clouds_cfg, 0, stream=1), c0.n, CHANNELS[0], True)).cuda().to(bf)
    coords_last = cur.coords()
    names = [f"conv{l}_{CHANNELS[l]}x{CHANNELS[l + 1]}_s{STRIDES[l]}+bn+relu" for l in range(8)] + ["avgpool", "linear", "loss"]
    n_layers = len(names)

    def iteration(ev):
        """One training iteration; ev[l] = (fwd start, fwd end, bwd start, bwd end) events of layer l, or None."""
        def mark(l, i):
            if ev is not None:
                ev[l][i].record()
        x, saved = x0, []
        for l in range(8):
            mark(l, 0)
            z = sp.sp_conv_fwd(maps[l], x, W[l])
            y, mean, rstd = sp.sp_bn_relu_fwd(z, gamma[l], beta[l])
            mark(l, 1)
            saved.append((x, z, y, mean, rstd))
            x = y
        mark(8, 0)
        pooled, counts = sp.sp_pool_avg_fwd(coords_last, x, nb)
        mark(8, 1)
        mark(9, 0)
        logits = sp.sp_linear_fwd(pooled, w_fc, b_fc)
        mark(9, 1)
        mark(10, 0)
        loss, dlogits = sp.sp_softmax_ce(logits, labels)     # the loss layer's backward is part of the same kernel
        mark(10, 1)
        mark(10, 2)
        mark(10, 3)
        mark(9, 2)
        dpooled, dw_fc, db_fc = sp.sp_linear_bwd(pooled, w_fc, dlogits)
        mark(9, 3)
        mark(8, 2)
        g = sp.sp_pool_avg_bwd(coords_last, dpooled, counts, x.shape[0], bf)
        mark(8, 3)
        for l in reversed(range(8)):
            xin, z, y, mean, rstd = saved[l]
            mark(l, 2)
            dz, dgamma, dbeta = sp.sp_bn_relu_bwd(z, y, g, gamma[l], mean, rstd)
            dw = sp.sp_conv_bwd_weight(maps[l], xin, dz)
            g = sp.sp_conv_bwd_data(maps[l], dz, W[l])
            mark(l, 3)
        return saved

    for _ in range(warmup):
        iteration(None)
    torch.cuda.synchronize()
    total = np.zeros(n_layers)
    for _ in range(iters):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n_layers)]
        iteration(ev)
        torch.cuda.synchronize()
        for l in range(n_layers):
            total[l] += ev[l][0].elapsed_time(ev[l][1]) + ev[l][2].elapsed_time(ev[l][3])
    avg_s = total / max(iters, 1) * 1e-3

    records = []
    for l in range(8):
        n_out = maps[l].n_out
        act = n_out * CHANNELS[l + 1] * 2 + n_out * 16                 # bf16 features + int32 coordinates
        par = 27 * CHANNELS[l] * CHANNELS[l + 1] * 2 + 2 * CHANNELS[l + 1] * 4
        records.append(partition.LayerRecord(names[l], float(avg_s[l]), int(act), int(par)))
    records.append(partition.LayerRecord(names[8], float(avg_s[8]), nb * 256 * 4, 0))
    records.append(partition.LayerRecord(names[9], float(avg_s[9]), nb * CLASSES * 4, CLASSES * 256 * 4 + CLASSES * 4))
    records.append(partition.LayerRecord(names[10], float(avg_s[10]), 4, 0))
    for h in keep:
        h.close()
    return records


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("out")
    ap.add_argument("--scale", type=float, default=1.0, help="fraction of the 131072 points per cloud")
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--iters", type=int, default=100)
    ap.add_argument("--gpu-type", default="MI355X")
    args = ap.parse_args()
    rec = profile_stack(args.scale, args.warmup, args.iters)
    partition.write_profile(args.out, args.gpu_type, rec, {"scale": args.scale, "warmup": args.warmup, "iters": args.iters,
                                                          "stack": "8 sparse convs 32-32-64-64-128-128-256-256-256, bf16"})
    print(f"wrote {args.out}: {len(rec)} layers, {sum(r.time_s for r in rec) * 1e3:.3f} ms per iteration")


if __name__ == "__main__":
    main()
