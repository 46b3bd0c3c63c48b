"""CPU oracle for (a) pooling over a kernel map and (b) the coordinates of a generative transposed convolution.

TEST INFRASTRUCTURE ONLY (tests, smoke check, benchmark's cpu_baseline leg); the product never imports this.

(a) The paper's stacks put pooling layers between the SparseConv blocks (Sec. III, caption of the
partition-overview figure) and give no formula.  The reading taken: pooling is Eq. 2 with the weighted sum
replaced by a reduction over the same neighbour set N(u, C_in): for u in C_out and every channel c,

    max:  y[u,c] = max_{i in N(u, C_in)} x[u+i, c]
    sum:  y[u,c] = sum_{i in N(u, C_in)} x[u+i, c]
    avg:  y[u,c] = sum / |N(u, C_in)|          (the number of inputs PRESENT, not the kernel volume)

An output with no input keeps 0.  Backward: sum passes dy to every linked input, avg passes dy / |N(u)|, max
passes dy to the input that attained the maximum; among equal maxima the link with the LOWEST offset number k
wins (the order a dense window scan meets them with z fastest).
Plain numpy, float64, one offset at a time in offset order (within one offset an output row occurs at most once,
so the per-offset update is a plain gather / compare / scatter).

(b) The paper defines no transposed convolution.  The coordinate-hierarchy-reusing reading is in
oracle.transpose_map.  The generative one creates the finer coordinates instead of looking them up: for an input
set C_in of tensor stride ts_in and a layer of kernel size K and stride s, ts_out = ts_in / s and

    C_out = { u + i_k * ts_out : u in C_in, k in 0..K^3-1 },

the same relation c_fine = c_coarse + i_k * ts_fine that links a stride-s convolution's inputs (fine) to its
outputs (coarse), with every offset of every input row generated.  Rows are numbered in first-occurrence order
over the candidates enumerated input row by input row, offsets in offset order inside a row.

Parity status: both parts are pinned by tests/test_oracle_pins.py (dense max_pool3d / avg_pool3d /
conv_transpose3d with autograd from a library, numpy unique for the row order); nothing here is unpinned.
"""
from __future__ import annotations

import numpy as np

from . import unique_coords

MODES = ("max", "avg", "sum")


def link_counts(pair_out, n_out: int) -> np.ndarray:
    """|N(u, C_in)| per output row: how many links end in it (all offsets)."""
    return np.bincount(np.asarray(pair_out, np.int64), minlength=n_out).astype(np.int64)


def pool_fwd(pair_in, pair_out, counts, X, n_out: int, mode: str):
    """Returns (Y float64 [n_out][c], arg int64 [n_out][c]): arg = offset number of the link that gave the
    maximum (-1 where the row has no link); arg is all -1 for avg / sum."""
    assert mode in MODES
    X = np.asarray(X, np.float64)
    c = X.shape[1]
    Y = np.zeros((n_out, c))
    arg = np.full((n_out, c), -1, np.int64)
    base = 0
    for k, cnt in enumerate(np.asarray(counts, np.int64)):
        i, o = pair_in[base:base + cnt], pair_out[base:base + cnt]
        base += cnt
        if cnt == 0:
            continue
        if mode == "max":
            cand, cur, seen = X[i], Y[o], arg[o] >= 0
            better = ~seen | (cand > cur)          # strictly greater: the lowest offset keeps a tie
            Y[o] = np.where(better, cand, cur)
            arg[o] = np.where(better, k, arg[o])
        else:
            Y[o] += X[i]
    if mode == "avg":
        n = link_counts(pair_out, n_out)
        Y /= np.maximum(n, 1)[:, None]
    return Y, arg


def pool_bwd(pair_in, pair_out, counts, dY, arg, n_in: int, mode: str) -> np.ndarray:
    """dX float64 [n_in][c] from dY [n_out][c] (and the forward pass's arg for max)."""
    assert mode in MODES
    dY = np.asarray(dY, np.float64)
    n_out, c = dY.shape
    dX = np.zeros((n_in, c))
    if mode == "avg":
        dY = dY / np.maximum(link_counts(pair_out, n_out), 1)[:, None]
    base = 0
    for k, cnt in enumerate(np.asarray(counts, np.int64)):
        i, o = pair_in[base:base + cnt], pair_out[base:base + cnt]
        base += cnt
        if cnt == 0:
            continue
        # within one offset an input row occurs at most once: a plain scatter
        dX[i] += np.where(arg[o] == k, dY[o], 0.0) if mode == "max" else dY[o]
    return dX


def kernel_offsets(K: int) -> np.ndarray:
    """[K^3][3] offsets, number k = (ax*K + ay)*K + az (z fastest); odd K centred, even K from 0."""
    ctr = (K - 1) // 2 if K % 2 else 0
    a = np.arange(K) - ctr
    return np.stack(np.meshgrid(a, a, a, indexing="ij"), -1).reshape(-1, 3).astype(np.int32)


def generative_coords(c_in, ts_in: int, K: int, stride: int):
    """Output coordinates of a generative transposed convolution (see the module text).

    Returns (c_out [n_out][4], where [n_in][K^3] = output row of candidate (input row, offset), ts_out)."""
    c_in = np.ascontiguousarray(c_in, np.int32)
    if ts_in % stride:
        raise ValueError("the input tensor stride must be a multiple of the layer stride")
    ts_out = ts_in // stride
    off = kernel_offsets(K) * ts_out
    cand = np.repeat(c_in[:, None, :], K ** 3, axis=1)
    cand[:, :, 1:] += off[None, :, :]
    c_out, inverse = unique_coords(cand.reshape(-1, 4))
    return c_out, inverse.reshape(len(c_in), K ** 3), ts_out
