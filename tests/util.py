"""Helpers shared by the parity tests: run the oracle's steps, sort pair lists, error metric."""
from __future__ import annotations

import numpy as np

import oracle

# tolerances of the parity bar: max relative error, fp32 path / bf16-in fp32-accumulate path
TOL_F32 = 1e-5
TOL_BF16 = 2e-2


def rel_err(got, ref) -> float:
    """max_j |g_j - r_j| / max(|r_j|, rms(r)).

    Plain elementwise relative error is undefined where a sum cancels to ~0, so the denominator
    is floored at the reference tensor's root-mean-square value.
    """
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    if r.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(r * r)))
    den = np.maximum(np.abs(r), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(g - r) / den))


def rel_err_large(got, ref) -> float:
    """Plain elementwise relative error max_j |g_j - r_j| / |r_j| over the elements with |r_j| >= rms(r): the
    part of rel_err's maximum that no floor of the denominator touches (reported next to rel_err)."""
    g = np.asarray(got, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    if r.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(r * r)))
    big = np.abs(r) >= rms
    if rms == 0 or not big.any():
        return 0.0
    return float(np.max(np.abs(g[big] - r[big]) / np.abs(r[big])))


def oracle_steps(raw, kernel_size, stride=1, dilation=1, tensor_stride=1):
    """Steps 0-2 on the CPU oracle.  Returns dict with coords, inverse, c_out, parent, ts_out, pairs."""
    c_in, inverse = oracle.unique_coords(raw)
    c_out, parent, ts_out = oracle.strided_coords(c_in, tensor_stride, stride)
    pin, pout, counts = oracle.kernel_map(c_in, c_out, kernel_size, dilation * tensor_stride)
    return dict(c_in=c_in, inverse=inverse, c_out=c_out, parent=parent, ts_out=ts_out,
                pair_in=pin, pair_out=pout, counts=counts)


def sort_lists(pair_in, pair_out, counts):
    """Each offset's list sorted by (in, out): the unique form two correct pair lists share."""
    pair_in = np.asarray(pair_in).copy()
    pair_out = np.asarray(pair_out).copy()
    base = 0
    for c in counts:
        c = int(c)
        order = np.lexsort((pair_out[base:base + c], pair_in[base:base + c]))
        pair_in[base:base + c] = pair_in[base:base + c][order]
        pair_out[base:base + c] = pair_out[base:base + c][order]
        base += c
    return pair_in, pair_out
