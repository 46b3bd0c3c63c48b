"""Parity at the full sizes of the BASELINE workloads, in the launch configuration bench.py times.

  - coordinates (every level of the hierarchy): compared in full with the oracle's sort-based merge;
  - kernel maps: compared IN FULL with the oracle's map, as per-offset (in, out)-sorted pair lists, pair
    counts and both neighbour tables, bit-exactly (the oracle's sort + binary search takes a few seconds per
    million voxels), plus properties that hold at any size (stride-1 count symmetry, k2s2 covers every
    input once);
  - forward / data gradient: the oracle cannot evaluate every row at these channel counts in seconds, so
    sampled rows are compared against the oracle evaluated on exactly those rows' links;
  - weight gradient: two whole offsets (the first and the centre/last) against the oracle.

`level` > 0 cases first apply that many 3x3x3 stride-2 downsamplings (the config-3 stack's hierarchy) and test
the map and the layer on the coarser level, at the row counts and tensor stride the stack really has there.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_13846_amd import spgen
from util import TOL_BF16, TOL_F32, rel_err, sort_lists

pytestmark = pytest.mark.gpu

N_SAMPLE = 4096


@pytest.fixture(scope="module")
def sp():
    from paper_2012_13846_amd import binding
    binding.lib()
    return binding


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(dtype) if dtype is not None else t


CASES = [
    # name, cfg, level, K, stride, dilation, cin, cout, bf16, transposed, rows sampled for fwd / dgrad
    ("cfg1_k3_f32_32x64", 1, 0, 3, 1, 1, 32, 64, False, False, N_SAMPLE),
    ("cfg2_k2s2_down_bf16_64x128", 2, 0, 2, 2, 1, 64, 128, True, False, N_SAMPLE),
    ("cfg2_k2s2_up_bf16_128x64", 2, 0, 2, 2, 1, 128, 64, True, True, N_SAMPLE),
    ("cfg3_k3_bf16_64x64", 3, 0, 3, 1, 1, 64, 64, True, False, N_SAMPLE),
    ("cfg3_k3s2_bf16_64x128", 3, 0, 3, 2, 1, 64, 128, True, False, N_SAMPLE),
    ("cfg4_k3_bf16_64x64", 4, 0, 3, 1, 1, 64, 64, True, False, N_SAMPLE),
    ("cfg4_k3d2_bf16_64x64", 4, 0, 3, 1, 2, 64, 64, True, False, N_SAMPLE),
    # wide layers of the config-3 stack at full row count: the row-stationary kernel (stride 1), and the
    # position-class order with offset masks (stride 2: data gradient, and forward of the transposed map)
    ("cfg3_k3_bf16_128x128", 3, 0, 3, 1, 1, 128, 128, True, False, N_SAMPLE),
    ("cfg3_k3s2_bf16_128x256", 3, 0, 3, 2, 1, 128, 256, True, False, N_SAMPLE),
    ("cfg3_k3s2_up_bf16_256x128", 3, 0, 3, 2, 1, 256, 128, True, True, N_SAMPLE),
    # the stack's coarser levels at their real shapes: level 1 (tensor stride 2, ~181 k rows) 128 -> 128 and its
    # stride-2 layer, level 2 (tensor stride 4, ~55 k rows, half of all row-offsets linked) 256 -> 256: the
    # 8-wavefront row-stationary kernel and the 256 x 256 weight-gradient tile
    ("cfg3_l1_k3_bf16_128x128", 3, 1, 3, 1, 1, 128, 128, True, False, 2048),
    ("cfg3_l1_k3s2_bf16_128x256", 3, 1, 3, 2, 1, 128, 256, True, False, 2048),
    ("cfg3_l2_k3_bf16_256x256", 3, 2, 3, 1, 1, 256, 256, True, False, 1024),
    # the sparsity sweep's batches as bench.py times them (fp32, 64 -> 64): the largest batch of each grid
    ("sweep32_p0.25_b512_f32_64x64", ("sweep", 32, 0.25, 512), 0, 3, 1, 1, 64, 64, False, False, N_SAMPLE),
    ("sweep50_p0.25_b256_f32_64x64", ("sweep", 50, 0.25, 256), 0, 3, 1, 1, 64, 64, False, False, N_SAMPLE),
    # the two literal readings bench.py also times: 2048 points per cloud, and the room at 5 cm voxels
    ("cfg2lit_2048pt_k2s2_bf16_64x128", ("literal", "cfg2_2048pt"), 0, 2, 2, 1, 64, 128, True, False, N_SAMPLE),
    ("cfg4lit_5cm_k3_bf16_64x64", ("literal", "cfg4_5cm"), 0, 3, 1, 1, 64, 64, True, False, N_SAMPLE),
]


def links_of_rows(pair_in, pair_out, counts, rows, side):
    """The links whose `side` row ("in" or "out") is in `rows`, that row renumbered to its position in `rows`.
    Returns (pair_in, pair_out, counts) in the oracle's list form."""
    key = pair_out if side == "out" else pair_in
    pos = np.full(int(key.max()) + 1 if len(key) else 1, -1, np.int64)
    pos[rows] = np.arange(len(rows))
    keep = pos[key] >= 0
    kidx = np.repeat(np.arange(len(counts)), counts)[keep]
    cnt = np.bincount(kidx, minlength=len(counts)).astype(np.int64)
    pi, po = pair_in[keep].copy(), pair_out[keep].copy()
    if side == "out":
        po = pos[po].astype(np.int32)
    else:
        pi = pos[pi].astype(np.int32)
    return pi, po, cnt


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_full_size(sp, case):
    name, cfg, level, K, stride, dil, cin, cout, bf16, transposed, n_sample = case
    kvol = K ** 3
    if isinstance(cfg, tuple):   # ("sweep", grid, p, clouds) or ("literal", name)
        raw = spgen.coords_sweep(cfg[1], cfg[2], cfg[3]) if cfg[0] == "sweep" else spgen.coords_literal(cfg[1])
        cfg = 5
    else:
        raw = spgen.coords_config(cfg)
    rng = np.random.default_rng(spgen.seed_for(cfg, 0, stream=7))

    # ---- coordinates of every level, in full
    c_in, inverse = oracle.unique_coords(raw)
    co_h = sp.sp_coords_build(dev(raw), 1)
    assert co_h.n == len(c_in)
    assert np.array_equal(co_h.coords().cpu().numpy(), c_in)
    assert np.array_equal(co_h.inverse().cpu().numpy(), inverse)
    ts = 1
    keep_alive = []
    for _ in range(level):
        c_in, parent, ts_next = oracle.strided_coords(c_in, ts, 2)
        km_l, co_next = sp.sp_kmap_build(co_h, 3, 2, 1)
        assert co_next.n == len(c_in) and co_next.tensor_stride == ts_next
        assert np.array_equal(co_next.coords().cpu().numpy(), c_in)
        assert np.array_equal(co_next.inverse().cpu().numpy(), parent)
        keep_alive += [km_l, co_h]
        co_h, ts = co_next, ts_next
    c_out, parent, ts_out = oracle.strided_coords(c_in, ts, stride)
    km, cout_h = sp.sp_kmap_build(co_h, K, stride, dil)
    assert cout_h.n == len(c_out) and cout_h.tensor_stride == ts_out
    assert np.array_equal(cout_h.coords().cpu().numpy(), c_out)
    if stride > 1:
        assert np.array_equal(cout_h.inverse().cpu().numpy(), parent)
    n_in, n_out = len(c_in), len(c_out)

    # ---- kernel map, in full: counts, (in, out)-sorted pair lists, both neighbour tables
    pin, pout, counts = oracle.kernel_map(c_in, c_out, K, dil * ts)
    assert (km.n_in, km.n_out) == (n_in, n_out)
    assert np.array_equal(km.counts, counts) and km.total == int(counts.sum())
    gin, gout = km.pairs()
    gin, gout = sort_lists(gin.cpu().numpy(), gout.cpu().numpy(), km.counts)
    assert np.array_equal(gin, pin)
    assert np.array_equal(gout, pout)
    del gin, gout
    nbr_out, nbr_in, rev_out, rev_in = km.table()
    assert not rev_out
    kidx = np.repeat(np.arange(kvol), counts)
    want = np.full((kvol, n_out), -1, np.int32)
    want[kidx, pout] = pin
    assert np.array_equal(nbr_out.cpu().numpy(), want)
    want = np.full((kvol, n_in), -1, np.int32)
    want[kidx, pin] = pout
    got_in = nbr_in.cpu().numpy()
    assert np.array_equal(got_in[::-1] if rev_in else got_in, want)
    del want, got_in
    if stride == 1 and K % 2 == 1:
        assert np.array_equal(km.counts, km.counts[::-1]) and km.counts[kvol // 2] == n_in
    if K == 2 and stride == 2:
        assert km.total == n_in

    # ---- features
    if transposed:   # transposed conv: sources are the coarse rows (c_out), destinations the fine rows (c_in)
        pin, pout, counts = oracle.transpose_map(pin, pout, counts)
        n_src, n_dst = n_out, n_in
        use = sp.sp_kmap_transpose(km)
    else:
        n_src, n_dst = n_in, n_out
        use = km
    s_dst = np.sort(rng.choice(n_dst, min(n_sample, n_dst), replace=False))
    s_src = np.sort(rng.choice(n_src, min(n_sample, n_src), replace=False))
    seed = spgen.seed_for(cfg, 0, stream=3)
    X = spgen.features(seed, n_src, cin, bf16)
    dY = spgen.features(seed + 1, n_dst, cout, bf16)
    W = spgen.weights(seed + 2, kvol, cin, cout, bf16)
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL_F32
    x, dy, w = dev(X, tdt), dev(dY, tdt), dev(W, tdt)
    y = sp.sp_conv_fwd(use, x, w)
    dx = sp.sp_conv_bwd_data(use, dy, w)
    dw = sp.sp_conv_bwd_weight(use, x, dy)
    torch.cuda.synchronize()

    # forward on the sampled destination rows, data gradient on the sampled source rows
    f_in, f_out, f_cnt = links_of_rows(pin, pout, counts, s_dst, "out")
    Y = oracle.conv_fwd(f_in, f_out, f_cnt, X, W, len(s_dst))
    e_y = rel_err(y[torch.from_numpy(s_dst).cuda()].float().cpu().numpy(), Y)
    b_in, b_out, b_cnt = links_of_rows(pin, pout, counts, s_src, "in")
    dX = oracle.conv_bwd_data(b_in, b_out, b_cnt, dY, W, len(s_src))
    e_dx = rel_err(dx[torch.from_numpy(s_src).cuda()].float().cpu().numpy(), dX)
    # weight gradient, two whole offsets
    e_dw = 0.0
    koff = np.concatenate([[0], np.cumsum(counts)])
    for k in sorted({0, kvol // 2 if K % 2 else kvol - 1}):
        sl = slice(int(koff[k]), int(koff[k + 1]))
        dWk = oracle.conv_bwd_weight(pin[sl], pout[sl], counts[k:k + 1], X, dY)[0]
        e_dw = max(e_dw, rel_err(dw[k].cpu().numpy(), dWk))
    print(f"{name}: n_in {n_in} n_out {n_out} pairs {km.total}; rel err fwd {e_y:.2e} dgrad {e_dx:.2e} "
          f"wgrad {e_dw:.2e} (tol {tol:g})")
    assert e_y <= tol and e_dx <= tol and e_dw <= tol
