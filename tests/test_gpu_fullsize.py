"""Parity at the full sizes of the BASELINE workloads, in the launch configuration bench.py times.

The oracle cannot do these sizes element by element in seconds, so:
  - coordinates: compared in full (the oracle's sort-based merge is fast);
  - kernel maps: the neighbour tables of 4096 sampled output rows and 4096 sampled input rows are compared
    bit-exactly with the oracle's map of exactly those rows, plus properties that hold at any size
    (pair counts = live table entries, stride-1 count symmetry, k2s2 covers every input once);
  - forward / data gradient: sampled rows against the oracle evaluated on those rows' links;
  - weight gradient: two whole offsets (the first and the centre/last) against the oracle, whose links for
    one offset are a kernel-size-1 map against shifted coordinates.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_13846_amd import spgen
from util import TOL_BF16, TOL_F32, rel_err

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


def offset_of(k, K):
    c = (K - 1) // 2 if K % 2 else 0
    return np.array([k // (K * K) - c, (k // K) % K - c, k % K - c], np.int32)


CASES = [
    # name, cfg, K, stride, dilation, cin, cout, bf16, transposed
    ("cfg1_k3_f32_32x64", 1, 3, 1, 1, 32, 64, False, False),
    ("cfg2_k2s2_down_bf16_64x128", 2, 2, 2, 1, 64, 128, True, False),
    ("cfg2_k2s2_up_bf16_128x64", 2, 2, 2, 1, 128, 64, True, True),
    ("cfg3_k3_bf16_64x64", 3, 3, 1, 1, 64, 64, True, False),
    ("cfg3_k3s2_bf16_64x128", 3, 3, 2, 1, 64, 128, True, False),
    ("cfg4_k3_bf16_64x64", 4, 3, 1, 1, 64, 64, True, False),
    ("cfg4_k3d2_bf16_64x64", 4, 3, 1, 2, 64, 64, True, False),
    # wide layers of the config-3 stack at full row count: the row-stationary kernel (stride 1), and the
    # position-class order with offset masks (stride 2: data gradient, and forward of the transposed map)
    ("cfg3_k3_bf16_128x128", 3, 3, 1, 1, 128, 128, True, False),
    ("cfg3_k3s2_bf16_128x256", 3, 3, 2, 1, 128, 256, True, False),
    ("cfg3_k3s2_up_bf16_256x128", 3, 3, 2, 1, 256, 128, True, True),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_full_size(sp, case):
    name, cfg, K, stride, dil, cin, cout, bf16, transposed = case
    kvol = K ** 3
    rng = np.random.default_rng(spgen.seed_for(cfg, 0, stream=7))
    raw = spgen.coords_config(cfg)

    # ---- coordinates, in full
    c_in, inverse = oracle.unique_coords(raw)
    c_out, parent, ts_out = oracle.strided_coords(c_in, 1, stride)
    co_h = sp.sp_coords_build(dev(raw), 1)
    assert co_h.n == len(c_in)
    assert np.array_equal(co_h.coords().cpu().numpy(), c_in)
    assert np.array_equal(co_h.inverse().cpu().numpy(), inverse)
    km, cout_h = sp.sp_kmap_build(co_h, K, stride, dil)
    assert cout_h.n == len(c_out) and cout_h.tensor_stride == ts_out
    assert np.array_equal(cout_h.coords().cpu().numpy(), c_out)
    if stride > 1:
        assert np.array_equal(cout_h.inverse().cpu().numpy(), parent)
    n_in, n_out = len(c_in), len(c_out)

    # ---- kernel map: sampled rows of both tables, bit-exact
    nbr_out, nbr_in, rev_out, rev_in = km.table()
    assert not rev_out
    s_out = np.sort(rng.choice(n_out, min(N_SAMPLE, n_out), replace=False))
    s_in = np.sort(rng.choice(n_in, min(N_SAMPLE, n_in), replace=False))
    po_in, po_out, po_cnt = oracle.kernel_map(c_in, c_out[s_out], K, dil)        # links of the sampled outputs
    pi_in, pi_out, pi_cnt = oracle.kernel_map(c_in[s_in], c_out, K, dil)         # links of the sampled inputs
    got_out = nbr_out[:, torch.from_numpy(s_out).cuda()].cpu().numpy()
    got_in = nbr_in[:, torch.from_numpy(s_in).cuda()].cpu().numpy()
    if rev_in:
        got_in = got_in[::-1]
    want_out = np.full((kvol, len(s_out)), -1, np.int32)
    want_in = np.full((kvol, len(s_in)), -1, np.int32)
    want_out[np.repeat(np.arange(kvol), po_cnt), po_out] = po_in
    want_in[np.repeat(np.arange(kvol), pi_cnt), pi_in] = pi_out
    assert np.array_equal(got_out, want_out)
    assert np.array_equal(got_in, want_in)
    # properties at any size
    live = (nbr_out >= 0).sum(dim=1).cpu().numpy()
    assert np.array_equal(live, km.counts) and km.total == int(km.counts.sum())
    if stride == 1 and K % 2 == 1:
        assert np.array_equal(km.counts, km.counts[::-1]) and km.counts[kvol // 2] == n_in
    if K == 2 and stride == 2:
        assert km.total == n_in
    gin, gout = km.pairs()
    base = int(km.counts[:kvol - 1].sum())     # the last offset's list against the table
    last_in, last_out = gin[base:].cpu().numpy(), gout[base:].cpu().numpy()
    assert np.array_equal(nbr_out[kvol - 1].cpu().numpy()[last_out], last_in)

    # ---- features
    if transposed:
        kmt = sp.sp_kmap_transpose(km)
        # transposed conv: sources are the coarse rows (c_out), destinations the fine rows (c_in)
        n_src, n_dst = n_out, n_in
        s_dst, s_src = s_in, s_out
        f_in, f_out, f_cnt = pi_out, pi_in, pi_cnt          # links of sampled destinations (fine rows)
        b_in, b_out, b_cnt = po_out, po_in, po_cnt          # links of sampled sources (coarse rows)
        use = kmt
    else:
        n_src, n_dst = n_in, n_out
        s_dst, s_src = s_out, s_in
        f_in, f_out, f_cnt = po_in, po_out, po_cnt
        b_in, b_out, b_cnt = pi_in, pi_out, pi_cnt
        use = km
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

    # forward on the sampled destination rows (f_out indexes the sample)
    Y = oracle.conv_fwd(f_in, f_out, f_cnt, X, W, len(s_dst))
    e_y = rel_err(y[torch.from_numpy(s_dst).cuda()].float().cpu().numpy(), Y)
    # data gradient on the sampled source rows (b_in indexes the sample)
    dX = oracle.conv_bwd_data(b_in, b_out, b_cnt, dY, W, len(s_src))
    e_dx = rel_err(dx[torch.from_numpy(s_src).cuda()].float().cpu().numpy(), dX)
    # weight gradient, two whole offsets
    e_dw = 0.0
    c_src, c_dst = (c_out, c_in) if transposed else (c_in, c_out)
    for k in sorted({0, kvol // 2 if K % 2 else kvol - 1}):
        off = offset_of(k, K) * dil
        if transposed:      # source (coarse) + offset = destination (fine)  <=>  K=1 map of shifted sources
            shifted = c_src.copy()
            shifted[:, 1:] += off
            l_dst, l_src, cnt1 = oracle.kernel_map(c_dst, shifted, 1, 1)      # in = destination row, out = source row
            links_in, links_out = l_src, l_dst
        else:               # destination + offset = source
            shifted = c_dst.copy()
            shifted[:, 1:] += off
            links_in, links_out, cnt1 = oracle.kernel_map(c_src, shifted, 1, 1)
        assert int(cnt1[0]) == int(use.counts[k])
        dWk = oracle.conv_bwd_weight(links_in, links_out, cnt1, X, dY)[0]
        e_dw = max(e_dw, rel_err(dw[k].cpu().numpy(), dWk))
    print(f"{name}: n_in {n_in} n_out {n_out} pairs {km.total}; rel err fwd {e_y:.2e} dgrad {e_dx:.2e} "
          f"wgrad {e_dw:.2e} (tol {tol:g})")
    assert e_y <= tol and e_dx <= tol and e_dw <= tol
