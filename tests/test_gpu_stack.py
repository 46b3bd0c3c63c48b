"""The layers between the convolutions, and the ResNet-style stack of BASELINE config 3, on the GPU.

Per-op parity: batch norm (+ReLU), per-cloud average pooling, linear and softmax cross-entropy, forward and
backward, against oracle/glue.py (float64 numpy) on generator inputs.

Stack: 8 sparse convs 3x3x3 (32-32, 32-64, 64-64, 64-128 stride 2, 128-128, 128-256 stride 2, 256-256,
256-256), BN+ReLU after each, global average pool, linear 256-40, cross-entropy over random labels, forward
and backward.  Checked layer by layer with teacher forcing: every GPU op gets the ORACLE's previous result
(rounded to the storage type) as its input, so each comparison is one op at the stack's real shapes and no
rounding difference is carried from layer to layer.  One free-running GPU pass is compared loosely at the end.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import glue
from paper_2012_13846_amd import spgen
from util import TOL_BF16, TOL_F32, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    from paper_2012_13846_amd import binding
    binding.lib()
    return binding


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(dtype) if dtype is not None else t


def host(t):
    return t.float().cpu().numpy()


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("n,c,nb", [(3000, 32, 3), (70001, 64, 8), (5000, 256, 4), (777, 48, 2), (1, 16, 1)])
def test_glue_ops_match_oracle(sp, n, c, nb, bf16):
    rng = np.random.default_rng(n + c)
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else 2e-5
    rnd = spgen.round_to_bf16 if bf16 else (lambda a: a)
    x = rnd((rng.standard_normal((n, c)) * 1.5 + 0.3).astype(np.float32))
    dy = rnd(rng.standard_normal((n, c)).astype(np.float32))
    gamma = (1 + 0.2 * rng.standard_normal(c)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(c)).astype(np.float32)
    coords = np.zeros((n, 4), np.int32)
    coords[:, 0] = np.sort(rng.integers(0, nb, n))
    if n > 10:
        coords[:5, 0] = nb - 1          # clouds need not be contiguous
    for relu in (True, False):
        y, mean, rstd = sp.sp_bn_relu_fwd(dev(x, tdt), dev(gamma), dev(beta), 1e-5, relu)
        Y, M, R = glue.bn_relu_fwd(x, gamma, beta, 1e-5, relu)
        assert rel_err(host(y), Y) <= tol
        assert rel_err(host(mean), M) <= 2e-5 and rel_err(host(rstd), R) <= 2e-5
        # backward from the oracle's forward results (rounded to storage)
        Ys = rnd(Y.astype(np.float32))
        dx, dgamma, dbeta = sp.sp_bn_relu_bwd(dev(x, tdt), dev(Ys, tdt), dev(dy, tdt), dev(gamma),
                                              dev(M.astype(np.float32)), dev(R.astype(np.float32)), relu)
        DX, DG, DB = glue.bn_relu_bwd(x, Ys, dy, gamma, M.astype(np.float32), R.astype(np.float32), relu)
        assert rel_err(host(dx), DX) <= tol
        assert rel_err(host(dgamma), DG) <= 1e-4 and rel_err(host(dbeta), DB) <= 1e-4
    pooled, counts = sp.sp_pool_avg_fwd(dev(coords), dev(x, tdt), nb)
    P, Cn = glue.pool_avg_fwd(coords[:, 0], x, nb)
    assert np.array_equal(host(counts), Cn) and rel_err(host(pooled), P) <= 2e-5
    dout = rng.standard_normal((nb, c)).astype(np.float32)
    dxp = sp.sp_pool_avg_bwd(dev(coords), dev(dout), dev(Cn.astype(np.float32)), n, tdt)
    assert rel_err(host(dxp), glue.pool_avg_bwd(coords[:, 0], dout, Cn)) <= tol
    m = 40
    w = (rng.standard_normal((m, c)) / np.sqrt(c)).astype(np.float32)
    bias = rng.standard_normal(m).astype(np.float32)
    labels = rng.integers(0, m, nb).astype(np.int32)
    Pf = P.astype(np.float32)
    logits = sp.sp_linear_fwd(dev(Pf), dev(w), dev(bias))
    L = glue.linear_fwd(Pf, w, bias)
    assert rel_err(host(logits), L) <= 2e-5
    Lf = L.astype(np.float32)
    loss, dlog = sp.sp_softmax_ce(dev(Lf), dev(labels))
    LOSS, DLOG = glue.softmax_ce(Lf, labels)
    assert abs(float(loss.item()) - LOSS) <= 2e-5 * max(1.0, abs(LOSS)) and rel_err(host(dlog), DLOG) <= 2e-5
    Df = DLOG.astype(np.float32)
    dxl, dwl, dbl = sp.sp_linear_bwd(dev(Pf), dev(w), dev(Df))
    DXL, DWL, DBL = glue.linear_bwd(Pf, w, Df)
    assert rel_err(host(dxl), DXL) <= 2e-5 and rel_err(host(dwl), DWL) <= 2e-5 and rel_err(host(dbl), DBL) <= 2e-5


CHANNELS = [32, 32, 64, 64, 128, 128, 256, 256, 256]   # c0 .. c8
STRIDES = [1, 1, 1, 2, 1, 2, 1, 1]                      # convs 4 and 6 downsample


@pytest.mark.parametrize("bf16", [True, False], ids=["bf16", "f32"])
def test_resnet_style_stack_teacher_forced(sp, bf16):
    scale = 0.04
    raw = spgen.coords_config(3, scale)
    nb = int(raw[:, 0].max()) + 1
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else 2e-5              # layers between the convolutions
    tol_conv = TOL_BF16 if bf16 else TOL_F32      # the convolution and its two gradients: the parity bar itself
    rnd = spgen.round_to_bf16 if bf16 else (lambda a: np.asarray(a, np.float32))
    seed = spgen.seed_for(3, 0, stream=5)

    # ---- coordinate hierarchy and maps, both sides
    c0_h = sp.sp_coords_build(dev(raw), 1)
    c_or, _ = oracle.unique_coords(raw)
    assert np.array_equal(host(c0_h.coords()).astype(np.int32), c_or)
    levels_or, levels_h = [(c_or, 1)], [c0_h]
    maps_or, maps_h = [], []
    for s in STRIDES:
        cin, ts = levels_or[-1]
        cout, _, ts_out = oracle.strided_coords(cin, ts, s)
        maps_or.append(oracle.kernel_map(cin, cout, 3, ts) + (len(cin), len(cout)))
        km, ch = sp.sp_kmap_build(levels_h[-1], 3, s, 1)
        assert np.array_equal(km.counts, maps_or[-1][2]) and ch.n == len(cout)
        maps_h.append(km)
        levels_or.append((cout, ts_out))
        levels_h.append(ch)

    # ---- forward, teacher forced
    x_or = rnd(spgen.features(seed, len(c_or), CHANNELS[0]))
    acts = []          # per layer: (x_in, W, conv_out, gamma, beta, y, mean, rstd)
    worst = 0.0         # layers between the convolutions
    conv_errs = {}      # sp_conv_fwd / _bwd_data / _bwd_weight, per layer
    for l in range(8):
        pin, pout, counts, n_in, n_out = maps_or[l]
        W = rnd(spgen.weights(seed + 10 + l, 27, CHANNELS[l], CHANNELS[l + 1]))
        Z = oracle.conv_fwd(pin, pout, counts, x_or, W, n_out)
        z = sp.sp_conv_fwd(maps_h[l], dev(x_or, tdt), dev(W, tdt))
        conv_errs[f"fwd{l}"] = rel_err(host(z), Z)
        z_or = rnd(Z.astype(np.float32))
        rng = np.random.default_rng(seed + 100 + l)
        gamma = (1 + 0.1 * rng.standard_normal(CHANNELS[l + 1])).astype(np.float32)
        beta = (0.1 * rng.standard_normal(CHANNELS[l + 1])).astype(np.float32)
        Y, M, R = glue.bn_relu_fwd(z_or, gamma, beta, 1e-5, True)
        y, mean, rstd = sp.sp_bn_relu_fwd(dev(z_or, tdt), dev(gamma), dev(beta), 1e-5, True)
        worst = max(worst, rel_err(host(y), Y))
        y_or = rnd(Y.astype(np.float32))
        acts.append((x_or, W, z_or, gamma, beta, y_or, M.astype(np.float32), R.astype(np.float32)))
        x_or = y_or
    c_last = levels_or[-1][0]
    P, Cn = glue.pool_avg_fwd(c_last[:, 0], x_or, nb)
    pooled, counts_d = sp.sp_pool_avg_fwd(levels_h[-1].coords(), dev(x_or, tdt), nb)
    worst = max(worst, rel_err(host(pooled), P))
    rng = np.random.default_rng(seed + 999)
    w_fc = (rng.standard_normal((40, 256)) / 16).astype(np.float32)
    b_fc = np.zeros(40, np.float32)
    labels = rng.integers(0, 40, nb).astype(np.int32)
    Pf = P.astype(np.float32)
    L = glue.linear_fwd(Pf, w_fc, b_fc)
    worst = max(worst, rel_err(host(sp.sp_linear_fwd(dev(Pf), dev(w_fc), dev(b_fc))), L))
    Lf = L.astype(np.float32)
    LOSS, DLOG = glue.softmax_ce(Lf, labels)
    loss, dlog = sp.sp_softmax_ce(dev(Lf), dev(labels))
    assert abs(float(loss.item()) - LOSS) <= 1e-4
    worst = max(worst, rel_err(host(dlog), DLOG))

    # ---- backward, teacher forced
    Df = DLOG.astype(np.float32)
    DP, DWFC, DBFC = glue.linear_bwd(Pf, w_fc, Df)
    dp, dwfc, dbfc = sp.sp_linear_bwd(dev(Pf), dev(w_fc), dev(Df))
    worst = max(worst, rel_err(host(dp), DP), rel_err(host(dwfc), DWFC))
    DPf = DP.astype(np.float32)
    G = glue.pool_avg_bwd(c_last[:, 0], DPf, Cn)
    g = sp.sp_pool_avg_bwd(levels_h[-1].coords(), dev(DPf), dev(Cn.astype(np.float32)), len(c_last), tdt)
    worst = max(worst, rel_err(host(g), G))
    g_or = rnd(G.astype(np.float32))
    # upstream gradients are tiny (1/N from the pooling); the error metric is relative to their own rms
    for l in reversed(range(8)):
        x_in, W, z_or, gamma, beta, y_or, M, R = acts[l]
        pin, pout, counts, n_in, n_out = maps_or[l]
        DZ, DG, DB = glue.bn_relu_bwd(z_or, y_or, g_or, gamma, M, R, True)
        dz, dg, db = sp.sp_bn_relu_bwd(dev(z_or, tdt), dev(y_or, tdt), dev(g_or, tdt), dev(gamma), dev(M), dev(R), True)
        worst = max(worst, rel_err(host(dz), DZ))
        assert rel_err(host(dg), DG) <= 1e-3 and rel_err(host(db), DB) <= 1e-3
        dz_or = rnd(DZ.astype(np.float32))
        DX = oracle.conv_bwd_data(pin, pout, counts, dz_or, W, n_in)
        DW = oracle.conv_bwd_weight(pin, pout, counts, x_in, dz_or)
        dx = sp.sp_conv_bwd_data(maps_h[l], dev(dz_or, tdt), dev(W, tdt))
        dw = sp.sp_conv_bwd_weight(maps_h[l], dev(x_in, tdt), dev(dz_or, tdt))
        conv_errs[f"dgrad{l}"] = rel_err(host(dx), DX)
        conv_errs[f"wgrad{l}"] = rel_err(host(dw), DW)
        g_or = rnd(DX.astype(np.float32))
    worst_conv = max(conv_errs.values())
    print("conv errors, largest first:", sorted(((round(v, 9), k) for k, v in conv_errs.items()), reverse=True)[:8])
    print(f"stack ({'bf16' if bf16 else 'f32'}): N per level {[len(c) for c, _ in levels_or]}, worst rel err: "
          f"convolutions {worst_conv:.2e} (tol {tol_conv:g}), other layers {worst:.2e} (tol {tol:g})")
    assert worst_conv <= tol_conv
    assert worst <= tol


def test_stack_free_running_loss_close_to_oracle(sp):
    """Whole forward pass on the GPU without teacher forcing (bf16 storage): the loss stays near the oracle's."""
    raw = spgen.coords_config(3, 0.02)
    nb = int(raw[:, 0].max()) + 1
    seed = spgen.seed_for(3, 0, stream=6)
    c_or, _ = oracle.unique_coords(raw)
    ch = sp.sp_coords_build(dev(raw), 1)
    x_or = spgen.features(seed, len(c_or), 32, True).astype(np.float64)
    x = dev(x_or.astype(np.float32), torch.bfloat16)
    cur_or, ts = c_or, 1
    for l, s in enumerate(STRIDES):
        cout, _, ts_out = oracle.strided_coords(cur_or, ts, s)
        pin, pout, counts = oracle.kernel_map(cur_or, cout, 3, ts)
        W = spgen.weights(seed + 10 + l, 27, CHANNELS[l], CHANNELS[l + 1], True)
        gamma, beta = np.ones(CHANNELS[l + 1], np.float32), np.zeros(CHANNELS[l + 1], np.float32)
        x_or = glue.bn_relu_fwd(oracle.conv_fwd(pin, pout, counts, x_or.astype(np.float32), W, len(cout)), gamma, beta, 1e-5, True)[0]
        km, ch = sp.sp_kmap_build(ch, 3, s, 1)
        x = sp.sp_bn_relu_fwd(sp.sp_conv_fwd(km, x, dev(W, torch.bfloat16)), dev(gamma), dev(beta), 1e-5, True)[0]
        cur_or, ts = cout, ts_out
    rng = np.random.default_rng(seed)
    w_fc = (rng.standard_normal((40, 256)) / 16).astype(np.float32)
    labels = rng.integers(0, 40, nb).astype(np.int32)
    P, _ = glue.pool_avg_fwd(cur_or[:, 0], x_or, nb)
    LOSS, _ = glue.softmax_ce(glue.linear_fwd(P, w_fc, np.zeros(40)), labels)
    pooled, _ = sp.sp_pool_avg_fwd(ch.coords(), x, nb)
    loss, _ = sp.sp_softmax_ce(sp.sp_linear_fwd(pooled, dev(w_fc), dev(np.zeros(40, np.float32))), dev(labels))
    print("free-running loss", float(loss.item()), "oracle", LOSS)
    assert abs(float(loss.item()) - LOSS) <= 0.03 * abs(LOSS)
