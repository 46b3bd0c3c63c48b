"""Pooling over kernel maps and generative transposed convolution on the GPU against oracle/pool.py.

Integer results (created coordinates, candidate table, maps, arg-max records) bit-exact; max pooling is a
selection, so its values are bit-exact too; avg / sum within the parity tolerance."""
import numpy as np
import pytest
import torch

import oracle
from oracle import pool as opool
from paper_2012_13846_amd import spgen
from util import TOL_BF16, TOL_F32, oracle_steps, rel_err, sort_lists

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


POOL_CASES = [
    # name, cfg, scale, K, stride, channels, bf16, transposed
    ("cfg1_k2s2_c32_f32", 1, 1.0, 2, 2, 32, False, False),
    ("cfg1_k3s2_c64_f32", 1, 0.5, 3, 2, 64, False, False),
    ("cfg1_k3s1_c32_f32", 1, 0.5, 3, 1, 32, False, False),      # one table serves both directions (reversed side)
    ("cfg3_k2s2_c64_bf16", 3, 0.1, 2, 2, 64, True, False),
    ("cfg3_k3s2_c128_bf16", 3, 0.05, 3, 2, 128, True, False),
    ("cfg0_k3s1_c5_f32_scalar", 0, 1.0, 3, 1, 5, False, False),  # channel count without 16-byte pieces
    ("cfg0_k2s2_c3_bf16_scalar", 0, 1.0, 2, 2, 3, True, False),
    ("cfg1_k2s2_up_c32_f32", 1, 0.5, 2, 2, 32, False, True),     # "unpooling": the transposed map
    ("cfg0_k5s1_c16_f32", 0, 1.0, 5, 1, 16, False, False),
]


@pytest.mark.parametrize("case", POOL_CASES, ids=[c[0] for c in POOL_CASES])
def test_pool_matches_oracle(sp, case):
    name, cfg, scale, K, stride, ch, bf16, transposed = case
    raw = spgen.coords_config(cfg, scale)
    want = oracle_steps(raw, K, stride, 1, 1)
    pin, pout, counts = want["pair_in"], want["pair_out"], want["counts"]
    n_in, n_out = len(want["c_in"]), len(want["c_out"])
    c = sp.sp_coords_build(dev(raw), 1)
    km, _ = sp.sp_kmap_build(c, K, stride, 1)
    if transposed:
        pin, pout, counts = oracle.transpose_map(pin, pout, counts)
        n_in, n_out = n_out, n_in
        km = sp.sp_kmap_transpose(km)
    rng = np.random.default_rng(500 + len(name))
    X = spgen.features(600 + len(name), n_in, ch, bf16)
    X[rng.random(X.shape) < 0.3] = 0.5          # ties inside windows: the lowest-offset rule is exercised
    dY = spgen.features(700 + len(name), n_out, ch, bf16)
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL_F32
    x, dy = dev(X, tdt), dev(dY, tdt)
    for mode in ("max", "avg", "sum"):
        Y, ARG = opool.pool_fwd(pin, pout, counts, X, n_out, mode)
        y, arg = sp.sp_pool_fwd(km, x, mode)
        if mode == "max":
            assert np.array_equal(host(y), Y.astype(np.float32))
            assert np.array_equal(arg.cpu().numpy().astype(np.int8), ARG.astype(np.int8))     # 255 = -1 = no link
        else:
            assert arg is None and rel_err(host(y), Y) <= tol
        DX = opool.pool_bwd(pin, pout, counts, dY, ARG, n_in, mode)
        dx = sp.sp_pool_bwd(km, dy, arg, mode)
        e = rel_err(host(dx), DX)
        assert e <= tol, (mode, e)
    # outputs without any link (possible for the transposed map's rows only if the map is empty there) are zero
    dead = np.setdiff1d(np.arange(n_out), pout)
    if len(dead):
        y, arg = sp.sp_pool_fwd(km, x, "max")
        assert torch.count_nonzero(y[torch.from_numpy(dead).cuda()]).item() == 0


def test_pool_empty_and_bad_arguments(sp):
    c = sp.sp_coords_build(torch.empty((0, 4), dtype=torch.int32, device="cuda"), 1)
    km, _ = sp.sp_kmap_build(c, 2, 2, 1)
    y, arg = sp.sp_pool_fwd(km, torch.empty((0, 8), device="cuda"), "max")
    assert y.shape == (0, 8)
    assert sp.sp_pool_bwd(km, torch.empty((0, 8), device="cuda"), arg, "max").shape == (0, 8)
    c = sp.sp_coords_build(dev(spgen.coords_config(0)), 1)
    km, _ = sp.sp_kmap_build(c, 2, 2, 1)
    with pytest.raises(sp.SpError) as e:
        sp.sp_pool_bwd(km, torch.zeros((km.n_out, 8), device="cuda"), None, "max")
    assert e.value.code == -1


GEN_CASES = [
    # name, raw coarse cells, coarse tensor stride, K, stride
    ("cfg0_cells_k2s2", 0, 1.0, 2, 2, 2),
    ("cfg0_cells_k3s2", 0, 1.0, 2, 3, 2),
    ("cfg1_cells_k2s2_ts4", 1, 0.3, 4, 2, 2),
    ("cfg1_cells_k3s2_ts2", 1, 0.3, 2, 3, 2),
    ("cfg0_k3s1_dilate", 0, 1.0, 1, 3, 1),
    ("cfg0_cells_k4s4", 0, 0.3, 4, 4, 4),
]


@pytest.mark.parametrize("case", GEN_CASES, ids=[c[0] for c in GEN_CASES])
def test_generative_map_matches_oracle(sp, case):
    name, cfg, scale, ts_in, K, stride = case
    kvol = K ** 3
    cells = spgen.coords_config(cfg, scale)
    cells[:, 1:] -= 7                                            # negative coordinates too
    raw = cells * np.array([1, ts_in, ts_in, ts_in], np.int32)
    c_in, _ = oracle.unique_coords(raw)
    c_out, where, ts_out = opool.generative_coords(c_in, ts_in, K, stride)
    fwd = oracle.kernel_map(c_out, c_in, K, ts_out)              # stride-s convolution fine -> coarse ...
    tin, tout, tcounts = oracle.transpose_map(*fwd)              # ... with the roles swapped

    ch = sp.sp_coords_build(dev(raw), ts_in)
    km, fine = sp.sp_kmap_build_generative(ch, K, stride)
    assert fine.n == len(c_out) and fine.tensor_stride == ts_out
    assert np.array_equal(fine.coords().cpu().numpy(), c_out)
    assert np.array_equal(fine.inverse().cpu().numpy(), where.reshape(-1))
    assert (km.n_in, km.n_out, km.kvol) == (len(c_in), len(c_out), kvol)
    assert np.array_equal(km.counts, tcounts) and (km.counts == len(c_in)).all()
    gin, gout = km.pairs()
    gin, gout = sort_lists(gin.cpu().numpy(), gout.cpu().numpy(), km.counts)
    assert np.array_equal(gin, tin) and np.array_equal(gout, tout)
    nbr_out, nbr_in, rev_out, rev_in = km.table()
    assert not rev_out and not rev_in
    kidx = np.repeat(np.arange(kvol), tcounts)
    w_out = np.full((kvol, len(c_out)), -1, np.int32)
    w_out[kidx, tout] = tin
    w_in = np.full((kvol, len(c_in)), -1, np.int32)
    w_in[kidx, tin] = tout
    assert np.array_equal(nbr_out.cpu().numpy(), w_out) and np.array_equal(nbr_in.cpu().numpy(), w_in)
    # the way back: the stride-s convolution from the created rows to the given rows
    kb = sp.sp_kmap_transpose(km)
    bin_, bout = kb.pairs()
    bin_, bout = sort_lists(bin_.cpu().numpy(), bout.cpu().numpy(), kb.counts)
    assert np.array_equal(bin_, fwd[0]) and np.array_equal(bout, fwd[1]) and np.array_equal(kb.counts, fwd[2])

    # the transposed convolution itself and its gradients, both precisions
    for bf16, cin_ch, cout_ch in ((False, 32, 16), (True, 128, 64)):
        if bf16 and len(c_in) * kvol > 400000:
            continue
        seed = 900 + len(name)
        X = spgen.features(seed, len(c_in), cin_ch, bf16)
        dY = spgen.features(seed + 1, len(c_out), cout_ch, bf16)
        W = spgen.weights(seed + 2, kvol, cin_ch, cout_ch, bf16)
        tdt = torch.bfloat16 if bf16 else torch.float32
        tol = TOL_BF16 if bf16 else TOL_F32
        y = sp.sp_conv_fwd(km, dev(X, tdt), dev(W, tdt))
        dx = sp.sp_conv_bwd_data(km, dev(dY, tdt), dev(W, tdt))
        dw = sp.sp_conv_bwd_weight(km, dev(X, tdt), dev(dY, tdt))
        assert rel_err(host(y), oracle.conv_fwd(tin, tout, tcounts, X, W, len(c_out))) <= tol
        assert rel_err(host(dx), oracle.conv_bwd_data(tin, tout, tcounts, dY, W, len(c_in))) <= tol
        assert rel_err(host(dw), oracle.conv_bwd_weight(tin, tout, tcounts, X, dY)) <= tol


def test_generative_bad_arguments_and_empty(sp):
    c = sp.sp_coords_build(dev(spgen.coords_config(0)), 1)
    with pytest.raises(sp.SpError) as e:
        sp.sp_kmap_build_generative(c, 2, 2)          # tensor stride 1 is not a multiple of 2
    assert e.value.code == -1
    with pytest.raises(sp.SpError):
        sp.sp_kmap_build_generative(c, 6, 1)
    c0 = sp.sp_coords_build(torch.empty((0, 4), dtype=torch.int32, device="cuda"), 2)
    km, fine = sp.sp_kmap_build_generative(c0, 2, 2)
    assert km.total == 0 and fine.n == 0 and fine.tensor_stride == 1


def test_generative_rows_beyond_the_packable_range_are_an_error(sp):
    """A created row is a coordinate like any other: one past the range is reported, not wrapped."""
    c = sp.sp_coords_build(dev(np.array([[0, 32767, 0, 0], [0, 5, 5, 5]], np.int32)), 1)
    with pytest.raises(sp.SpError) as e:
        sp.sp_kmap_build_generative(c, 3, 1)          # 32767 + 1 has no key
    assert e.value.code == -2
    c = sp.sp_coords_build(dev(np.array([[0, -32768, 0, 0]], np.int32)), 2)
    with pytest.raises(sp.SpError) as e:
        sp.sp_kmap_build_generative(c, 3, 2)          # -32768 - 1
    assert e.value.code == -2
    km, fine = sp.sp_kmap_build_generative(c, 2, 2)   # even kernel: offsets 0 and +1 only, all rows fit
    assert fine.n == 8 and km.total == 8
