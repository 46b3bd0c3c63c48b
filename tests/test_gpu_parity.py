"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Integer work (coordinates, inverse maps, pair lists, counts) must match bit-exactly; pair lists are
compared per offset after sorting by (in, out) because the order inside one list is free.  Features are
compared with util.rel_err against the fp64 oracle: <= 1e-5 for fp32, <= 2e-2 for bf16-in/fp32-accumulate.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_13846_amd import spgen
from util import TOL_BF16, TOL_F32, oracle_steps, rel_err, rel_err_large, sort_lists

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    from paper_2012_13846_amd import binding
    binding.lib()
    return binding


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(dtype) if dtype is not None else t


def random_coords(seed, n, grid, batches=2, lo=0):
    rng = np.random.default_rng(seed)
    c = np.empty((n, 4), np.int32)
    c[:, 0] = rng.integers(0, batches, n)
    c[:, 1:] = rng.integers(lo, lo + grid, (n, 3))
    return c


# ------------------------------------------------------------------ step 0: coordinates
@pytest.mark.parametrize("name,raw", [
    ("cfg0", spgen.coords_config(0)),
    ("cfg1", spgen.coords_config(1)),
    ("negatives", random_coords(3, 70000, 40, batches=3, lo=-20)),
    ("all_same", np.tile(np.array([[2, -5, 7, 9]], np.int32), (1000, 1))),
    ("single", np.array([[0, 1, 2, 3]], np.int32)),
    ("extremes", np.array([[65535, 32767, -32768, 0], [0, -32768, 32767, 5], [65535, 32767, -32768, 0]], np.int32)),
])
def test_coords_build_matches_oracle(sp, name, raw):
    want_c, want_inv = oracle.unique_coords(raw)
    c = sp.sp_coords_build(dev(raw), 1)
    assert c.n == len(want_c)
    assert np.array_equal(c.coords().cpu().numpy(), want_c)
    assert np.array_equal(c.inverse().cpu().numpy(), want_inv)


def test_coords_build_more_than_4M_rows_few_distinct(sp):
    """4.5 M raw rows drawn from ~50 k distinct coordinates: 4395 numbering blocks, i.e. look-back chains that
    span dozens of 64-block windows."""
    rng = np.random.default_rng(21)
    distinct = random_coords(22, 50000, 60, batches=4, lo=-30)
    raw = distinct[rng.integers(0, len(distinct), 4_500_000)]
    want_c, want_inv = oracle.unique_coords(raw)
    c = sp.sp_coords_build(dev(raw), 1)
    assert c.n == len(want_c)
    assert np.array_equal(c.coords().cpu().numpy(), want_c)
    assert np.array_equal(c.inverse().cpu().numpy(), want_inv)


def test_more_unresolved_builds_than_mail_slots(sp):
    """2048 builds may have their counts waiting in pinned host memory; the builds beyond that fall back to a
    blocking read-back.  2200 handles are built before any count is asked for; all must be right, and the slots
    must come back when the handles are destroyed."""
    rng = np.random.default_rng(5)
    raws = [rng.integers(0, 6, size=(int(rng.integers(1, 40)), 4)).astype(np.int32) for _ in range(2200)]
    big = dev(np.concatenate(raws))
    hs, at = [], 0
    for r in raws:
        hs.append(sp.sp_coords_build(big[at:at + len(r)], 1))
        at += len(r)
    for i in (0, 1, 2047, 2048, 2049, 2199, 1000):
        want_c, want_inv = oracle.unique_coords(raws[i])
        assert hs[i].n == len(want_c)
        assert np.array_equal(hs[i].coords().cpu().numpy(), want_c)
        assert np.array_equal(hs[i].inverse().cpu().numpy(), want_inv)
    assert [h.n for h in hs] == [len(np.unique(r, axis=0)) for r in raws]
    for h in hs:
        h.close()
    # handles dropped before anybody asked for their counts: their slots are parked until the kernels have
    # delivered, then reused; builds on another stream meanwhile must not see a late delivery
    side = torch.cuda.Stream()
    for rnd in range(3):
        hs, at = [], 0
        for r in raws[:900]:
            hs.append(sp.sp_coords_build(big[at:at + len(r)], 1))
            at += len(r)
        for h in hs:
            h.close()
        with torch.cuda.stream(side):
            side.wait_stream(torch.cuda.current_stream())
            c2 = sp.sp_coords_build(big[:len(raws[0])], 1)
            assert c2.n == len(np.unique(raws[0], axis=0))
            c2.close()
    torch.cuda.synchronize()
    want = oracle_steps(raws[0], 3, 1, 1, 1)     # slots are free again: builds work as before
    c = sp.sp_coords_build(dev(raws[0]), 1)
    km, co = sp.sp_kmap_build(c, 3, 1, 1)
    check_map(sp, km, want, len(want["c_in"]), len(want["c_out"]))


def test_coords_build_empty(sp):
    c = sp.sp_coords_build(torch.empty((0, 4), dtype=torch.int32, device="cuda"), 1)
    assert c.n == 0
    km, co = sp.sp_kmap_build(c, 3, 1, 1)
    assert km.total == 0 and km.n_in == 0 and km.n_out == 0 and co.n == 0
    w = torch.zeros((27, 16, 16), device="cuda")
    y = sp.sp_conv_fwd(km, torch.empty((0, 16), device="cuda"), w)
    assert y.shape == (0, 16)
    dw = sp.sp_conv_bwd_weight(km, torch.empty((0, 16), device="cuda"), torch.empty((0, 16), device="cuda"))
    assert torch.count_nonzero(dw).item() == 0


def test_coords_out_of_range_is_an_error(sp):
    for bad in ([[0, 40000, 0, 0]], [[70000, 0, 0, 0]], [[-1, 0, 0, 0]], [[0, 0, 0, -32769]]):
        c = sp.sp_coords_build(dev(np.array(bad, np.int32)), 1)      # found on the device ...
        with pytest.raises(sp.SpError) as e:
            c.n                                                      # ... reported when the count is asked for
        assert e.value.code == -2
        c = sp.sp_coords_build(dev(np.array(bad, np.int32)), 1)
        km, _ = sp.sp_kmap_build(c, 3, 1, 1)                         # a map built on it reports it as well
        with pytest.raises(sp.SpError) as e:
            km.n_in
        assert e.value.code == -2


def test_measured_mfma_roof_is_plausible(sp):
    """The register-resident MFMA loop must land between a third of the published dense peaks and just above them
    (157.3 TFLOP/s fp32, 2.5 PFLOP/s bf16 on this GPU): it is what bench.py prints as the measured roof."""
    f32 = sp.sp_measure_mfma_peak(torch.float32)
    bf16 = sp.sp_measure_mfma_peak(torch.bfloat16)
    assert 50.0 < f32 < 170.0, f32
    assert 800.0 < bf16 < 2700.0, bf16


def test_bad_arguments(sp):
    c = sp.sp_coords_build(dev(spgen.coords_config(0)), 1)
    for args, code in (((0, 1, 1), -1), ((6, 1, 1), -1), ((3, 0, 1), -1), ((3, 1, 0), -1), ((3, 2, 2), -5)):
        with pytest.raises(sp.SpError) as e:
            sp.sp_kmap_build(c, *args)
        assert e.value.code == code


# ------------------------------------------------------------------ steps 1 + 2: kernel maps
MAP_CASES = [
    # name, raw coords, tensor stride, K, stride, dilation
    ("cfg0_k3", spgen.coords_config(0), 1, 3, 1, 1),
    ("cfg1_k3", spgen.coords_config(1), 1, 3, 1, 1),
    ("cfg1_k3_d2", spgen.coords_config(1), 1, 3, 1, 2),
    ("cfg1_k2s2", spgen.coords_config(1), 1, 2, 2, 1),
    ("cfg1_k3s2", spgen.coords_config(1), 1, 3, 2, 1),
    ("cfg0_k5", spgen.coords_config(0), 1, 5, 1, 1),
    ("cfg0_k1", spgen.coords_config(0), 1, 1, 1, 1),
    ("cfg0_k2s1", spgen.coords_config(0), 1, 2, 1, 1),
    ("cfg0_k4s1", spgen.coords_config(0), 1, 4, 1, 1),
    ("cfg1_k4s2", spgen.coords_config(1, 0.3), 1, 4, 2, 1),
    ("neg_k4s4", random_coords(4, 30000, 30, batches=2, lo=-15), 1, 4, 4, 1),
    ("neg_k3s2", random_coords(5, 30000, 30, batches=2, lo=-15), 1, 3, 2, 1),
    ("neg_k2s2", random_coords(6, 30000, 30, batches=2, lo=-15), 1, 2, 2, 1),
    ("ts2_k3", random_coords(7, 20000, 20, batches=2, lo=-10) * np.array([1, 2, 2, 2], np.int32), 2, 3, 1, 1),
    ("ts2_k2s2", random_coords(8, 20000, 20, batches=2, lo=-10) * np.array([1, 2, 2, 2], np.int32), 2, 2, 2, 1),
    ("tail_257", random_coords(9, 257, 7, batches=1)[:257], 1, 3, 1, 1),
    ("one_voxel", np.array([[0, 0, 0, 0]], np.int32), 1, 3, 1, 1),
    # voxels on the faces of the packable range: a neighbour beyond it is absent, never a wrapped-around key
    ("range_faces_k3", np.array([[65535, 32767, 32767, 32767], [65535, 32766, 32767, 32767], [0, -32768, -32768, -32768],
                                 [0, -32768, -32768, -32767], [65534, -32768, 32767, 0], [65535, -32768, 32767, 0],
                                 [0, 32767, -32768, 5], [1, -32768, -32768, 5]], np.int32), 1, 3, 1, 1),
    ("range_faces_k5_d2", np.array([[65535, 32767, 32767, 32767], [65535, 32763, 32767, 32767], [0, -32768, -32768, -32768],
                                    [0, -32768, -32764, -32768], [1, 32767, 32767, 32767]], np.int32), 1, 5, 1, 2),
    ("range_faces_k2s2", np.array([[65535, 32767, 32767, 32767], [65535, 32766, 32766, 32766], [0, -32768, -32768, -32768],
                                   [0, -32767, -32768, -32767]], np.int32), 1, 2, 2, 1),
]


def check_map(sp, km, want, n_in, n_out):
    assert (km.n_in, km.n_out) == (n_in, n_out)
    assert np.array_equal(km.counts, want["counts"])
    assert km.total == int(want["counts"].sum())
    gin, gout = km.pairs()
    gin, gout = sort_lists(gin.cpu().numpy(), gout.cpu().numpy(), km.counts)
    assert np.array_equal(gin, want["pair_in"])
    assert np.array_equal(gout, want["pair_out"])


@pytest.mark.parametrize("name,raw,ts,K,stride,dil", MAP_CASES, ids=[c[0] for c in MAP_CASES])
def test_kmap_matches_oracle(sp, name, raw, ts, K, stride, dil):
    want = oracle_steps(raw, K, stride, dil, ts)
    c = sp.sp_coords_build(dev(raw), ts)
    km, co = sp.sp_kmap_build(c, K, stride, dil)
    assert co.n == len(want["c_out"]) and co.tensor_stride == want["ts_out"]
    assert np.array_equal(co.coords().cpu().numpy(), want["c_out"])
    if stride > 1:
        assert np.array_equal(co.inverse().cpu().numpy(), want["parent"])
    check_map(sp, km, want, len(want["c_in"]), len(want["c_out"]))

    # neighbour tables agree with the pair lists
    nbr_out, nbr_in, rev_out, rev_in = km.table()
    nbr_out, nbr_in = nbr_out.cpu().numpy(), nbr_in.cpu().numpy()
    assert not rev_out
    if rev_in:
        nbr_in = nbr_in[::-1]
    base = 0
    for k, cnt in enumerate(want["counts"]):
        i, o = want["pair_in"][base:base + cnt], want["pair_out"][base:base + cnt]
        exp_out = np.full(km.n_out, -1, np.int32)
        exp_out[o] = i
        exp_in = np.full(km.n_in, -1, np.int32)
        exp_in[i] = o
        assert np.array_equal(nbr_out[k], exp_out)
        assert np.array_equal(nbr_in[k], exp_in)
        base += cnt

    # transposed map: same pairs, roles swapped
    kt = sp.sp_kmap_transpose(km)
    tin, tout, tcounts = oracle.transpose_map(want["pair_in"], want["pair_out"], want["counts"])
    check_map(sp, kt, dict(pair_in=tin, pair_out=tout, counts=tcounts), len(want["c_out"]), len(want["c_in"]))


def test_map_build_is_deterministic(sp):
    raw = dev(spgen.coords_config(1))
    ref = None
    for _ in range(20):
        c = sp.sp_coords_build(raw, 1)
        km, co = sp.sp_kmap_build(c, 3, 2, 1)
        got = (c.coords().cpu().numpy().tobytes(), co.coords().cpu().numpy().tobytes(),
               km.pairs()[0].cpu().numpy().tobytes(), km.pairs()[1].cpu().numpy().tobytes(),
               km.table()[0].cpu().numpy().tobytes(), km.table()[1].cpu().numpy().tobytes())
        if ref is None:
            ref = got
        assert got == ref


# ------------------------------------------------------------------ step 3 and gradients
def conv_case(sp, raw, ts, K, stride, dil, cin, cout, bf16, seed, transposed=False):
    want = oracle_steps(raw, K, stride, dil, ts)
    pin, pout, counts = want["pair_in"], want["pair_out"], want["counts"]
    n_in, n_out = len(want["c_in"]), len(want["c_out"])
    c = sp.sp_coords_build(dev(raw), ts)
    km, _ = sp.sp_kmap_build(c, K, stride, dil)
    if transposed:
        pin, pout, counts = oracle.transpose_map(pin, pout, counts)
        n_in, n_out = n_out, n_in
        km = sp.sp_kmap_transpose(km)
    kvol = K ** 3
    X = spgen.features(seed, n_in, cin, bf16)
    dY = spgen.features(seed + 1, n_out, cout, bf16)
    W = spgen.weights(seed + 2, kvol, cin, cout, bf16)
    tdt = torch.bfloat16 if bf16 else torch.float32
    tol = TOL_BF16 if bf16 else TOL_F32
    x, dy, w = dev(X, tdt), dev(dY, tdt), dev(W, tdt)

    y = sp.sp_conv_fwd(km, x, w)
    dx = sp.sp_conv_bwd_data(km, dy, w)
    dw = sp.sp_conv_bwd_weight(km, x, dy)
    torch.cuda.synchronize()
    assert dw.dtype == torch.float32
    Y = oracle.conv_fwd(pin, pout, counts, X, W, n_out)
    dX = oracle.conv_bwd_data(pin, pout, counts, dY, W, n_in)
    dW = oracle.conv_bwd_weight(pin, pout, counts, X, dY)
    e_y = rel_err(y.float().cpu().numpy(), Y)
    e_dx = rel_err(dx.float().cpu().numpy(), dX)
    e_dw = rel_err(dw.cpu().numpy(), dW)
    print(f"rel err fwd {e_y:.2e} dgrad {e_dx:.2e} wgrad {e_dw:.2e} (tol {tol:g}); plain |g-r|/|r| over |r| >= rms: "
          f"{rel_err_large(y.float().cpu().numpy(), Y):.2e} {rel_err_large(dx.float().cpu().numpy(), dX):.2e} "
          f"{rel_err_large(dw.cpu().numpy(), dW):.2e}; n_in {n_in} n_out {n_out} pairs {int(counts.sum())}")
    assert e_y <= tol and e_dx <= tol
    assert e_dw <= (TOL_F32 if not bf16 else TOL_BF16)       # dW is fp32 storage for both
    # rows / offsets without pairs are exact zeros
    dead = np.setdiff1d(np.arange(n_out), pout)
    if len(dead):
        assert torch.count_nonzero(y[torch.from_numpy(dead).cuda()]).item() == 0
    for k, cnt in enumerate(counts):
        if cnt == 0:
            assert torch.count_nonzero(dw[k]).item() == 0


CONV_CASES = [
    # name, cfg / raw, scale, ts, K, stride, dil, cin, cout, bf16, transposed
    ("cfg0_f32_16x16", 0, 1.0, 1, 3, 1, 1, 16, 16, False, False),
    ("cfg1_f32_32x64", 1, 1.0, 1, 3, 1, 1, 32, 64, False, False),
    ("cfg1_f32_d2", 1, 0.25, 1, 3, 1, 2, 32, 64, False, False),
    ("cfg1_f32_k3s2", 1, 0.25, 1, 3, 2, 1, 32, 32, False, False),
    ("cfg1_f32_64x16", 1, 0.1, 1, 3, 1, 1, 64, 16, False, False),
    ("cfg1_f32_64x64", 1, 0.25, 1, 3, 1, 1, 64, 64, False, False),      # weight matrix held in two halves
    ("cfg1_f32_64x128", 1, 0.1, 1, 3, 1, 1, 64, 128, False, False),
    ("cfg1_bf16_128x64_sparse", 1, 0.25, 1, 3, 1, 1, 128, 64, True, False),
    ("cfg1_f32_128x128", 1, 0.05, 1, 3, 1, 1, 128, 128, False, False),
    ("cfg1_f32_256x48", 1, 0.02, 1, 3, 1, 1, 256, 48, False, False),
    ("cfg0_f32_3x5_plain", 0, 1.0, 1, 3, 1, 1, 3, 5, False, False),
    ("cfg0_f32_20x24_plain", 0, 1.0, 1, 3, 1, 1, 20, 24, False, False),
    ("cfg2_bf16_down", 2, 0.05, 1, 2, 2, 1, 64, 128, True, False),
    ("cfg2_bf16_up", 2, 0.05, 1, 2, 2, 1, 128, 64, True, True),
    ("cfg3_bf16_32x64", 3, 0.05, 1, 3, 1, 1, 32, 64, True, False),
    ("cfg3_bf16_128x128", 3, 0.02, 1, 3, 1, 1, 128, 128, True, False),
    ("cfg3_bf16_256x256", 3, 0.01, 1, 3, 1, 1, 256, 256, True, False),
    ("cfg3_bf16_k3s2_64x128", 3, 0.05, 1, 3, 2, 1, 64, 128, True, False),
    ("cfg0_bf16_16x16_plain", 0, 1.0, 1, 3, 1, 1, 16, 16, True, False),
    ("cfg4_bf16_64x64_d2", 4, 0.02, 1, 3, 1, 2, 64, 64, True, False),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=[c[0] for c in CONV_CASES])
def test_conv_matches_oracle(sp, case):
    name, cfg, scale, ts, K, stride, dil, cin, cout, bf16, transposed = case
    raw = spgen.coords_config(cfg, scale)
    conv_case(sp, raw, ts, K, stride, dil, cin, cout, bf16, seed=1000 + len(name), transposed=transposed)


def test_plain_kernel_long_sums_stay_within_tolerance(sp):
    """5x5x5 kernel on a full cube, 48 -> 48 fp32 (a shape the plain one-thread-per-output kernel takes): up to 6000
    terms per output.  Summed as one chain this measured 8e-6; per-link dot products first, it is 1.3e-6."""
    conv_case(sp, full_cubes(10, 1), 1, 5, 1, 1, 48, 48, False, seed=4848)


def full_cubes(side, batches):
    """Every voxel of a side^3 cube per cloud, rows shuffled: interior rows have all 27 neighbours, so the map is
    dense enough for the row-stationary wide-layer kernel to be chosen."""
    g = np.arange(side, dtype=np.int32)
    x, y, z = np.meshgrid(g, g, g, indexing="ij")
    one = np.stack([x.ravel(), y.ravel(), z.ravel()], 1)
    rows = np.concatenate([np.concatenate([np.full((len(one), 1), b, np.int32), one], 1) for b in range(batches)])
    return rows[np.random.default_rng(11).permutation(len(rows))]


@pytest.mark.parametrize("cin,cout,side,batches", [(128, 128, 9, 2), (256, 256, 8, 3), (128, 256, 7, 1), (256, 128, 10, 1),
                                                  (64, 64, 9, 2), (64, 128, 8, 1), (128, 64, 8, 2)])
def test_wide_bf16_on_dense_maps(sp, cin, cout, side, batches):
    # rows are not a multiple of the 256-row tile: ragged last tile; forward and both gradients
    conv_case(sp, full_cubes(side, batches), 1, 3, 1, 1, cin, cout, True, seed=77 + cin + side)


@pytest.mark.parametrize("K,cin,cout,transposed,side", [(3, 128, 256, False, 9), (2, 64, 128, False, 10),
                                                        (2, 256, 128, True, 8), (3, 256, 64, True, 7)])
def test_wide_bf16_strided_maps_with_position_classes(sp, K, cin, cout, transposed, side):
    # stride 2: the input side of the map is walked in position-class order with per-tile offset masks
    # (data gradient of the strided conv; forward of the transposed one)
    conv_case(sp, full_cubes(side, 2), 1, K, 2, 1, cin, cout, True, seed=99 + K + cin, transposed=transposed)


@pytest.mark.parametrize("K,stride,cin,cout,side,batches", [
    (1, 1, 128, 128, 6, 1),      # one offset
    (5, 1, 128, 64, 6, 1),       # 125 offsets: four mask words
    (3, 3, 128, 128, 9, 1),      # stride 3: 27 position classes
    (3, 4, 128, 64, 8, 1),       # stride 4: more classes than the class order handles, plain row order
    (2, 1, 256, 128, 5, 2),      # even kernel at stride 1: two separate map sides
])
def test_wide_bf16_corner_shapes(sp, K, stride, cin, cout, side, batches):
    conv_case(sp, full_cubes(side, batches), 1, K, stride, 1, cin, cout, True, seed=31 + K * 7 + stride)


def test_wide_bf16_tiny_inputs(sp):
    one = np.array([[0, 3, -2, 5]], np.int32)
    conv_case(sp, one, 1, 3, 1, 1, 128, 128, True, seed=5)
    conv_case(sp, random_coords(12, 257, 5, batches=1), 1, 3, 1, 1, 256, 256, True, seed=6)


def test_identity_weights_reproduce_input_bit_exactly(sp):
    raw = spgen.coords_config(1, 0.2)
    c = sp.sp_coords_build(dev(raw), 1)
    km, _ = sp.sp_kmap_build(c, 3, 1, 1)
    X = spgen.features(5, c.n, 32)
    W = np.zeros((27, 32, 32), np.float32)
    W[13] = np.eye(32)
    y = sp.sp_conv_fwd(km, dev(X), dev(W))
    assert np.array_equal(y.cpu().numpy(), X)


def test_conv_is_reproducible_run_to_run(sp):
    raw = spgen.coords_config(1, 0.5)
    c = sp.sp_coords_build(dev(raw), 1)
    km, _ = sp.sp_kmap_build(c, 3, 1, 1)
    x = dev(spgen.features(1, c.n, 32))
    dy = dev(spgen.features(2, c.n, 64))
    w = dev(spgen.weights(3, 27, 32, 64))
    ref = None
    for _ in range(3):
        got = (sp.sp_conv_fwd(km, x, w).cpu().numpy().tobytes(), sp.sp_conv_bwd_data(km, dy, w).cpu().numpy().tobytes(),
               sp.sp_conv_bwd_weight(km, x, dy).cpu().numpy().tobytes())
        if ref is None:
            ref = got
        assert got == ref
