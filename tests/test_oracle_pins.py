"""Pins for the CPU oracle: everything here checks `oracle/` against something other than itself.

  - library routines: numpy unique / floor_divide, torch dense conv3d / conv_transpose3d (+ autograd), fp64
  - brute-force coordinate comparison on tiny inputs
  - closed forms and invariants of the kernel map and of Eq. 2 (Sec. III-B)

No GPU, no HIP code.  A plausible mistake in the oracle (dropped term, wrong sign, transposed
operand, wrong offset numbering, truncation instead of floor) fails at least one test.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2012_13846_amd import spgen


def offsets(K):
    """Offset list in the oracle's documented numbering, written independently: z fastest, low to high."""
    c = (K - 1) // 2 if K % 2 else 0
    return [(ax - c, ay - c, az - c) for ax in range(K) for ay in range(K) for az in range(K)]


def random_coords(rng, n, grid, batches=2, lo=0):
    c = np.empty((n, 4), np.int32)
    c[:, 0] = rng.integers(0, batches, n)
    c[:, 1:] = rng.integers(lo, lo + grid, (n, 3))
    return c


def split_lists(pin, pout, counts):
    out, base = [], 0
    for c in counts:
        out.append(np.stack([pin[base:base + c], pout[base:base + c]], 1))
        base += c
    return out


# ------------------------------------------------------------------ coordinates
def test_unique_matches_numpy_first_occurrence():
    rng = np.random.default_rng(1)
    raw = random_coords(rng, 5000, 9, batches=3, lo=-4)
    c, inv = oracle.unique_coords(raw)
    u, first, inverse = np.unique(raw, axis=0, return_index=True, return_inverse=True)
    order = np.argsort(first)                       # first-occurrence order
    assert np.array_equal(c, u[order])
    rank = np.empty_like(order)
    rank[order] = np.arange(len(order))
    assert np.array_equal(inv, rank[inverse.reshape(-1)])
    assert np.array_equal(c[inv], raw)


def test_unique_empty_and_single():
    c, inv = oracle.unique_coords(np.zeros((0, 4), np.int32))
    assert c.shape == (0, 4) and inv.shape == (0,)
    c, inv = oracle.unique_coords(np.array([[1, 2, 3, 4]] * 3, np.int32))
    assert c.tolist() == [[1, 2, 3, 4]] and inv.tolist() == [0, 0, 0]


def test_strided_coords_true_floor_with_negatives():
    rng = np.random.default_rng(2)
    cin, _ = oracle.unique_coords(random_coords(rng, 3000, 21, lo=-10))
    for ts, s in ((1, 2), (2, 2), (1, 3)):
        cin_ts = cin.copy()
        cin_ts[:, 1:] *= ts
        cout, parent, ts_out = oracle.strided_coords(cin_ts, ts, s)
        assert ts_out == ts * s
        fl = cin_ts.copy()
        fl[:, 1:] = np.floor_divide(cin_ts[:, 1:], ts * s) * (ts * s)   # numpy's floor division
        assert np.array_equal(cout[parent], fl)
        u, first = np.unique(fl, axis=0, return_index=True)
        assert np.array_equal(cout, u[np.argsort(first)])


def test_stride1_keeps_coordinates():
    cin, _ = oracle.unique_coords(random_coords(np.random.default_rng(3), 500, 8))
    cout, parent, ts = oracle.strided_coords(cin, 4, 1)
    assert np.array_equal(cout, cin) and ts == 4 and np.array_equal(parent, np.arange(len(cin)))


# ------------------------------------------------------------------ kernel maps
def brute_force_map(cin, cout, K, step):
    """O(n_out * n_in * K^3) coordinate comparison, numpy broadcasting, no search structure."""
    lists = []
    for off in offsets(K):
        tgt = cout.copy()
        tgt[:, 1:] += np.asarray(off, np.int32) * step
        eq = np.all(cin[:, None, :] == tgt[None, :, :], axis=2)     # [n_in][n_out]
        i, o = np.nonzero(eq)                                       # row-major: sorted by (in, out)
        lists.append(np.stack([i, o], 1).astype(np.int32))
    return lists


@pytest.mark.parametrize("K,stride,dil,ts", [(3, 1, 1, 1), (3, 1, 2, 1), (3, 1, 1, 2), (2, 2, 1, 1),
                                             (3, 2, 1, 1), (2, 2, 1, 2), (5, 1, 1, 1), (1, 1, 1, 1)])
def test_kmap_equals_brute_force(K, stride, dil, ts):
    rng = np.random.default_rng(10 + K + stride + dil + ts)
    cin, _ = oracle.unique_coords(random_coords(rng, 260, 7, lo=-3))
    cin = cin[:200].copy()
    cin[:, 1:] *= ts
    cout, _, _ = oracle.strided_coords(cin, ts, stride)
    pin, pout, counts = oracle.kernel_map(cin, cout, K, dil * ts)
    got = split_lists(pin, pout, counts)
    want = brute_force_map(cin, cout, K, dil * ts)
    assert len(got) == K ** 3
    for g, w in zip(got, want):
        assert np.array_equal(g, w)


def test_full_cube_closed_form_counts():
    # full n^3 cube, K=3: offset (ix,iy,iz) links prod(n - |i_axis|) pairs; total (3n-2)^3
    n = 6
    g = np.stack(np.meshgrid(*[np.arange(n)] * 3, indexing="ij"), -1).reshape(-1, 3)
    cin = np.concatenate([np.zeros((n ** 3, 1), np.int64), g], 1).astype(np.int32)
    _, _, counts = oracle.kernel_map(cin, cin, 3, 1)
    want = [np.prod([n - abs(a) for a in off]) for off in offsets(3)]
    assert counts.tolist() == want
    assert counts.sum() == (3 * n - 2) ** 3


def test_stride1_symmetry_and_identity_centre():
    cin, _ = oracle.unique_coords(spgen.coords_config(0))
    N = len(cin)
    pin, pout, counts = oracle.kernel_map(cin, cin, 3, 1)
    L = split_lists(pin, pout, counts)
    assert np.array_equal(L[13], np.stack([np.arange(N)] * 2, 1))
    for k in range(27):
        mirror = L[26 - k][:, ::-1]
        mirror = mirror[np.lexsort((mirror[:, 1], mirror[:, 0]))]
        assert np.array_equal(L[k], mirror)
        assert counts[k] == counts[26 - k]


def test_k2s2_every_input_in_exactly_one_pair():
    cin, _ = oracle.unique_coords(spgen.coords_config(0))
    cout, parent, _ = oracle.strided_coords(cin, 1, 2)
    pin, pout, counts = oracle.kernel_map(cin, cout, 2, 1)
    assert counts.sum() == len(cin)
    assert np.array_equal(np.sort(pin), np.arange(len(cin)))
    assert np.array_equal(np.unique(pout), np.arange(len(cout)))
    assert np.array_equal(parent[pin], pout)        # the pair's output is the input's coarse parent
    # the offset number is the child's position inside its 2x2x2 cell, z fastest
    child = cin[:, 1:] - cout[parent][:, 1:]
    k_of = (child[:, 0] * 2 + child[:, 1]) * 2 + child[:, 2]
    k_pair = np.repeat(np.arange(8), counts)
    assert np.array_equal(k_of[pin], k_pair)


def test_transposed_map_pair_symmetry():
    cin, _ = oracle.unique_coords(spgen.coords_config(0))
    cout, _, _ = oracle.strided_coords(cin, 1, 2)
    pin, pout, counts = oracle.kernel_map(cin, cout, 2, 1)
    tin, tout, tcounts = oracle.transpose_map(pin, pout, counts)
    assert np.array_equal(tcounts, counts)
    for a, b in zip(split_lists(pin, pout, counts), split_lists(tin, tout, tcounts)):
        assert {tuple(r) for r in a.tolist()} == {(o, i) for (i, o) in b.tolist()}
        assert np.array_equal(b, b[np.lexsort((b[:, 1], b[:, 0]))])


def test_no_pair_crosses_batches_and_batch_independence():
    rng = np.random.default_rng(5)
    a, _ = oracle.unique_coords(random_coords(rng, 400, 6, batches=1))
    b, _ = oracle.unique_coords(random_coords(rng, 300, 6, batches=1))
    b2 = b.copy()
    b2[:, 0] = 1
    both = np.concatenate([a, b2])
    pin, pout, counts = oracle.kernel_map(both, both, 3, 1)
    assert np.array_equal(both[pin, 0], both[pout, 0])
    _, _, ca = oracle.kernel_map(a, a, 3, 1)
    _, _, cb = oracle.kernel_map(b, b, 3, 1)
    assert np.array_equal(counts, ca + cb)
    X = spgen.features(1, len(both), 3)
    W = spgen.weights(2, 27, 3, 5)
    Y = oracle.conv_fwd(pin, pout, counts, X, W, len(both))
    pa = oracle.kernel_map(a, a, 3, 1)
    pb = oracle.kernel_map(b, b, 3, 1)
    Ya = oracle.conv_fwd(*pa, X[:len(a)], W, len(a))
    Yb = oracle.conv_fwd(*pb, X[len(a):], W, len(b))
    assert np.array_equal(Y, np.concatenate([Ya, Yb]))


def test_translation_by_stride_multiple_keeps_maps():
    rng = np.random.default_rng(6)
    cin, _ = oracle.unique_coords(random_coords(rng, 500, 12))
    cout, _, _ = oracle.strided_coords(cin, 1, 2)
    ref = oracle.kernel_map(cin, cout, 3, 1)
    moved = cin.copy()
    moved[:, 1:] += np.array([-40, 2, -6], np.int32)          # multiples of 2, into negatives
    mout, _, _ = oracle.strided_coords(moved, 1, 2)
    got = oracle.kernel_map(moved, mout, 3, 1)
    for r, g in zip(ref, got):
        assert np.array_equal(r, g)
    assert np.array_equal(mout[:, 1:] - cout[:, 1:], np.broadcast_to([-40, 2, -6], cout[:, 1:].shape))


def test_dilation_reduces_to_scaled_coordinates():
    rng = np.random.default_rng(7)
    c, _ = oracle.unique_coords(random_coords(rng, 600, 8))
    c3 = c.copy()
    c3[:, 1:] *= 3
    for r, g in zip(oracle.kernel_map(c, c, 3, 1), oracle.kernel_map(c3, c3, 3, 3)):
        assert np.array_equal(r, g)


def test_row_permutation_equivariance():
    rng = np.random.default_rng(8)
    c, _ = oracle.unique_coords(random_coords(rng, 500, 7))
    N = len(c)
    perm = rng.permutation(N)
    X = spgen.features(3, N, 4)
    W = spgen.weights(4, 27, 4, 6)
    Y = oracle.conv_fwd(*oracle.kernel_map(c, c, 3, 1), X, W, N)
    Yp = oracle.conv_fwd(*oracle.kernel_map(c[perm], c[perm], 3, 1), X[perm], W, N)
    assert np.allclose(Yp, Y[perm], rtol=0, atol=1e-12)


# ------------------------------------------------------------------ convolution vs dense library conv
def dense_case(seed, grid, n, cin_ch, cout_ch, batches=2, lo=0):
    rng = np.random.default_rng(seed)
    c, _ = oracle.unique_coords(random_coords(rng, n, grid, batches, lo))
    X = rng.standard_normal((len(c), cin_ch)).astype(np.float32)
    return rng, c, X


def to_dense(c, F, batches, grid, lo=0):
    d = torch.zeros(batches, F.shape[1], grid, grid, grid, dtype=torch.float64)
    d[c[:, 0], :, c[:, 1] - lo, c[:, 2] - lo, c[:, 3] - lo] = torch.from_numpy(np.asarray(F, np.float64))
    return d


def dense_weight(W, K):
    """[K^3][cout][cin] with z-fastest offset numbering -> torch conv3d weight [cout][cin][Kx][Ky][Kz]."""
    kvol, cout, cin = W.shape
    return torch.from_numpy(np.asarray(W, np.float64)).reshape(K, K, K, cout, cin).permute(3, 4, 0, 1, 2).contiguous()


@pytest.mark.parametrize("K,dil", [(3, 1), (3, 2), (5, 1), (1, 1)])
def test_fwd_bwd_equal_dense_conv3d_stride1(K, dil):
    grid, B, ci, co = 9, 2, 3, 4
    rng, c, X = dense_case(20 + K + dil, grid, 500, ci, co, B, lo=-4)
    N = len(c)
    W = rng.standard_normal((K ** 3, co, ci)).astype(np.float32)
    dY = rng.standard_normal((N, co)).astype(np.float32)
    maps = oracle.kernel_map(c, c, K, dil)
    Y = oracle.conv_fwd(*maps, X, W, N)
    dX = oracle.conv_bwd_data(*maps, dY, W, N)
    dW = oracle.conv_bwd_weight(*maps, X, dY)

    xd = to_dense(c, X, B, grid, lo=-4).requires_grad_(True)
    wd = dense_weight(W, K).requires_grad_(True)
    yd = torch.nn.functional.conv3d(xd, wd, padding=dil * (K - 1) // 2, dilation=dil)   # cross-correlation, Eq. 1
    idx = (c[:, 0], slice(None), c[:, 1] + 4, c[:, 2] + 4, c[:, 3] + 4)
    assert np.allclose(Y, yd[idx].detach().numpy(), rtol=0, atol=1e-12)
    # gradient of <dY, Y restricted to active output sites>
    (yd[idx] * torch.from_numpy(dY.astype(np.float64))).sum().backward()
    assert np.allclose(dX, xd.grad[idx].numpy(), rtol=0, atol=1e-12)
    dWd = wd.grad.permute(2, 3, 4, 0, 1).reshape(K ** 3, co, ci).numpy()
    assert np.allclose(dW, dWd, rtol=0, atol=1e-11)


@pytest.mark.parametrize("K", [2, 3])
def test_fwd_bwd_equal_dense_conv3d_stride2(K):
    grid, B, ci, co = 10, 2, 3, 5
    rng, c, X = dense_case(40 + K, grid, 600, ci, co, B)
    cout, _, ts = oracle.strided_coords(c, 1, 2)
    assert ts == 2
    W = rng.standard_normal((K ** 3, co, ci)).astype(np.float32)
    dY = rng.standard_normal((len(cout), co)).astype(np.float32)
    maps = oracle.kernel_map(c, cout, K, 1)
    Y = oracle.conv_fwd(*maps, X, W, len(cout))
    dX = oracle.conv_bwd_data(*maps, dY, W, len(c))
    dW = oracle.conv_bwd_weight(*maps, X, dY)

    xd = to_dense(c, X, B, grid).requires_grad_(True)
    wd = dense_weight(W, K).requires_grad_(True)
    if K == 2:      # offsets {0,1}^3: a stride-2 window starting at the coarse coordinate, no padding
        yd = torch.nn.functional.conv3d(xd, wd, stride=2)
    else:           # offsets {-1,0,1}^3 centred on the coarse coordinate (an even site)
        yd = torch.nn.functional.conv3d(xd, wd, padding=1, stride=2)
    idx_o = (cout[:, 0], slice(None), cout[:, 1] // 2, cout[:, 2] // 2, cout[:, 3] // 2)
    idx_i = (c[:, 0], slice(None), c[:, 1], c[:, 2], c[:, 3])
    assert np.allclose(Y, yd[idx_o].detach().numpy(), rtol=0, atol=1e-12)
    (yd[idx_o] * torch.from_numpy(dY.astype(np.float64))).sum().backward()
    assert np.allclose(dX, xd.grad[idx_i].numpy(), rtol=0, atol=1e-12)
    assert np.allclose(dW, wd.grad.permute(2, 3, 4, 0, 1).reshape(K ** 3, co, ci).numpy(), rtol=0, atol=1e-11)


def test_transposed_k2s2_equals_dense_conv_transpose3d():
    grid, B, cf, cc = 10, 2, 3, 5            # fine channels (output of the upsampling), coarse channels (its input)
    rng, c_fine, _ = dense_case(50, grid, 600, cf, cc, B)
    c_coarse, _, _ = oracle.strided_coords(c_fine, 1, 2)
    fwd = oracle.kernel_map(c_fine, c_coarse, 2, 1)
    tin, tout, tcounts = oracle.transpose_map(*fwd)
    Yc = rng.standard_normal((len(c_coarse), cc)).astype(np.float32)
    V = rng.standard_normal((8, cf, cc)).astype(np.float32)          # [K^3][out = fine ch][in = coarse ch]
    Z = oracle.conv_fwd(tin, tout, tcounts, Yc, V, len(c_fine))

    yd = torch.zeros(B, cc, grid // 2, grid // 2, grid // 2, dtype=torch.float64)
    yd[c_coarse[:, 0], :, c_coarse[:, 1] // 2, c_coarse[:, 2] // 2, c_coarse[:, 3] // 2] = torch.from_numpy(Yc.astype(np.float64))
    # conv_transpose3d weight is [in][out][Kx][Ky][Kz]
    wt = torch.from_numpy(V.astype(np.float64)).reshape(2, 2, 2, cf, cc).permute(4, 3, 0, 1, 2).contiguous()
    zd = torch.nn.functional.conv_transpose3d(yd, wt, stride=2)
    got = zd[c_fine[:, 0], :, c_fine[:, 1], c_fine[:, 2], c_fine[:, 3]].numpy()
    assert np.allclose(Z, got, rtol=0, atol=1e-12)


def test_identity_and_single_offset_shift():
    c, _ = oracle.unique_coords(spgen.coords_config(0))
    N, ch = len(c), 4
    X = spgen.features(9, N, ch)
    maps = oracle.kernel_map(c, c, 3, 1)
    lookup = {tuple(r): j for j, r in enumerate(c.tolist())}
    for k, off in enumerate(offsets(3)):
        W = np.zeros((27, ch, ch), np.float32)
        W[k] = np.eye(ch)
        Y = oracle.conv_fwd(*maps, X, W, N)
        want = np.zeros((N, ch))
        for o, (b, x, y, z) in enumerate(c.tolist()):
            j = lookup.get((b, x + off[0], y + off[1], z + off[2]))     # x_in[u + i], Eq. 2
            if j is not None:
                want[o] = X[j]
        assert np.array_equal(Y, want)
        if off == (0, 0, 0):
            assert np.array_equal(Y, X.astype(np.float64))


def test_adjoint_identities():
    cfine, _ = oracle.unique_coords(spgen.coords_config(0))
    for K, stride in ((3, 1), (2, 2), (3, 2)):
        cout, _, _ = oracle.strided_coords(cfine, 1, stride)
        maps = oracle.kernel_map(cfine, cout, K, 1)
        ci, co = 5, 3
        X = spgen.features(11, len(cfine), ci)
        dY = spgen.features(12, len(cout), co)
        W = spgen.weights(13, K ** 3, ci, co)
        a = np.sum(dY * oracle.conv_fwd(*maps, X, W, len(cout)))
        b = np.sum(oracle.conv_bwd_data(*maps, dY, W, len(cfine)) * X)
        c = np.sum(oracle.conv_bwd_weight(*maps, X, dY) * W)
        assert abs(a - b) <= 1e-9 * abs(a) and abs(a - c) <= 1e-9 * abs(a)


def test_bf16_helpers_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, -2.5, 3.140625, 1e-3, 65504.0], np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()     # library rounding
    assert np.array_equal(spgen.round_to_bf16(x), want)
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(spgen.round_to_bf16(r), torch.from_numpy(r).to(torch.bfloat16).to(torch.float32).numpy())


def test_generated_occupancy_is_surface_like():
    # the stand-in clouds live in the paper's thin-surface regime (Sec. IV: a few % of the grid occupied)
    c, _ = oracle.unique_coords(spgen.coords_config(0))
    assert 1200 < len(c) < 1800
    assert 0.02 < len(c) / 32 ** 3 < 0.08
    _, _, counts = oracle.kernel_map(c, c, 3, 1)
    assert 4.0 < counts.sum() / len(c) < 12.0


def _paper_values():
    vals = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")):
        line = line.split("#")[0].split()
        if line:
            vals[line[0]] = [float(v) for v in line[1:]]
    return vals


def test_offsets_match_the_set_the_paper_prints():
    # Sec. III-B gives V^1(3) = {-1, 0, 1}; the 3-D offsets of a 3x3x3 kernel are its cube, z fastest
    want = _paper_values()["offsets_1d_k3"]
    # recover offset k from the map of one output voxel inside a full 3x3x3 cube of inputs: its only pair at k
    # is the input at c_out + i_k
    cube = np.array([[0, x, y, z] for x in (-1, 0, 1) for y in (-1, 0, 1) for z in (-1, 0, 1)], np.int32)
    rng = np.random.default_rng(3)
    cube = cube[rng.permutation(27)]
    pin, pout, counts = oracle.kernel_map(cube, np.zeros((1, 4), np.int32), 3, 1)
    assert counts.tolist() == [1] * 27
    off = cube[pin][:, 1:]
    assert sorted(set(off[:, 0].tolist())) == sorted(set(off[:, 1].tolist())) == sorted(set(off[:, 2].tolist())) == want
    assert len(off) == 27 and len({tuple(o) for o in off.tolist()}) == 27
    assert off[:3].tolist() == [[-1, -1, -1], [-1, -1, 0], [-1, -1, 1]]


def test_sweep_clouds_have_the_occupancy_and_dropout_the_paper_reports():
    """The sparsity-sweep stand-ins (Sec. IV-C, Table II): full shapes of 4096 points occupy about 7.6 % of the 32^3
    grid and 2.6 % of the 50^3 grid; with dropout setting p a shape keeps a fraction U[p, 1] of its points, so the
    mean kept fraction is (1 + p) / 2, the ratio Table II's epoch times follow at fixed batch size."""
    pv = _paper_values()
    assert spgen.SWEEP_POINTS == int(pv["points_per_shape"][0]) and list(spgen.SWEEP_P) == pv["sweep_p"]
    for grid, key in ((32, "occupancy_32"), (50, "occupancy_50")):
        occ = [len(oracle.unique_coords(spgen.sweep_cloud(spgen.seed_for(5, c, 3), grid, 1.0))[0]) / grid ** 3 for c in range(48)]
        assert abs(np.mean(occ) - pv[key][0]) < 0.15 * pv[key][0], (grid, np.mean(occ))
    for p in spgen.SWEEP_P:   # kept fraction of the shape's own points (a few of the 4096 fall outside the grid's cube)
        kept = [len(spgen.sweep_cloud(spgen.seed_for(5, c, 4), 32, p)) / len(spgen.sweep_cloud(spgen.seed_for(5, c, 4), 32, 1.0))
                for c in range(400)]
        assert abs(np.mean(kept) - (1 + p) / 2) < 0.03 and min(kept) >= p - 1e-3
    t = pv["epoch_time_sparse_32"]            # batch 256: p = 1, 0.5, 0.25
    for p, ratio in zip((0.5, 0.25), (t[2] / t[1], t[3] / t[1])):
        assert abs(ratio - (1 + p) / 2) < 0.08, (p, ratio)


# ------------------------------------------------------------------ layers between the convolutions
def test_glue_layers_match_torch_library_routines():
    from oracle import glue
    rng = np.random.default_rng(77)
    n, c, B, m = 500, 6, 3, 5
    x = rng.standard_normal((n, c)) * 2 + 0.5
    gamma, beta = rng.standard_normal(c), rng.standard_normal(c)
    bidx = np.sort(rng.integers(0, B, n))
    labels = rng.integers(0, m, B)
    w, bias = rng.standard_normal((m, c)), rng.standard_normal(m)

    xt = torch.tensor(x, requires_grad=True)
    gt, bt = torch.tensor(gamma, requires_grad=True), torch.tensor(beta, requires_grad=True)
    wt, bit = torch.tensor(w, requires_grad=True), torch.tensor(bias, requires_grad=True)
    yt = torch.relu(torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=1e-5))
    yt.retain_grad()
    onehot = torch.nn.functional.one_hot(torch.tensor(bidx), B).double()
    pt = (onehot.T @ yt) / onehot.sum(0)[:, None]
    pt.retain_grad()
    lt = torch.nn.functional.linear(pt, wt, bit)
    lt.retain_grad()
    loss_t = torch.nn.functional.cross_entropy(lt, torch.tensor(labels))
    loss_t.backward()

    y, mean, rstd = glue.bn_relu_fwd(x, gamma, beta, 1e-5, True)
    pooled, counts = glue.pool_avg_fwd(bidx, y, B)
    logits = glue.linear_fwd(pooled, w, bias)
    loss, dlogits = glue.softmax_ce(logits, labels)
    dpool, dw, dbias = glue.linear_bwd(pooled, w, dlogits)
    dy = glue.pool_avg_bwd(bidx, dpool, counts)
    dx, dgamma, dbeta = glue.bn_relu_bwd(x, y, dy, gamma, mean, rstd, True)
    for got, want in ((y, yt), (pooled, pt), (logits, lt), (loss, loss_t), (dlogits, lt.grad), (dpool, pt.grad),
                      (dw, wt.grad), (dbias, bit.grad), (dy, yt.grad), (dx, xt.grad), (dgamma, gt.grad),
                      (dbeta, bt.grad)):
        assert np.allclose(got, want.detach().numpy(), rtol=1e-10, atol=1e-12)
    # without the activation
    y2, mean2, rstd2 = glue.bn_relu_fwd(x, gamma, beta, 1e-3, False)
    x2 = torch.tensor(x, requires_grad=True)
    y2t = torch.nn.functional.batch_norm(x2, None, None, torch.tensor(gamma), torch.tensor(beta), training=True, eps=1e-3)
    g = rng.standard_normal((n, c))
    y2t.backward(torch.tensor(g))
    assert np.allclose(y2, y2t.detach().numpy(), atol=1e-12)
    assert np.allclose(glue.bn_relu_bwd(x, y2, g, gamma, mean2, rstd2, False)[0], x2.grad.numpy(), atol=1e-11)


def test_glue_closed_forms():
    from oracle import glue
    # a single row has variance 0: y = beta, mean = the row, rstd = eps^-1/2
    x = np.array([[1.5, -2.0]])
    y, mean, rstd = glue.bn_relu_fwd(x, np.array([2.0, 3.0]), np.array([0.5, -1.0]), 1e-5, False)
    assert np.allclose(mean, x[0]) and np.allclose(rstd, 1e-5 ** -0.5) and np.allclose(y, [[0.5, -1.0]])
    # two rows +-a: xhat = +-a/sqrt(a^2+eps); ReLU keeps the positive one
    a = 3.0
    y, mean, rstd = glue.bn_relu_fwd(np.array([[a], [-a]]), np.array([1.0]), np.array([0.0]), 1e-5, True)
    assert np.allclose(mean, 0.0) and np.allclose(y[:, 0], [a / np.sqrt(a * a + 1e-5), 0.0])
    # pooling a per-cloud constant returns it; counts are the cloud sizes; the backward spreads g / count
    bidx = np.array([0, 0, 0, 2, 2])
    xs = np.where(bidx[:, None] == 0, 4.0, -1.0) * np.ones((5, 3))
    pooled, counts = glue.pool_avg_fwd(bidx, xs, 3)
    assert np.array_equal(counts, [3, 0, 2])
    assert np.allclose(pooled, [[4, 4, 4], [0, 0, 0], [-1, -1, -1]])
    g = np.arange(9.0).reshape(3, 3)
    dx = glue.pool_avg_bwd(bidx, g, counts)
    assert np.allclose(dx[0], g[0] / 3) and np.allclose(dx[4], g[2] / 2)
    # uniform logits: loss = log(m); dlogits = (1/m - onehot) / clouds
    m, B = 7, 4
    labels = np.array([0, 3, 6, 3])
    loss, d = glue.softmax_ce(np.zeros((B, m)), labels)
    assert np.isclose(loss, np.log(m))
    want = np.full((B, m), 1.0 / m)
    want[np.arange(B), labels] -= 1.0
    assert np.allclose(d, want / B)


@pytest.mark.parametrize("K,stride,ts", [(3, 2, 1), (2, 2, 1), (3, 3, 1), (3, 2, 2), (5, 2, 1)])
def test_strided_links_follow_the_position_class(K, stride, ts):
    """In a strided map an input voxel at residue r (its lattice position modulo the stride, per axis) can only be
    linked by offsets whose displacement is congruent to r modulo the stride: the output coordinates are multiples
    of the stride.  (The GPU path orders the input rows of strided maps by that residue and skips the other
    offsets; this pins the property on the oracle's maps.)"""
    rng = np.random.default_rng(100 + K * 10 + stride)
    raw = np.concatenate([rng.integers(0, 2, (4000, 1)), rng.integers(-12, 12, (4000, 3)) * ts], 1).astype(np.int32)
    c_in, _ = oracle.unique_coords(raw)
    c_out, _, ts_out = oracle.strided_coords(c_in, ts, stride)
    pin, pout, counts = oracle.kernel_map(c_in, c_out, K, ts)
    assert counts.sum() > 0
    centre = (K - 1) // 2 if K % 2 else 0
    k = np.repeat(np.arange(K ** 3), counts)
    d = np.stack([k // (K * K) - centre, (k // K) % K - centre, k % K - centre], 1)
    r = (c_in[pin][:, 1:] // ts) % stride            # numpy's floor modulo
    assert np.array_equal(d % stride, r)
    # and for an even kernel as wide as the stride (offsets 0 .. K-1) the class fixes the offset completely
    if K == stride and K % 2 == 0:
        assert np.array_equal(d, r)


# ------------------------------------------------------------------ pooling over kernel maps
from oracle import pool as opool


def _pool_dense_case(seed, K, stride, grid=8, B=2, ch=3, n=260, ties=False):
    rng = np.random.default_rng(seed)
    c, _ = oracle.unique_coords(random_coords(rng, n, grid, B))
    X = rng.standard_normal((len(c), ch))
    if ties:
        X = np.round(X)                      # many equal values inside one window
    cout, _, _ = oracle.strided_coords(c, 1, stride)
    maps = oracle.kernel_map(c, cout, K, 1)
    return rng, c, cout, X, maps


@pytest.mark.parametrize("K,stride,ties", [(2, 2, False), (3, 1, False), (3, 2, False), (2, 2, True), (3, 1, True)])
def test_pool_max_equals_dense_max_pool3d_with_autograd(K, stride, ties):
    grid, B, ch = 8, 2, 3
    rng, c, cout, X, maps = _pool_dense_case(60 + K + stride, K, stride, grid, B, ch, ties=ties)
    Y, arg = opool.pool_fwd(*maps, X, len(cout), "max")
    dY = rng.standard_normal(Y.shape)
    dX = opool.pool_bwd(*maps, dY, arg, len(c), "max")
    # dense: absent sites hold -inf, so a window's maximum is the maximum over the inputs present
    neg = -1e300
    leaf = torch.from_numpy(X).requires_grad_(True)
    idx = tuple(torch.from_numpy(c[:, j].astype(np.int64)) for j in range(4))
    xd = torch.full((B, grid, grid, grid, ch), neg, dtype=torch.float64).index_put(idx, leaf).permute(0, 4, 1, 2, 3)
    pad = (K - 1) // 2 if K % 2 else 0
    if pad:
        xd = torch.nn.functional.pad(xd, (pad,) * 6, value=neg)
    yd = torch.nn.functional.max_pool3d(xd, K, stride=stride)
    q = stride
    got = yd[cout[:, 0], :, cout[:, 1] // q, cout[:, 2] // q, cout[:, 3] // q]
    assert np.array_equal(Y, got.detach().numpy())
    if not ties:        # with ties the gradient's destination is a convention (lowest offset), pinned below
        (got * torch.from_numpy(dY)).sum().backward()
        assert np.allclose(dX, leaf.grad.numpy(), rtol=0, atol=1e-13)


def test_pool_max_ties_go_to_the_lowest_offset_and_gradient_is_conserved():
    rng, c, cout, X, maps = _pool_dense_case(71, 3, 1, ties=True)
    pin, pout, counts = maps
    Y, arg = opool.pool_fwd(*maps, X, len(cout), "max")
    lists = split_lists(pin, pout, counts)
    # brute force per output row and channel: the lowest offset among the links attaining the maximum
    for o in rng.choice(len(cout), 60, replace=False):
        links = [(k, int(l[l[:, 1] == o][0, 0])) for k, l in enumerate(lists) if (l[:, 1] == o).any()]
        for ch in range(X.shape[1]):
            best = max(X[i, ch] for _, i in links)
            assert Y[o, ch] == best
            assert arg[o, ch] == min(k for k, i in links if X[i, ch] == best)
    dY = rng.standard_normal(Y.shape)
    dX = opool.pool_bwd(*maps, dY, arg, len(c), "max")
    assert np.allclose(dX.sum(0), dY.sum(0), rtol=0, atol=1e-11)      # every output's gradient lands on one input


@pytest.mark.parametrize("K,stride", [(2, 2), (3, 1), (3, 2)])
def test_pool_avg_and_sum_equal_dense_avg_pool3d_with_autograd(K, stride):
    grid, B, ch = 8, 2, 3
    rng, c, cout, X, maps = _pool_dense_case(80 + K + stride, K, stride, grid, B, ch)
    leaf = torch.from_numpy(X).requires_grad_(True)
    idx = tuple(torch.from_numpy(c[:, j].astype(np.int64)) for j in range(4))
    xd = torch.zeros(B, grid, grid, grid, ch, dtype=torch.float64).index_put(idx, leaf).permute(0, 4, 1, 2, 3)
    occ = torch.zeros(B, 1, grid, grid, grid, dtype=torch.float64)
    occ[c[:, 0], :, c[:, 1], c[:, 2], c[:, 3]] = 1.0
    pad = (K - 1) // 2 if K % 2 else 0
    # avg_pool3d with zero padding counted divides by K^3: times K^3 it is the window sum
    win_sum = torch.nn.functional.avg_pool3d(xd, K, stride=stride, padding=pad, count_include_pad=True) * K ** 3
    win_cnt = torch.nn.functional.avg_pool3d(occ, K, stride=stride, padding=pad, count_include_pad=True) * K ** 3
    q = stride
    at = (cout[:, 0], slice(None), cout[:, 1] // q, cout[:, 2] // q, cout[:, 3] // q)
    n_links = opool.link_counts(maps[1], len(cout))
    assert np.array_equal(n_links, np.rint(win_cnt[at].numpy()[:, 0]).astype(np.int64))
    for mode, dense in (("sum", win_sum[at]), ("avg", win_sum[at] / win_cnt[at])):
        Y, arg = opool.pool_fwd(*maps, X, len(cout), mode)
        assert np.allclose(Y, dense.detach().numpy(), rtol=0, atol=1e-12) and (arg == -1).all()
        dY = rng.standard_normal(Y.shape)
        leaf.grad = None
        (dense * torch.from_numpy(dY)).sum().backward(retain_graph=True)
        dX = opool.pool_bwd(*maps, dY, arg, len(c), mode)
        assert np.allclose(dX, leaf.grad.numpy(), rtol=0, atol=1e-12)


def test_pool_closed_forms():
    # a constant feature is its own max and average; its window sum is the link count
    rng, c, cout, X, maps = _pool_dense_case(90, 3, 2)
    ones = np.full((len(c), 2), 2.5)
    n_links = opool.link_counts(maps[1], len(cout))
    assert (n_links >= 1).all()
    assert np.array_equal(opool.pool_fwd(*maps, ones, len(cout), "max")[0], np.full((len(cout), 2), 2.5))
    assert np.allclose(opool.pool_fwd(*maps, ones, len(cout), "avg")[0], 2.5, rtol=0, atol=1e-14)
    assert np.allclose(opool.pool_fwd(*maps, ones, len(cout), "sum")[0], 2.5 * n_links[:, None])
    # sum pooling is the convolution of Eq. 2 with every W_k the identity
    W = np.tile(np.eye(3, dtype=np.float32), (27, 1, 1))
    Xf = X.astype(np.float32)
    assert np.allclose(opool.pool_fwd(*maps, Xf, len(cout), "sum")[0], oracle.conv_fwd(*maps, Xf, W, len(cout)), atol=1e-12)
    assert opool.kernel_offsets(3).tolist() == [list(o) for o in offsets(3)]
    assert opool.kernel_offsets(2).tolist() == [list(o) for o in offsets(2)]


# ------------------------------------------------------------------ generative transposed convolution
@pytest.mark.parametrize("K,stride,ts_in", [(2, 2, 2), (3, 2, 2), (3, 2, 4), (3, 1, 1), (2, 2, 8)])
def test_generative_coords_first_occurrence_order_matches_numpy(K, stride, ts_in):
    rng = np.random.default_rng(100 + K + stride + ts_in)
    c_in, _ = oracle.unique_coords(random_coords(rng, 300, 6, 2, lo=-3) * np.array([1, ts_in, ts_in, ts_in], np.int32))
    c_out, where, ts_out = opool.generative_coords(c_in, ts_in, K, stride)
    assert ts_out == ts_in // stride
    # candidates written out independently, input row by input row, offsets in offset order
    cand = np.array([[r[0], r[1] + o[0] * ts_out, r[2] + o[1] * ts_out, r[3] + o[2] * ts_out]
                     for r in c_in.tolist() for o in offsets(K)], np.int32)
    u, first, inverse = np.unique(cand, axis=0, return_index=True, return_inverse=True)
    order = np.argsort(first)
    assert np.array_equal(c_out, u[order])
    rank = np.empty_like(order)
    rank[order] = np.arange(len(order))
    assert np.array_equal(where.reshape(-1), rank[inverse.reshape(-1)])
    # the map of the generative layer is the stride-`stride` convolution's map from C_out to C_in, transposed:
    # every candidate is one link, so each offset has exactly n_in pairs
    pin, pout, counts = oracle.kernel_map(c_out, c_in, K, ts_out)
    assert (counts == len(c_in)).all()
    tin, tout, tcounts = oracle.transpose_map(pin, pout, counts)
    for k, l in enumerate(split_lists(tin, tout, tcounts)):          # (coarse row, fine row) sorted by coarse row
        assert np.array_equal(l[:, 0], np.arange(len(c_in))) and np.array_equal(l[:, 1], where[:, k])
    if K == stride:
        assert len(c_out) == len(c_in) * K ** 3                      # children of distinct cells never coincide


@pytest.mark.parametrize("K,stride", [(2, 2), (3, 2), (3, 1)])
def test_generative_transposed_conv_equals_dense_conv_transpose3d(K, stride):
    grid, B, cc, cf = 5, 2, 4, 3            # coarse grid cells, coarse channels (input), fine channels (output)
    rng = np.random.default_rng(110 + K + stride)
    cells, _ = oracle.unique_coords(random_coords(rng, 90, grid, B))
    c_in = cells * np.array([1, stride, stride, stride], np.int32)   # tensor stride = stride, so ts_out = 1
    c_out, where, ts_out = opool.generative_coords(c_in, stride, K, stride)
    assert ts_out == 1
    pin, pout, counts = oracle.kernel_map(c_out, c_in, K, 1)
    tin, tout, tcounts = oracle.transpose_map(pin, pout, counts)
    Xc = rng.standard_normal((len(c_in), cc)).astype(np.float32)
    V = rng.standard_normal((K ** 3, cf, cc)).astype(np.float32)     # [K^3][out = fine ch][in = coarse ch]
    Z = oracle.conv_fwd(tin, tout, tcounts, Xc, V, len(c_out))

    xd = torch.zeros(B, cc, grid, grid, grid, dtype=torch.float64)
    xd[cells[:, 0], :, cells[:, 1], cells[:, 2], cells[:, 3]] = torch.from_numpy(Xc.astype(np.float64))
    wt = torch.from_numpy(V.astype(np.float64)).reshape(K, K, K, cf, cc).permute(4, 3, 0, 1, 2).contiguous()
    zd = torch.nn.functional.conv_transpose3d(xd, wt, stride=stride)          # zd[s*u + a] += W[a] x[u], a in 0..K-1
    ctr = (K - 1) // 2 if K % 2 else 0                                         # dense index = coordinate + ctr
    got = zd[c_out[:, 0], :, c_out[:, 1] + ctr, c_out[:, 2] + ctr, c_out[:, 3] + ctr].numpy()
    assert np.allclose(Z, got, rtol=0, atol=1e-12)
    # C_out is exactly the set of sites a transposed convolution with an all-positive kernel reaches
    reach = torch.nn.functional.conv_transpose3d((xd.abs().sum(1, keepdim=True) > 0).double(),
                                                 torch.ones(1, 1, K, K, K, dtype=torch.float64), stride=stride)
    sites = torch.nonzero(reach[:, 0] > 0).numpy()
    sites[:, 1:] -= ctr
    assert {tuple(r) for r in sites.tolist()} == {tuple(r) for r in c_out.tolist()}


# ------------------------------------------------------------------ stage-boundary packing of (C, F)
from oracle import pack as opack


@pytest.mark.parametrize("n,c,dtype", [(0, 8, 0), (1, 1, 1), (1001, 5, 0), (777, 3, 1), (4096, 64, 1)])
def test_pack_layout_parsed_independently_and_round_trip(n, c, dtype):
    import struct
    rng = np.random.default_rng(n + c)
    coords = rng.integers(-30000, 30000, (n, 4)).astype(np.int32)
    feats = rng.standard_normal((n, c)).astype(np.float32)
    bits = feats if dtype == 0 else spgen.f32_to_bf16_bits(feats)
    buf = opack.pack(coords, bits, dtype, 4)
    raw = buf.tobytes()
    magic, ver, nn, cc, dd, ts, zero, c_off, f_off, total = struct.unpack("<4sIqiiiiqqq", raw[:56])
    assert (magic, ver, nn, cc, dd, ts, zero) == (b"SPCF", 1, n, c, dtype, 4, 0)
    elt = 4 if dtype == 0 else 2
    up = lambda v: -(-v // 256) * 256
    assert (c_off, f_off, total) == (256, 256 + up(16 * n), 256 + up(16 * n) + up(n * c * elt))
    assert len(raw) == total == opack.packed_bytes(n, c, dtype)
    assert raw[c_off:c_off + 16 * n] == coords.tobytes()
    assert raw[f_off:f_off + n * c * elt] == bits.tobytes()
    payload = set(range(c_off, c_off + 16 * n)) | set(range(f_off, f_off + n * c * elt)) | set(range(56))
    assert all(raw[i] == 0 for i in range(total) if i not in payload and i < 4096)    # padding is zero
    c2, f2, d2, ts2 = opack.unpack(buf)
    assert np.array_equal(c2, coords) and np.array_equal(f2, bits) and (d2, ts2) == (dtype, 4)
    bad = buf.copy()
    bad[0] = 0
    with pytest.raises(ValueError):
        opack.unpack(bad)
