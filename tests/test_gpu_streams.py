"""Device memory and streams: two streams driving the library at once (the pool hands blocks from one stream to
the other only behind an event), and the caller's allocator installed through sp_set_allocator.  Results are
compared with the CPU oracle as everywhere else."""
import numpy as np
import pytest
import torch

import oracle
from paper_2012_13846_amd import spgen
from util import TOL_F32, oracle_steps, rel_err, sort_lists

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    from paper_2012_13846_amd import binding
    binding.lib()
    return binding


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(dtype) if dtype is not None else t


def oracle_case(raw, K, stride, cin, cout, seed):
    want = oracle_steps(raw, K, stride, 1, 1)
    n_in, n_out = len(want["c_in"]), len(want["c_out"])
    X = spgen.features(seed, n_in, cin)
    dY = spgen.features(seed + 1, n_out, cout)
    W = spgen.weights(seed + 2, K ** 3, cin, cout)
    pin, pout, counts = want["pair_in"], want["pair_out"], want["counts"]
    return dict(want=want, X=X, dY=dY, W=W, n_in=n_in, n_out=n_out,
                Y=oracle.conv_fwd(pin, pout, counts, X, W, n_out),
                dX=oracle.conv_bwd_data(pin, pout, counts, dY, W, n_in),
                dW=oracle.conv_bwd_weight(pin, pout, counts, X, dY))


def check_case(sp, case, got):
    km_lists, y, dx, dw = got
    want = case["want"]
    gin, gout, counts = km_lists
    assert np.array_equal(counts, want["counts"])
    gin, gout = sort_lists(gin, gout, counts)
    assert np.array_equal(gin, want["pair_in"]) and np.array_equal(gout, want["pair_out"])
    assert rel_err(y, case["Y"]) <= TOL_F32
    assert rel_err(dx, case["dX"]) <= TOL_F32
    assert rel_err(dw, case["dW"]) <= TOL_F32


def test_two_streams_interleaved(sp):
    """The same workload driven from two streams with no synchronisation between them, handles dropped at different
    moments so that freed blocks of one stream are picked up by the other."""
    raw = spgen.coords_config(1, 0.4)
    cases = [oracle_case(raw, 3, 1, 32, 64, 300), oracle_case(raw, 3, 2, 32, 32, 310)]
    params = [(3, 1), (3, 2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    d_raw = dev(raw)
    ins = [(dev(c["X"]), dev(c["dY"]), dev(c["W"])) for c in cases]
    torch.cuda.synchronize()
    crossed0 = sp.sp_pool_cross_stream()
    results = []
    pending = [None, None]
    for rnd in range(6):
        for i in (0, 1):
            j = (i + rnd) % 2               # alternate which stream runs which case
            with torch.cuda.stream(streams[i]):
                c = sp.sp_coords_build(d_raw, 1)
                km, co = sp.sp_kmap_build(c, *params[j], 1)
                x, dy, w = ins[j]
                y = sp.sp_conv_fwd(km, x, w)
                dx = sp.sp_conv_bwd_data(km, dy, w)
                dw = sp.sp_conv_bwd_weight(km, x, dy)
                gin, gout = km.pairs()
                lists = (gin.clone(), gout.clone(), km.counts.copy())
                results.append((j, lists, y, dx, dw))
                # keep this round's handles until the stream's next round: they are freed while the other
                # stream is in the middle of its own build
                pending[i] = (c, km, co)
    pending = None
    torch.cuda.synchronize()
    for j, lists, y, dx, dw in results:
        check_case(sp, cases[j], ((lists[0].cpu().numpy(), lists[1].cpu().numpy(), lists[2]),
                                  y.cpu().numpy(), dx.cpu().numpy(), dw.cpu().numpy()))
    print("blocks handed between streams:", sp.sp_pool_cross_stream() - crossed0)
    assert sp.sp_pool_cross_stream() > crossed0


def test_callers_allocator(sp):
    """All device memory of a map build and the three convolutions from torch's caching allocator."""
    raw = spgen.coords_config(1, 0.3)
    case = oracle_case(raw, 3, 2, 32, 64, 320)
    torch.cuda.synchronize()
    held = sp.sp_pool_bytes()
    calls0 = dict(sp.allocator_calls)
    sp.use_torch_allocator(True)
    try:
        c = sp.sp_coords_build(dev(raw), 1)
        km, co = sp.sp_kmap_build(c, 3, 2, 1)
        x, dy, w = dev(case["X"]), dev(case["dY"]), dev(case["W"])
        y = sp.sp_conv_fwd(km, x, w)
        dx = sp.sp_conv_bwd_data(km, dy, w)
        dw = sp.sp_conv_bwd_weight(km, x, dy)
        gin, gout = km.pairs()
        got = ((gin.cpu().numpy(), gout.cpu().numpy(), km.counts), y.cpu().numpy(), dx.cpu().numpy(), dw.cpu().numpy())
    finally:
        sp.use_torch_allocator(False)
    check_case(sp, case, got)
    assert sp.sp_pool_bytes() == held, "the library's own pool grew while the caller's allocator was installed"
    n_alloc = sp.allocator_calls["alloc"] - calls0["alloc"]
    assert n_alloc > 10
    # handles made under the caller's allocator give their blocks back to it, also after the pool is restored
    c.close(), km.close(), co.close()
    assert sp.allocator_calls["free"] - calls0["free"] == n_alloc
    # and the pool works again
    c2 = sp.sp_coords_build(dev(raw), 1)
    assert c2.n == case["n_in"]


def test_steady_state_steps_hold_the_pool_and_host_memory_still(sp):
    """The same step over and over: after the first few the pool holds what it held (no HIP allocation per
    step), the process's resident memory does not creep (handles, mail slots and plans are given back), results
    stay identical, and once every handle is closed a trim leaves nothing in the pool."""
    import gc
    import psutil
    raw = dev(spgen.coords_config(1, 0.2))
    kvol, cin, cout = 27, 32, 64
    w = torch.randn(kvol, cout, cin, device="cuda") * 0.1

    def step(stride):
        c = sp.sp_coords_build(raw, 1)
        km, co = sp.sp_kmap_build(c, 3, stride, 1)
        x = torch.ones(km.n_in, cin, device="cuda")
        dy = torch.ones(km.n_out, cout, device="cuda")
        y = sp.sp_conv_fwd(km, x, w)
        dx = sp.sp_conv_bwd_data(km, dy, w)
        dw = sp.sp_conv_bwd_weight(km, x, dy)
        out = (float(y.sum()), float(dx.sum()), float(dw.sum()))
        km.close(), co.close(), c.close()
        return out

    ref = {}
    for i in range(10):
        ref[1 + i % 2] = step(1 + i % 2)
    torch.cuda.synchronize()
    gc.collect()
    held = sp.sp_pool_bytes()
    rss = psutil.Process().memory_info().rss
    for i in range(300):
        assert step(1 + i % 2) == ref[1 + i % 2]
    torch.cuda.synchronize()
    gc.collect()
    assert sp.sp_pool_bytes() == held, "the pool grew in steady state"
    grown = psutil.Process().memory_info().rss - rss
    assert grown < 32 << 20, f"resident memory grew by {grown >> 20} MiB over 300 steps"
    sp.sp_pool_trim()
    assert sp.sp_pool_bytes() == 0 or sp.sp_pool_bytes() < held   # only blocks of still-open handles remain


def test_host_threads_with_their_own_streams(sp):
    """Four host threads, each with a stream of its own, build maps and run the three convolutions at the same
    time (ctypes drops the interpreter lock inside the library): every thread gets, every time, bit for bit
    what the same work gave when it ran alone."""
    import threading
    jobs = []
    for t in range(4):
        raw = dev(spgen.coords_config(1, 0.1 + 0.05 * t))
        stride = 1 + t % 2
        cin, cout = (32, 64) if t < 2 else (64, 32)
        g = torch.Generator(device="cuda").manual_seed(100 + t)
        w = torch.randn(27, cout, cin, device="cuda", generator=g) * 0.1
        jobs.append((raw, stride, cin, cout, w))

    def work(job):
        raw, stride, cin, cout, w = job
        c = sp.sp_coords_build(raw, 1)
        km, co = sp.sp_kmap_build(c, 3, stride, 1)
        g = torch.Generator(device="cuda").manual_seed(7)
        x = torch.randn(km.n_in, cin, device="cuda", generator=g)
        dy = torch.randn(km.n_out, cout, device="cuda", generator=g)
        y = sp.sp_conv_fwd(km, x, w)
        dx = sp.sp_conv_bwd_data(km, dy, w)
        dw = sp.sp_conv_bwd_weight(km, x, dy)
        gin, gout = km.pairs()
        out = [t.clone() for t in (c.coords(), co.coords(), gin, gout, y, dx, dw)]
        torch.cuda.current_stream().synchronize()
        km.close(), co.close(), c.close()
        return out

    alone = [work(j) for j in jobs]
    errors = []

    def run(t):
        try:
            with torch.cuda.stream(torch.cuda.Stream()):
                for _ in range(25):
                    got = work(jobs[t])
                    for a, b in zip(got, alone[t]):
                        if not torch.equal(a, b):
                            raise AssertionError(f"thread {t}: a result differs from the single-threaded one")
        except Exception as e:   # reported by the main thread
            errors.append(e)

    threads = [threading.Thread(target=run, args=(t,)) for t in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
