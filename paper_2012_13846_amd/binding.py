"""ctypes binding of the C-ABI library (include/sp_conv.h).  Argument marshalling only.

Function names equal the C entry points.  torch supplies device memory and the current
stream; every step of the path runs in the library's HIP kernels.  If the library is
missing this module raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsp_conv.so")

SP_F32, SP_BF16 = 0, 1
_vp = C.c_void_p
_lib = None


class SpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sp_conv error {code}: {msg}")
        self.code = code


def lib() -> C.CDLL:
    """Loads libsp_conv.so (built in-tree by paper_2012_13846_amd.build); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2012_13846_amd.build` "
                               "(there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        l.sp_last_error.restype = C.c_char_p
        l.sp_version.restype = C.c_char_p
        l.sp_pool_bytes.restype = C.c_int64
        l.sp_coords_build.argtypes = [_vp, C.c_int64, C.c_int32, _vp, C.POINTER(_vp)]
        l.sp_coords_size.argtypes = [_vp, C.POINTER(C.c_int64), C.POINTER(C.c_int32)]
        l.sp_coords_data.argtypes = [_vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(C.c_int64)]
        l.sp_coords_destroy.argtypes = [_vp]
        l.sp_kmap_build.argtypes = [_vp, C.c_int32, C.c_int32, C.c_int32, _vp, C.POINTER(_vp), C.POINTER(_vp)]
        l.sp_kmap_transpose.argtypes = [_vp, C.POINTER(_vp)]
        l.sp_kmap_build_generative.argtypes = [_vp, C.c_int32, C.c_int32, _vp, C.POINTER(_vp), C.POINTER(_vp)]
        l.sp_pool_fwd.argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, _vp]
        l.sp_pool_bwd.argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, _vp]
        l.sp_kmap_info.argtypes = [_vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32),
                                   C.POINTER(C.c_int64), _vp]
        l.sp_kmap_pairs.argtypes = [_vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(C.c_int64)]
        l.sp_kmap_table.argtypes = [_vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        l.sp_kmap_destroy.argtypes = [_vp]
        for name in ("sp_conv_fwd", "sp_conv_bwd_data", "sp_conv_bwd_weight", "sp_conv_fwd_noalloc"):
            getattr(l, name).argtypes = [_vp, _vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, _vp]
        _lib = l
    return _lib


def _check(rc: int):
    if rc != 0:
        raise SpError(rc, lib().sp_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class _DevView:
    """Borrowed device memory exposed through the CUDA array interface (torch wraps it without copying)."""

    def __init__(self, ptr: int, shape, typestr: str):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": typestr, "data": (ptr, False), "version": 2}


def _view(ptr, shape, typestr, dtype) -> torch.Tensor:
    n = int(np.prod(shape))
    if n == 0 or not ptr:
        return torch.empty(tuple(shape), dtype=dtype, device="cuda")
    return torch.as_tensor(_DevView(int(ptr), shape, typestr), device="cuda")


class Coords:
    """Owns one reference to an sp_coords_t.  The row count `n` is asked for (and waited for) on first use."""

    def __init__(self, handle):
        self._h = handle
        self._n = None
        ts = C.c_int32()
        _check(lib().sp_coords_size(self._h, None, C.byref(ts)))
        self.tensor_stride = ts.value

    @property
    def n(self) -> int:
        if self._n is None:
            n = C.c_int64()
            _check(lib().sp_coords_size(self._h, C.byref(n), None))
            self._n = n.value
        return self._n

    def _data(self):
        pc, pi, nr = _vp(), _vp(), C.c_int64()
        _check(lib().sp_coords_data(self._h, C.byref(pc), C.byref(pi), C.byref(nr)))
        return pc.value, pi.value, nr.value

    def coords(self) -> torch.Tensor:
        """int32 [N][4] view of the distinct coordinates (borrowed: valid while this object lives)."""
        pc, _, _ = self._data()
        return _view(pc, (self.n, 4), "<i4", torch.int32)

    def inverse(self) -> torch.Tensor:
        """int32 [n_raw] view: distinct row each source row merged into."""
        _, pi, nr = self._data()
        return _view(pi, (nr,), "<i4", torch.int32)

    def close(self):
        if self._h:
            lib().sp_coords_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class KMap:
    """Owns an sp_kmap_t.  Sizes and pair counts are asked for (and waited for) on first use."""

    def __init__(self, handle):
        self._h = handle
        self._info = None
        kv = C.c_int32()
        _check(lib().sp_kmap_info(self._h, None, None, C.byref(kv), None, None))
        self.kvol = kv.value

    def _sizes(self):
        if self._info is None:
            ni, no, tot = C.c_int64(), C.c_int64(), C.c_int64()
            counts = np.zeros(self.kvol, dtype=np.int64)
            _check(lib().sp_kmap_info(self._h, C.byref(ni), C.byref(no), None, C.byref(tot), counts.ctypes.data_as(_vp)))
            self._info = (ni.value, no.value, tot.value, counts)
        return self._info

    n_in = property(lambda self: self._sizes()[0])
    n_out = property(lambda self: self._sizes()[1])
    total = property(lambda self: self._sizes()[2])
    counts = property(lambda self: self._sizes()[3])

    def pairs_strided(self):
        """(pair_in, pair_out): int32 [kvol][pair_stride] views; list k is the first counts[k] entries of row k."""
        a, b, st = _vp(), _vp(), C.c_int64()
        _check(lib().sp_kmap_pairs(self._h, C.byref(a), C.byref(b), C.byref(st)))
        shape = (self.kvol, st.value)
        return _view(a.value, shape, "<i4", torch.int32), _view(b.value, shape, "<i4", torch.int32)

    def pairs(self):
        """(pair_in, pair_out): int32 [total], the lists of all offsets concatenated in offset order (a copy)."""
        pi, po = self.pairs_strided()
        counts = self.counts
        if self.total == 0:
            e = torch.empty((0,), dtype=torch.int32, device="cuda")
            return e, e.clone()
        return (torch.cat([pi[k, :int(c)] for k, c in enumerate(counts)]),
                torch.cat([po[k, :int(c)] for k, c in enumerate(counts)]))

    def table(self):
        """(nbr_out [kvol][n_out], nbr_in [kvol][n_in], out_reversed, in_reversed) views."""
        a, b, ro, ri = _vp(), _vp(), C.c_int32(), C.c_int32()
        _check(lib().sp_kmap_table(self._h, C.byref(a), C.byref(b), C.byref(ro), C.byref(ri)))
        return (_view(a.value, (self.kvol, self.n_out), "<i4", torch.int32),
                _view(b.value, (self.kvol, self.n_in), "<i4", torch.int32), bool(ro.value), bool(ri.value))

    def close(self):
        if self._h:
            lib().sp_kmap_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _need_cuda(t: torch.Tensor, dtype=None, name="tensor"):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}")


def sp_coords_build(raw: torch.Tensor, tensor_stride: int = 1) -> Coords:
    _need_cuda(raw, torch.int32, "raw")
    if raw.ndim != 2 or raw.shape[1] != 4:
        raise ValueError("raw must be [n][4] rows (b,x,y,z)")
    h = _vp()
    _check(lib().sp_coords_build(raw.data_ptr() if raw.numel() else None, raw.shape[0], tensor_stride, _stream(),
                                 C.byref(h)))
    return Coords(h)


def sp_kmap_build(coords: Coords, kernel_size: int, stride: int = 1, dilation: int = 1):
    """Returns (KMap, Coords of the output)."""
    hk, hc = _vp(), _vp()
    _check(lib().sp_kmap_build(coords._h, kernel_size, stride, dilation, _stream(), C.byref(hk), C.byref(hc)))
    return KMap(hk), Coords(hc)


def sp_kmap_build_generative(coords: Coords, kernel_size: int, stride: int = 1):
    """Generative transposed convolution: returns (KMap with inputs = `coords`' rows and outputs = the created
    rows, Coords of the created rows)."""
    hk, hc = _vp(), _vp()
    _check(lib().sp_kmap_build_generative(coords._h, kernel_size, stride, _stream(), C.byref(hk), C.byref(hc)))
    return KMap(hk), Coords(hc)


def sp_kmap_transpose(kmap: KMap) -> KMap:
    h = _vp()
    _check(lib().sp_kmap_transpose(kmap._h, C.byref(h)))
    return KMap(h)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SP_F32
    if t.dtype == torch.bfloat16:
        return SP_BF16
    raise ValueError("features must be float32 or bfloat16")


def sp_conv_fwd(kmap: KMap, x: torch.Tensor, w: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """y [n_out][cout] from x [n_in][cin], w [kvol][cout][cin]."""
    _need_cuda(x, None, "x"), _need_cuda(w, x.dtype, "w")
    kvol, cout, cin = w.shape
    if kvol != kmap.kvol or tuple(x.shape) != (kmap.n_in, cin):
        raise ValueError("shape mismatch between kmap, x and w")
    y = out if out is not None else torch.empty((kmap.n_out, cout), dtype=x.dtype, device=x.device)
    _need_cuda(y, x.dtype, "out")
    if tuple(y.shape) != (kmap.n_out, cout):
        raise ValueError("out has the wrong shape")
    _check(lib().sp_conv_fwd(kmap._h, x.data_ptr(), w.data_ptr(), y.data_ptr(), cin, cout, _dt(x), _stream()))
    return y


def sp_conv_fwd_noalloc(kmap: KMap, x: torch.Tensor, w: torch.Tensor, out: torch.Tensor) -> torch.Tensor:
    """sp_conv_fwd into the caller's `out`, through the entry point that allocates no device memory."""
    _need_cuda(x, None, "x"), _need_cuda(w, x.dtype, "w"), _need_cuda(out, x.dtype, "out")
    kvol, cout, cin = w.shape
    if kvol != kmap.kvol or tuple(x.shape) != (kmap.n_in, cin) or tuple(out.shape) != (kmap.n_out, cout):
        raise ValueError("shape mismatch between kmap, x, w and out")
    _check(lib().sp_conv_fwd_noalloc(kmap._h, x.data_ptr(), w.data_ptr(), out.data_ptr(), cin, cout, _dt(x),
                                     _stream()))
    return out


def sp_conv_bwd_data(kmap: KMap, dy: torch.Tensor, w: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """dx [n_in][cin] from dy [n_out][cout], w [kvol][cout][cin]."""
    _need_cuda(dy, None, "dy"), _need_cuda(w, dy.dtype, "w")
    kvol, cout, cin = w.shape
    if kvol != kmap.kvol or tuple(dy.shape) != (kmap.n_out, cout):
        raise ValueError("shape mismatch between kmap, dy and w")
    dx = out if out is not None else torch.empty((kmap.n_in, cin), dtype=dy.dtype, device=dy.device)
    _need_cuda(dx, dy.dtype, "out")
    if tuple(dx.shape) != (kmap.n_in, cin):
        raise ValueError("out has the wrong shape")
    _check(lib().sp_conv_bwd_data(kmap._h, dy.data_ptr(), w.data_ptr(), dx.data_ptr(), cin, cout, _dt(dy), _stream()))
    return dx


def sp_conv_bwd_weight(kmap: KMap, x: torch.Tensor, dy: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """dw fp32 [kvol][cout][cin] from x [n_in][cin], dy [n_out][cout]."""
    _need_cuda(x, None, "x"), _need_cuda(dy, x.dtype, "dy")
    cin, cout = x.shape[1], dy.shape[1]
    if x.shape[0] != kmap.n_in or dy.shape[0] != kmap.n_out:
        raise ValueError("shape mismatch between kmap, x and dy")
    dw = out if out is not None else torch.empty((kmap.kvol, cout, cin), dtype=torch.float32, device=x.device)
    _need_cuda(dw, torch.float32, "out")
    if tuple(dw.shape) != (kmap.kvol, cout, cin):
        raise ValueError("out has the wrong shape")
    _check(lib().sp_conv_bwd_weight(kmap._h, x.data_ptr(), dy.data_ptr(), dw.data_ptr(), cin, cout, _dt(x), _stream()))
    return dw


def sp_pack(coords: torch.Tensor, feats: torch.Tensor, tensor_stride: int = 1) -> torch.Tensor:
    """(C, F) -> one contiguous uint8 device buffer (header + coordinates + features)."""
    _need_cuda(coords, torch.int32, "coords"), _need_cuda(feats, None, "feats")
    n, c = feats.shape
    if tuple(coords.shape) != (n, 4):
        raise ValueError("coords must be [n][4] with the features' row count")
    l = lib()
    l.sp_pack_bytes.restype = C.c_int64
    l.sp_pack_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
    l.sp_pack.argtypes = [_vp, _vp, C.c_int64, C.c_int32, C.c_int32, C.c_int32, _vp, _vp]
    total = l.sp_pack_bytes(n, c, _dt(feats))
    if total < 0:
        raise ValueError("sizes cannot be packed")
    buf = torch.empty(total, dtype=torch.uint8, device=feats.device)
    _check(l.sp_pack(coords.data_ptr() if n else None, feats.data_ptr() if n else None, n, c, _dt(feats), tensor_stride,
                     buf.data_ptr(), _stream()))
    return buf


def sp_unpack(buf: torch.Tensor):
    """Packed buffer -> (coords int32 [n][4], feats [n][c], tensor_stride)."""
    _need_cuda(buf, torch.uint8, "buf")
    l = lib()
    l.sp_unpack_info.argtypes = [_vp, _vp, C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                 C.POINTER(C.c_int32), C.POINTER(C.c_int64)]
    l.sp_unpack.argtypes = [_vp, C.c_int64, C.c_int32, C.c_int32, _vp, _vp, _vp]
    n, c, dt, ts, total = C.c_int64(), C.c_int32(), C.c_int32(), C.c_int32(), C.c_int64()
    if buf.numel() < 256:
        raise ValueError("buffer shorter than a header")
    _check(l.sp_unpack_info(buf.data_ptr(), _stream(), C.byref(n), C.byref(c), C.byref(dt), C.byref(ts), C.byref(total)))
    if total.value > buf.numel():
        raise ValueError("buffer shorter than its header says")
    coords = torch.empty((n.value, 4), dtype=torch.int32, device=buf.device)
    feats = torch.empty((n.value, c.value), dtype=torch.float32 if dt.value == SP_F32 else torch.bfloat16,
                        device=buf.device)
    _check(l.sp_unpack(buf.data_ptr(), n.value, c.value, dt.value, coords.data_ptr() if n.value else None,
                       feats.data_ptr() if n.value else None, _stream()))
    return coords, feats, ts.value


SP_POOL_MAX, SP_POOL_AVG, SP_POOL_SUM = 0, 1, 2
_POOL_MODES = {"max": SP_POOL_MAX, "avg": SP_POOL_AVG, "sum": SP_POOL_SUM}


def sp_pool_fwd(kmap: KMap, x: torch.Tensor, mode: str, want_arg: bool = True):
    """Pooling over the map's neighbour sets.  Returns (y [n_out][c], arg uint8 [n_out][c] or None)."""
    _need_cuda(x, None, "x")
    if x.shape[0] != kmap.n_in:
        raise ValueError("x does not have the map's input rows")
    c = x.shape[1]
    y = torch.empty((kmap.n_out, c), dtype=x.dtype, device=x.device)
    arg = torch.empty((kmap.n_out, c), dtype=torch.uint8, device=x.device) if (mode == "max" and want_arg) else None
    _check(lib().sp_pool_fwd(kmap._h, x.data_ptr() if x.numel() else None, y.data_ptr() if y.numel() else None,
                             arg.data_ptr() if arg is not None and arg.numel() else None, c, _POOL_MODES[mode], _dt(x),
                             _stream()))
    return y, arg


def sp_pool_bwd(kmap: KMap, dy: torch.Tensor, arg, mode: str) -> torch.Tensor:
    _need_cuda(dy, None, "dy")
    if dy.shape[0] != kmap.n_out:
        raise ValueError("dy does not have the map's output rows")
    c = dy.shape[1]
    dx = torch.empty((kmap.n_in, c), dtype=dy.dtype, device=dy.device)
    _check(lib().sp_pool_bwd(kmap._h, dy.data_ptr() if dy.numel() else None,
                             arg.data_ptr() if arg is not None and arg.numel() else None,
                             dx.data_ptr() if dx.numel() else None, c, _POOL_MODES[mode], _dt(dy), _stream()))
    return dx


def sp_pool_trim():
    _check(lib().sp_pool_trim())


def sp_pool_cross_stream() -> int:
    l = lib()
    l.sp_pool_cross_stream.restype = C.c_int64
    return int(l.sp_pool_cross_stream())


_ALLOC_T = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p)
_FREE_T = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)
_allocator_refs = None          # keeps the ctypes callbacks alive while they are installed
allocator_calls = {"alloc": 0, "free": 0}


def sp_set_allocator(alloc=None, free=None):
    """Installs Python callables alloc(nbytes, stream) -> device address (0 on failure) and free(address) as the
    library's device allocator; sp_set_allocator() restores the library's own pool."""
    global _allocator_refs
    l = lib()
    l.sp_set_allocator.argtypes = [_ALLOC_T, _FREE_T, _vp]
    if alloc is None and free is None:
        _check(l.sp_set_allocator(C.cast(None, _ALLOC_T), C.cast(None, _FREE_T), None))
        return

    def _a(nbytes, stream, ctx):
        try:
            allocator_calls["alloc"] += 1
            return int(alloc(int(nbytes), int(stream or 0)))
        except Exception:
            return 0

    def _f(ptr, ctx):
        try:
            allocator_calls["free"] += 1
            free(int(ptr))
        except Exception:
            pass

    refs = (_ALLOC_T(_a), _FREE_T(_f))
    _check(l.sp_set_allocator(refs[0], refs[1], None))
    _allocator_refs = (_allocator_refs, refs)   # earlier callbacks stay alive: blocks taken from them return to them


def use_torch_allocator(enable: bool = True):
    """Routes all of the library's device memory through torch's caching allocator (one allocator owns the
    GPU's memory), or back to the library's own pool."""
    if not enable:
        sp_set_allocator()
        return
    sp_set_allocator(lambda nbytes, stream: torch.cuda.caching_allocator_alloc(nbytes, stream=stream),
                     lambda ptr: torch.cuda.caching_allocator_delete(ptr))


def sp_pool_bytes() -> int:
    return int(lib().sp_pool_bytes())


def sp_conv_kernel_name(kmap: KMap, cin: int, cout: int, dtype: torch.dtype, direction: int = 0) -> str:
    l = lib()
    l.sp_conv_kernel_name.restype = C.c_char_p
    l.sp_conv_kernel_name.argtypes = [_vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    return l.sp_conv_kernel_name(kmap._h, cin, cout, SP_F32 if dtype == torch.float32 else SP_BF16, direction).decode()


def sp_measure_mfma_peak(dtype: torch.dtype) -> float:
    """Measured matrix-core rate (TFLOP/s) of a register-resident MFMA loop in this dtype, on the current stream."""
    out = C.c_double(0.0)
    l = lib()
    l.sp_measure_mfma_peak.argtypes = [C.c_int32, _vp, C.POINTER(C.c_double)]
    _check(l.sp_measure_mfma_peak(SP_F32 if dtype == torch.float32 else SP_BF16, _stream(), C.byref(out)))
    return float(out.value)


def sp_version() -> str:
    return lib().sp_version().decode()


# ---- the layers between sparse convolutions --------------------------------------------------------------
def _glue_argtypes():
    l = lib()
    if getattr(l, "_glue_ready", False):
        return l
    f = C.c_float
    l.sp_bn_relu_fwd.argtypes = [_vp, C.c_int64, C.c_int32, _vp, _vp, f, C.c_int32, _vp, _vp, _vp, C.c_int32, _vp]
    l.sp_bn_relu_bwd.argtypes = [_vp, _vp, _vp, C.c_int64, C.c_int32, _vp, _vp, _vp, C.c_int32, _vp, _vp, _vp,
                                 C.c_int32, _vp]
    l.sp_pool_avg_fwd.argtypes = [_vp, _vp, C.c_int64, C.c_int32, C.c_int32, _vp, _vp, C.c_int32, _vp]
    l.sp_pool_avg_bwd.argtypes = [_vp, _vp, _vp, C.c_int64, C.c_int32, C.c_int32, _vp, C.c_int32, _vp]
    l.sp_linear_fwd.argtypes = [_vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, _vp, _vp]
    l.sp_linear_bwd.argtypes = [_vp, _vp, _vp, C.c_int32, C.c_int32, C.c_int32, _vp, _vp, _vp, _vp]
    l.sp_softmax_ce.argtypes = [_vp, _vp, C.c_int32, C.c_int32, _vp, _vp, _vp]
    l._glue_ready = True
    return l


def _f32(shape, dev):
    return torch.empty(shape, dtype=torch.float32, device=dev)


def sp_bn_relu_fwd(x: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor, eps: float = 1e-5, relu: bool = True):
    """Returns (y, mean, rstd)."""
    _need_cuda(x, None, "x"), _need_cuda(gamma, torch.float32, "gamma"), _need_cuda(beta, torch.float32, "beta")
    n, c = x.shape
    y, mean, rstd = torch.empty_like(x), _f32((c,), x.device), _f32((c,), x.device)
    _check(_glue_argtypes().sp_bn_relu_fwd(x.data_ptr(), n, c, gamma.data_ptr(), beta.data_ptr(), eps, int(relu),
                                           y.data_ptr(), mean.data_ptr(), rstd.data_ptr(), _dt(x), _stream()))
    return y, mean, rstd


def sp_bn_relu_bwd(x, y, dy, gamma, mean, rstd, relu: bool = True):
    """Returns (dx, dgamma, dbeta)."""
    _need_cuda(x, None, "x"), _need_cuda(y, x.dtype, "y"), _need_cuda(dy, x.dtype, "dy")
    n, c = x.shape
    dx, dgamma, dbeta = torch.empty_like(x), _f32((c,), x.device), _f32((c,), x.device)
    _check(_glue_argtypes().sp_bn_relu_bwd(x.data_ptr(), y.data_ptr(), dy.data_ptr(), n, c, gamma.data_ptr(),
                                           mean.data_ptr(), rstd.data_ptr(), int(relu), dx.data_ptr(),
                                           dgamma.data_ptr(), dbeta.data_ptr(), _dt(x), _stream()))
    return dx, dgamma, dbeta


def sp_pool_avg_fwd(coords: torch.Tensor, x: torch.Tensor, n_clouds: int):
    """coords: int32 [n][4] (device).  Returns (pooled fp32 [n_clouds][c], counts fp32 [n_clouds])."""
    _need_cuda(coords, torch.int32, "coords"), _need_cuda(x, None, "x")
    n, c = x.shape
    out, counts = _f32((n_clouds, c), x.device), _f32((n_clouds,), x.device)
    _check(_glue_argtypes().sp_pool_avg_fwd(coords.data_ptr(), x.data_ptr(), n, c, n_clouds, out.data_ptr(),
                                            counts.data_ptr(), _dt(x), _stream()))
    return out, counts


def sp_pool_avg_bwd(coords, dout, counts, n: int, dtype):
    _need_cuda(coords, torch.int32, "coords"), _need_cuda(dout, torch.float32, "dout")
    n_clouds, c = dout.shape
    dx = torch.empty((n, c), dtype=dtype, device=dout.device)
    _check(_glue_argtypes().sp_pool_avg_bwd(coords.data_ptr(), dout.data_ptr(), counts.data_ptr(), n, c, n_clouds,
                                            dx.data_ptr(), _dt(dx), _stream()))
    return dx


def sp_linear_fwd(x, w, bias):
    _need_cuda(x, torch.float32, "x"), _need_cuda(w, torch.float32, "w")
    nb, c = x.shape
    m = w.shape[0]
    out = _f32((nb, m), x.device)
    _check(_glue_argtypes().sp_linear_fwd(x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None,
                                          nb, c, m, out.data_ptr(), _stream()))
    return out


def sp_linear_bwd(x, w, dout):
    """Returns (dx, dw, dbias)."""
    nb, c = x.shape
    m = w.shape[0]
    dx, dw, db = _f32((nb, c), x.device), _f32((m, c), x.device), _f32((m,), x.device)
    _check(_glue_argtypes().sp_linear_bwd(x.data_ptr(), w.data_ptr(), dout.data_ptr(), nb, c, m, dx.data_ptr(),
                                          dw.data_ptr(), db.data_ptr(), _stream()))
    return dx, dw, db


def sp_softmax_ce(logits, labels):
    """labels int32 [n_clouds].  Returns (loss fp32 [1], dlogits)."""
    _need_cuda(logits, torch.float32, "logits"), _need_cuda(labels, torch.int32, "labels")
    nb, m = logits.shape
    loss, d = _f32((1,), logits.device), torch.empty_like(logits)
    _check(_glue_argtypes().sp_softmax_ce(logits.data_ptr(), labels.data_ptr(), nb, m, loss.data_ptr(), d.data_ptr(),
                                          _stream()))
    return loss, d
