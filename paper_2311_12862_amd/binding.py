"""ctypes binding of include/spconv.h: same names, argument marshalling only.

torch is used for device memory and the current HIP stream; every step of the
computation runs inside libspconv.so.

Stream ordering: every call enqueues its work on `stream` (default: torch's
current stream) and returns without waiting.  A tensor that a call returns or
fills is therefore ordered on that stream only: read it on the same stream, or
synchronise that stream first (`tensor.cpu()` runs on torch's current stream).
"""
from __future__ import annotations

import ctypes as C
import os

import torch

OP_FWD, OP_DGRAD, OP_WGRAD = 0, 1, 2
FLAG_SLABS = 1
_DTYPES = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}


class SpconvError(RuntimeError):
    def __init__(self, status: int, where: str):
        lib = load_library()
        msg = lib.spconv_strerror(status).decode()
        hip = lib.spconv_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({status})" + (f" [{hip}]" if status == -6 and hip else ""))
        self.status = status


class Config(C.Structure):
    """Mirror of spconv_config (zero = library defaults)."""
    _fields_ = [("n_split", C.c_int32), ("tile_m", C.c_int32), ("tile_n", C.c_int32),
                ("wgrad_pairs", C.c_int32), ("kernel", C.c_int32), ("flags", C.c_int32), ("reserved", C.c_int32 * 2)]

    def __repr__(self):
        return (f"Config(n_split={self.n_split}, tile_m={self.tile_m}, tile_n={self.tile_n}, "
                f"wgrad_pairs={self.wgrad_pairs}, kernel={self.kernel}" + (f", flags={self.flags}" if self.flags else "") + ")")


class LayerShape(C.Structure):
    """Mirror of spconv_layer_shape."""
    _fields_ = [("c_in", C.c_int32), ("c_out", C.c_int32)]


class LaunchInfo(C.Structure):
    """Mirror of spconv_launch_info."""
    _fields_ = [("kernel", C.c_int32), ("parts", C.c_int32), ("sorted", C.c_int32), ("tile_m", C.c_int32),
                ("tile_n", C.c_int32), ("k_steps", C.c_int32), ("waves", C.c_int32), ("threads", C.c_int32),
                ("grid", C.c_int32 * 3), ("xcd_ranges", C.c_int32), ("lo", C.c_int32 * 4), ("width", C.c_int32 * 4),
                ("lds_bytes", C.c_int64), ("slab_bytes", C.c_int64), ("slab_map_bytes", C.c_int64),
                ("rows_pad", C.c_int64), ("n_tiles", C.c_int64), ("map_elems", C.c_int64 * 4)]


_LIB = None


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libspconv.so")


def load_library():
    """Loads libspconv.so and declares every prototype of include/spconv.h."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2311_12862_amd.build` "
                          "(there is no fallback implementation)")
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    cfgp = C.POINTER(Config)
    protos = {
        "spconv_build_kmap": (i32, [vp, i64, i32, i32, i32, vp, C.POINTER(vp)]),
        "spconv_build_kmap_async": (i32, [vp, i64, i32, i32, i32, vp, C.POINTER(vp)]),
        "spconv_build_kmap_dilated": (i32, [vp, i64, i32, vp, C.POINTER(vp)]),
        "spconv_kmap_status": (i32, [vp, vp]),
        "spconv_kmap_transpose": (i32, [vp, vp, C.POINTER(vp)]),
        "spconv_kmap_pointwise": (i32, [vp, i32, vp, C.POINTER(vp)]),
        "spconv_kmap_sizes": (i32, [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]),
        "spconv_kmap_out_coords": (i32, [vp, vp, vp]),
        "spconv_kmap_in_coords": (i32, [vp, vp, vp]),
        "spconv_kmap_export": (i32, [vp, vp, vp]),
        "spconv_kmap_export_mask": (i32, [vp, vp, vp]),
        "spconv_kmap_prepare": (i32, [vp, i32, cfgp, vp]),
        "spconv_kmap_drop_plans": (i32, [vp]),
        "spconv_kmap_export_perm": (i32, [vp, i32, cfgp, i32, vp, vp]),
        "spconv_kmap_mac_units": (i32, [vp, i32, cfgp, C.POINTER(i64), C.POINTER(i64), vp]),
        "spconv_kmap_destroy": (None, [vp]),
        "spconv_fwd": (i32, [vp, vp, vp, i32, i32, i32, cfgp, vp, vp]),
        "spconv_fwd_noalloc": (i32, [vp, vp, vp, i32, i32, i32, cfgp, vp, vp]),
        "spconv_dgrad": (i32, [vp, vp, vp, i32, i32, i32, cfgp, vp, vp]),
        "spconv_wgrad": (i32, [vp, vp, vp, i32, i32, i32, cfgp, vp, vp]),
        "spconv_tune": (i32, [vp, i32, i32, i32, i32, i32, cfgp, C.POINTER(C.c_float), vp]),
        "spconv_tune_group": (i32, [vp, C.POINTER(LayerShape), i32, i32, i32, i32, cfgp, cfgp, cfgp,
                                    C.POINTER(C.c_float), vp]),
        "spconv_ew": (i32, [i32, vp, vp, vp, i64, i32, vp]),
        "spconv_copy_cols": (i32, [vp, i32, i32, vp, i32, i32, i32, i64, i32, vp]),
        "spconv_set_allocator": (i32, [vp, vp, vp]),
        "spconv_describe_launch": (i32, [i32, i64, i64, i32, i32, i32, cfgp, i32, C.POINTER(LaunchInfo)]),
        "spconv_measure_peaks": (i32, [C.POINTER(C.c_double), C.POINTER(C.c_double), vp]),
        "spconv_strerror": (C.c_char_p, [i32]),
        "spconv_last_hip_error": (C.c_char_p, []),
        "spconv_version": (i32, []),
    }
    for name, (res, args) in protos.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _LIB = lib
    return lib


_ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p)
_FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p, C.c_void_p)
_allocator_refs = None   # keeps the ctypes thunks of the installed callbacks alive


def set_allocator(alloc=None, free=None):
    """spconv_set_allocator: alloc(bytes, stream) -> device address (int, 0 = out of memory) and
    free(address, stream) serve every device allocation the library makes from now on; stream is the
    raw hipStream_t (int, 0 = null stream) of the library call in progress.  (None, None) restores the
    library's own pool.  Switch only while no kmap is alive."""
    global _allocator_refs
    if (alloc is None) != (free is None):
        raise ValueError("give both callbacks or neither")
    lib = load_library()
    if alloc is None:
        _check(lib.spconv_set_allocator(None, None, None), "spconv_set_allocator")
        _allocator_refs = None
        return
    a = _ALLOC_FN(lambda n, stream, _user: int(alloc(int(n), int(stream or 0))) or None)
    f = _FREE_FN(lambda ptr, stream, _user: free(int(ptr or 0), int(stream or 0)))
    _check(lib.spconv_set_allocator(C.cast(a, C.c_void_p), C.cast(f, C.c_void_p), None), "spconv_set_allocator")
    _allocator_refs = (a, f)


def _check(status: int, where: str):
    if status != 0:
        raise SpconvError(status, where)


def _stream(stream):
    """None: torch's current stream; a torch stream; or a raw hipStream_t handle as int (0 = null stream)."""
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _cfg(cfg):
    return None if cfg is None else C.byref(cfg)


def _ptr(t):
    return None if t is None or t.numel() == 0 else t.data_ptr()


def _dev_tensor(t, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return t


class KMap:
    """Owner of an spconv_kmap handle."""

    def __init__(self, handle, K):
        self._h = handle
        self.K = K
        self.V = K ** 3
        n_in, n_out = C.c_int64(), C.c_int64()
        _check(load_library().spconv_kmap_sizes(self._h, C.byref(n_in), C.byref(n_out), None), "spconv_kmap_sizes")
        self.n_in, self.n_out = n_in.value, n_out.value

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("kmap was destroyed")
        return self._h

    def status(self, stream=None):
        """spconv_kmap_status: raises on a range / duplicate error of an asynchronous build."""
        _check(load_library().spconv_kmap_status(self.handle, _stream(stream)), "spconv_kmap_status")

    def transpose(self, stream=None) -> "KMap":
        """spconv_kmap_transpose: the kmap of the paired transposed convolution, derived from this one."""
        h = C.c_void_p()
        _check(load_library().spconv_kmap_transpose(self.handle, _stream(stream), C.byref(h)), "spconv_kmap_transpose")
        return KMap(h, self.K)

    def pointwise(self, on_outputs: bool = False, stream=None) -> "KMap":
        """spconv_kmap_pointwise: the K = 1 kmap over this kmap's input (or output) rows."""
        h = C.c_void_p()
        _check(load_library().spconv_kmap_pointwise(self.handle, int(bool(on_outputs)), _stream(stream), C.byref(h)),
               "spconv_kmap_pointwise")
        return KMap(h, 1)

    def n_pairs(self) -> int:
        v = C.c_int64()
        _check(load_library().spconv_kmap_sizes(self.handle, None, None, C.byref(v)), "spconv_kmap_sizes")
        return v.value

    def out_coords(self, stream=None):
        dst = torch.empty((self.n_out, 4), dtype=torch.int32, device="cuda")
        _check(load_library().spconv_kmap_out_coords(self.handle, _ptr(dst), _stream(stream)), "spconv_kmap_out_coords")
        return dst

    def in_coords(self, stream=None):
        dst = torch.empty((self.n_in, 4), dtype=torch.int32, device="cuda")
        _check(load_library().spconv_kmap_in_coords(self.handle, _ptr(dst), _stream(stream)), "spconv_kmap_in_coords")
        return dst

    def export(self, stream=None):
        dst = torch.empty((self.n_out, self.V), dtype=torch.int32, device="cuda")
        _check(load_library().spconv_kmap_export(self.handle, _ptr(dst), _stream(stream)), "spconv_kmap_export")
        return dst

    def export_mask(self, stream=None):
        # bit patterns of uint32; K = 5: four words per row (bit k of the mask is bit k % 32 of word k // 32)
        shape = (self.n_out, 4) if self.K == 5 else (self.n_out,)
        dst = torch.empty(shape, dtype=torch.int32, device="cuda")
        _check(load_library().spconv_kmap_export_mask(self.handle, _ptr(dst), _stream(stream)), "spconv_kmap_export_mask")
        return dst

    def prepare(self, op, cfg=None, stream=None):
        _check(load_library().spconv_kmap_prepare(self.handle, op, _cfg(cfg), _stream(stream)), "spconv_kmap_prepare")

    def drop_plans(self):
        _check(load_library().spconv_kmap_drop_plans(self.handle), "spconv_kmap_drop_plans")

    def export_perm(self, op, cfg, split, stream=None):
        rows = self.n_out if op == OP_FWD else self.n_in
        dst = torch.empty((rows,), dtype=torch.int32, device="cuda")
        _check(load_library().spconv_kmap_export_perm(self.handle, op, _cfg(cfg), split, _ptr(dst), _stream(stream)),
               "spconv_kmap_export_perm")
        return dst

    def mac_units(self, op, cfg=None, stream=None):
        ex, ef = C.c_int64(), C.c_int64()
        _check(load_library().spconv_kmap_mac_units(self.handle, op, _cfg(cfg), C.byref(ex), C.byref(ef),
                                                    _stream(stream)), "spconv_kmap_mac_units")
        return ex.value, ef.value

    def destroy(self):
        if self._h is not None:
            load_library().spconv_kmap_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def build_kmap(coords, K: int = 3, stride: int = 1, transposed: bool = False, stream=None,
               asynchronous: bool = False, dilate: bool = False) -> KMap:
    """spconv_build_kmap (or spconv_build_kmap_async, or spconv_build_kmap_dilated with dilate=True):
    coords is an int32 device tensor [N, 4] = (b, x, y, z)."""
    _dev_tensor(coords, torch.int32)
    if coords.ndim != 2 or coords.shape[1] != 4:
        raise ValueError("coords must be [N, 4]")
    h = C.c_void_p()
    lib = load_library()
    if dilate:
        if stride != 1 or transposed or asynchronous:
            raise ValueError("dilated kmaps are stride 1, not transposed, built synchronously")
        _check(lib.spconv_build_kmap_dilated(_ptr(coords), coords.shape[0], K, _stream(stream), C.byref(h)),
               "spconv_build_kmap_dilated")
        return KMap(h, K)
    fn, name = (lib.spconv_build_kmap_async, "spconv_build_kmap_async") if asynchronous else \
               (lib.spconv_build_kmap, "spconv_build_kmap")
    _check(fn(_ptr(coords), coords.shape[0], K, stride, int(transposed), _stream(stream), C.byref(h)), name)
    return KMap(h, K)


def _out_tensor(out, shape, dtype, like):
    """A caller-supplied output: exactly the shape, type and device the call writes (the C ABI has
    no row count to catch a wrong one), contiguous."""
    _dev_tensor(out, dtype)
    if tuple(out.shape) != tuple(shape) or out.device != like.device:
        raise SpconvError(-5, f"out is {tuple(out.shape)} on {out.device}, the call writes {tuple(shape)} on {like.device}")
    return out


def _conv_args(a, w_or_b, kmap, rows_a):
    _dev_tensor(a)
    if a.dtype not in _DTYPES:
        raise ValueError(f"unsupported dtype {a.dtype}")
    if a.ndim != 2 or a.shape[0] != rows_a:
        raise SpconvError(-5, f"feature rows {tuple(a.shape)} do not fit the kmap ({rows_a} rows)")
    _dev_tensor(w_or_b, a.dtype)
    return _DTYPES[a.dtype]


def fwd(feats, weights, kmap: KMap, cfg: Config | None = None, out=None, stream=None):
    """spconv_fwd: feats [n_in, C_in], weights [K^3, C_in, C_out] -> out [n_out, C_out]."""
    dt = _conv_args(feats, weights, kmap, kmap.n_in)
    V, c_in, c_out = weights.shape
    if V != kmap.V or c_in != feats.shape[1]:
        raise SpconvError(-5, "weights shape does not fit")
    if out is None:
        out = torch.empty((kmap.n_out, c_out), dtype=feats.dtype, device=feats.device)
    _out_tensor(out, (kmap.n_out, c_out), feats.dtype, feats)
    _check(load_library().spconv_fwd(_ptr(feats), _ptr(weights), kmap.handle, c_in, c_out, dt, _cfg(cfg),
                                     _ptr(out), _stream(stream)), "spconv_fwd")
    return out


def fwd_noalloc(feats, weights, kmap: KMap, out, cfg: Config | None = None, stream=None):
    """spconv_fwd_noalloc: spconv_fwd into the caller's `out` on a prepared plan, without any allocation."""
    dt = _conv_args(feats, weights, kmap, kmap.n_in)
    V, c_in, c_out = weights.shape
    if V != kmap.V or c_in != feats.shape[1]:
        raise SpconvError(-5, "weights shape does not fit")
    _out_tensor(out, (kmap.n_out, c_out), feats.dtype, feats)
    _check(load_library().spconv_fwd_noalloc(_ptr(feats), _ptr(weights), kmap.handle, c_in, c_out, dt, _cfg(cfg),
                                             _ptr(out), _stream(stream)), "spconv_fwd_noalloc")
    return out


def dgrad(dout, weights, kmap: KMap, cfg: Config | None = None, out=None, stream=None):
    """spconv_dgrad: dout [n_out, C_out], weights [K^3, C_in, C_out] -> din [n_in, C_in]."""
    dt = _conv_args(dout, weights, kmap, kmap.n_out)
    V, c_in, c_out = weights.shape
    if V != kmap.V or c_out != dout.shape[1]:
        raise SpconvError(-5, "weights shape does not fit")
    if out is None:
        out = torch.empty((kmap.n_in, c_in), dtype=dout.dtype, device=dout.device)
    _out_tensor(out, (kmap.n_in, c_in), dout.dtype, dout)
    _check(load_library().spconv_dgrad(_ptr(dout), _ptr(weights), kmap.handle, c_in, c_out, dt, _cfg(cfg),
                                       _ptr(out), _stream(stream)), "spconv_dgrad")
    return out


def wgrad(feats, dout, kmap: KMap, cfg: Config | None = None, out=None, stream=None):
    """spconv_wgrad: feats [n_in, C_in], dout [n_out, C_out] -> dweights fp32 [K^3, C_in, C_out]."""
    dt = _conv_args(feats, dout, kmap, kmap.n_in)
    if dout.ndim != 2 or dout.shape[0] != kmap.n_out:
        raise SpconvError(-5, "dout rows do not fit the kmap")
    c_in, c_out = feats.shape[1], dout.shape[1]
    if out is None:
        out = torch.empty((kmap.V, c_in, c_out), dtype=torch.float32, device=feats.device)
    _out_tensor(out, (kmap.V, c_in, c_out), torch.float32, feats)
    _check(load_library().spconv_wgrad(_ptr(feats), _ptr(dout), kmap.handle, c_in, c_out, dt, _cfg(cfg),
                                       _ptr(out), _stream(stream)), "spconv_wgrad")
    return out


def tune(kmap: KMap, c_in: int, c_out: int, dtype, op: int, layers_sharing_kmap: int = 1, stream=None):
    """spconv_tune: returns (Config, microseconds)."""
    best, us = Config(), C.c_float()
    _check(load_library().spconv_tune(kmap.handle, c_in, c_out, _DTYPES[dtype], op, layers_sharing_kmap,
                                      C.byref(best), C.byref(us), _stream(stream)), "spconv_tune")
    return best, us.value


def tune_group(kmap: KMap, layers, dtype, training: bool = False, bind_fwd_dgrad: bool = True, stream=None):
    """spconv_tune_group: layers is a sequence of (c_in, c_out) of the layers that run on kmap.
    Returns (fwd, dgrad, wgrad, microseconds): lists of Config, one per layer (dgrad and wgrad are
    None for training=False)."""
    n = len(layers)
    shapes = (LayerShape * n)(*[LayerShape(int(ci), int(co)) for ci, co in layers])
    fwd = (Config * n)()
    dg = (Config * n)() if training else None
    wg = (Config * n)() if training else None
    us = C.c_float()
    _check(load_library().spconv_tune_group(kmap.handle, shapes, n, _DTYPES[dtype], int(training), int(bind_fwd_dgrad),
                                            fwd, dg, wg, C.byref(us), _stream(stream)), "spconv_tune_group")
    copy = lambda arr: None if arr is None else [Config.from_buffer_copy(c) for c in arr]
    return copy(fwd), copy(dg), copy(wg), us.value


def describe_launch(K: int, rows: int, rows_src: int, c_red: int, c_cols: int, dtype, cfg: Config | None = None,
                    dgrad: bool = False) -> LaunchInfo:
    """spconv_describe_launch: the launch geometry of a forward / dgrad call (host arithmetic; needs no GPU)."""
    info = LaunchInfo()
    _check(load_library().spconv_describe_launch(K, rows, rows_src, c_red, c_cols, _DTYPES[dtype], _cfg(cfg), int(dgrad),
                                                 C.byref(info)), "spconv_describe_launch")
    return info


def measure_peaks(stream=None):
    """spconv_measure_peaks: (streaming-copy GB/s, fp16 MFMA TFLOP/s) measured on the current device."""
    hbm, mfma = C.c_double(), C.c_double()
    _check(load_library().spconv_measure_peaks(C.byref(hbm), C.byref(mfma), _stream(stream)), "spconv_measure_peaks")
    return hbm.value, mfma.value


EW_RELU, EW_ADD, EW_ADD_RELU, EW_RELU_BWD = 0, 1, 2, 3


def ew(op: int, a, b=None, out=None, stream=None):
    """spconv_ew: element-wise glue (see include/spconv.h); out defaults to a new tensor like a."""
    _dev_tensor(a)
    if b is not None:
        _dev_tensor(b, a.dtype)
        if b.shape != a.shape:
            raise ValueError("shape mismatch")
    if out is None:
        out = torch.empty_like(a)
    _check(load_library().spconv_ew(op, _ptr(a), _ptr(b), _ptr(out), a.numel(), _DTYPES[a.dtype], _stream(stream)),
           "spconv_ew")
    return out


def copy_cols(src, src_off: int, dst, dst_off: int, cols: int, stream=None):
    """spconv_copy_cols on two [rows, ld] tensors."""
    _dev_tensor(src)
    _dev_tensor(dst, src.dtype)
    if src.shape[0] != dst.shape[0]:
        raise ValueError("row mismatch")
    _check(load_library().spconv_copy_cols(_ptr(src), src.shape[1], src_off, _ptr(dst), dst.shape[1], dst_off, cols,
                                           src.shape[0], _DTYPES[src.dtype], _stream(stream)), "spconv_copy_cols")
    return dst
