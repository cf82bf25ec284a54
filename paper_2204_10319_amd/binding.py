"""ctypes binding of libts.so: argument marshalling only, same names as ``include/ts.h``.

PyTorch supplies device memory (tensors) and the stream; every step of the layer runs in
the library's HIP kernels.  There is no fallback: if ``libts.so`` has not been built or
cannot be loaded, the first call raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

TS_F32, TS_F16 = 0, 1
TS_DATAFLOW_AUTO, TS_DATAFLOW_EXPLICIT, TS_DATAFLOW_FUSED, TS_DATAFLOW_FUSED_STAGED, TS_DATAFLOW_FETCH = 0, 1, 2, 3, 4

TS_OK = 0
TS_ERR_INVALID_ARG, TS_ERR_SHAPE, TS_ERR_COORD_RANGE, TS_ERR_DUPLICATE_COORD = -1, -2, -3, -4
TS_ERR_OOM, TS_ERR_HIP, TS_ERR_UNSUPPORTED = -5, -6, -7

TS_BATCH_MAX, TS_COORD_MIN, TS_COORD_MAX = 8190, -65528, 65527

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libts.so")
_lib = None

EXPORTS = [
    "ts_build_kmap", "ts_build_kmap_async", "ts_build_kmap_ex", "ts_identity_kmap", "ts_kmap_status", "ts_kmap_prepare", "ts_free", "ts_kmap_sort_rows", "ts_kmap_transpose", "ts_kmap_num_in", "ts_kmap_num_out", "ts_kmap_num_pairs",
    "ts_kmap_kernel_volume", "ts_kmap_out_coords", "ts_kmap_out_box", "ts_kmap_in_coords", "ts_kmap_sizes", "ts_kmap_pairs",
    "ts_sparse_conv", "ts_sparse_conv_ex", "ts_sparse_conv_static", "ts_sparse_conv_act", "ts_weights_prepare", "ts_weights_free",
    "ts_sparse_conv_prepared", "ts_sparse_conv_prepared2", "ts_gather", "ts_gather_ex", "ts_grouped_matmul", "ts_scatter_reduce", "ts_adaptive_groups", "ts_grouped_matmul_adaptive",
    "ts_set_stream", "ts_set_allocator", "ts_release_cache", "ts_last_error", "ts_version", "ts_profile_enable", "ts_profile_read", "ts_copy_bytes", "ts_mfma_loop", "ts_bias_act", "ts_concat_cols",
]


TS_SEARCH_AUTO, TS_SEARCH_HASH, TS_SEARCH_GRID = 0, 1, 2


class KMapOptions(ctypes.Structure):
    """ts_kmap_options of the header."""
    _fields_ = [("search", ctypes.c_int32), ("wait", ctypes.c_int32), ("has_boundary", ctypes.c_int32),
                ("boundary", ctypes.c_int32 * 3), ("grid_lo", ctypes.c_int32 * 3), ("grid_hi", ctypes.c_int32 * 3),
                ("grid_batches", ctypes.c_int32)]


class TsError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libts error {code}: {message}")
        self.code = code


class ts_tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


def load_library(path: str | None = None):
    """Load libts.so and declare the signatures of ``include/ts.h``."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or _LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(f"{p} is missing: build it with `python -m paper_2204_10319_amd.build` "
                           "(there is no CPU fallback)")
    lib = ctypes.CDLL(p)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    tp = ctypes.POINTER(ts_tensor)
    lib.ts_build_kmap.argtypes = [vp, i64, ci, ci, ci, ctypes.POINTER(vp)]
    lib.ts_build_kmap.restype = ci
    lib.ts_build_kmap_async.argtypes = [vp, i64, ci, ci, ci, ctypes.POINTER(vp)]
    lib.ts_build_kmap_async.restype = ci
    lib.ts_kmap_prepare.argtypes = [vp]
    lib.ts_kmap_prepare.restype = ci
    lib.ts_build_kmap_ex.argtypes = [vp, i64, ci, ci, ci, ctypes.POINTER(KMapOptions), ctypes.POINTER(vp)]
    lib.ts_build_kmap_ex.restype = ci
    lib.ts_kmap_status.argtypes = [vp]
    lib.ts_kmap_status.restype = ci
    lib.ts_free.argtypes = [vp]
    lib.ts_free.restype = None
    lib.ts_kmap_sort_rows.argtypes = [vp]
    lib.ts_kmap_sort_rows.restype = ci
    lib.ts_kmap_transpose.argtypes = [vp, ctypes.POINTER(vp)]
    lib.ts_kmap_transpose.restype = ci
    lib.ts_identity_kmap.argtypes = [i64, ctypes.POINTER(vp)]
    lib.ts_identity_kmap.restype = ci
    for name in ("ts_kmap_num_in", "ts_kmap_num_out", "ts_kmap_num_pairs"):
        getattr(lib, name).argtypes = [vp]
        getattr(lib, name).restype = i64
    lib.ts_kmap_kernel_volume.argtypes = [vp]
    lib.ts_kmap_kernel_volume.restype = ci
    lib.ts_kmap_out_coords.argtypes = [vp, vp]
    lib.ts_kmap_in_coords.argtypes = [vp, vp]
    lib.ts_kmap_out_box.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    lib.ts_kmap_out_box.restype = ci
    lib.ts_kmap_sizes.argtypes = [vp, ctypes.POINTER(i64)]
    lib.ts_kmap_pairs.argtypes = [vp, vp, vp]
    lib.ts_sparse_conv.argtypes = [tp, tp, vp, tp]
    lib.ts_sparse_conv_ex.argtypes = [tp, tp, vp, tp, ci]
    lib.ts_sparse_conv_static.argtypes = [tp, tp, vp, tp]
    lib.ts_sparse_conv_static.restype = ci
    lib.ts_sparse_conv_act.argtypes = [tp, tp, vp, vp, tp, ci, tp]
    lib.ts_sparse_conv_act.restype = ci
    lib.ts_weights_prepare.argtypes = [tp, ci, ctypes.POINTER(vp)]
    lib.ts_weights_prepare.restype = ci
    lib.ts_weights_free.argtypes = [vp]
    lib.ts_weights_free.restype = None
    lib.ts_sparse_conv_prepared.argtypes = [tp, vp, vp, vp, tp, ci, tp]
    lib.ts_sparse_conv_prepared.restype = ci
    lib.ts_sparse_conv_prepared2.argtypes = [tp, tp, vp, vp, vp, tp, ci, tp]
    lib.ts_sparse_conv_prepared2.restype = ci
    lib.ts_gather.argtypes = [tp, vp, tp]
    lib.ts_gather_ex.argtypes = [tp, vp, tp, ci]
    lib.ts_gather_ex.restype = ci
    lib.ts_grouped_matmul.argtypes = [tp, tp, tp, vp, tp]
    lib.ts_scatter_reduce.argtypes = [tp, vp, tp]
    lib.ts_adaptive_groups.argtypes = [ctypes.POINTER(ctypes.c_int64), ctypes.c_int32, ctypes.c_double,
                                       ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    lib.ts_adaptive_groups.restype = ci
    lib.ts_grouped_matmul_adaptive.argtypes = [tp, tp, tp, vp, ctypes.c_double, ctypes.c_int64, tp,
                                               ctypes.POINTER(ctypes.c_int64)]
    lib.ts_grouped_matmul_adaptive.restype = ci
    lib.ts_set_stream.argtypes = [vp]
    lib.ts_set_allocator.argtypes = [vp, vp, vp]
    lib.ts_set_allocator.restype = ci
    lib.ts_release_cache.argtypes = []
    for name in ("ts_kmap_out_coords", "ts_kmap_out_box", "ts_kmap_in_coords", "ts_kmap_sizes", "ts_kmap_pairs", "ts_sparse_conv",
                 "ts_sparse_conv_ex", "ts_gather", "ts_grouped_matmul", "ts_scatter_reduce", "ts_set_stream",
                 "ts_release_cache"):
        getattr(lib, name).restype = ci
    lib.ts_bias_act.argtypes = [tp, vp, tp, ci, tp]
    lib.ts_bias_act.restype = ci
    lib.ts_concat_cols.argtypes = [tp, tp, tp]
    lib.ts_concat_cols.restype = ci
    lib.ts_copy_bytes.argtypes = [vp, vp, ctypes.c_size_t]
    lib.ts_copy_bytes.restype = ci
    lib.ts_mfma_loop.argtypes = [ci, vp, ctypes.POINTER(ctypes.c_double)]
    lib.ts_mfma_loop.restype = ci
    lib.ts_profile_enable.argtypes = [ci, ctypes.c_char_p]
    lib.ts_profile_enable.restype = ci
    lib.ts_profile_read.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
    lib.ts_profile_read.restype = ci
    lib.ts_last_error.argtypes = []
    lib.ts_last_error.restype = ctypes.c_char_p
    lib.ts_version.argtypes = []
    lib.ts_version.restype = ctypes.c_char_p
    if path is None:
        _lib = lib
    return lib


def _check(rc: int):
    if rc != TS_OK:
        raise TsError(rc, load_library().ts_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return TS_F16
    if t.dtype == torch.float32:
        return TS_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _as_ts(t: torch.Tensor, rows: int | None = None, cols: int | None = None) -> ts_tensor:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    r = t.shape[0] if rows is None else rows
    c = t.shape[-1] if cols is None else cols
    return ts_tensor(t.data_ptr() if t.numel() else None, r, c, _dtype_code(t))


def _use_current_stream():
    _check(load_library().ts_set_stream(torch.cuda.current_stream().cuda_stream))


def ts_set_stream(stream: torch.cuda.Stream | None):
    _check(load_library().ts_set_stream(stream.cuda_stream if stream is not None else None))


def ts_mfma_loop(iters: int, sink: torch.Tensor) -> float:
    """Runs the register-only MFMA loop once; returns the FLOPs it executes (time it with ts_profile_enable)."""
    _use_current_stream()
    if not sink.is_cuda or sink.numel() * sink.element_size() < (1 << 20):
        raise ValueError("sink must be a device tensor of at least 1 MiB")
    flops = ctypes.c_double(0.0)
    _check(load_library().ts_mfma_loop(int(iters), sink.data_ptr(), ctypes.byref(flops)))
    return flops.value


def ts_release_cache():
    _check(load_library().ts_release_cache())


def ts_version() -> str:
    return load_library().ts_version().decode()


def ts_bias_act(x: torch.Tensor, bias: torch.Tensor | None = None, residual: torch.Tensor | None = None,
                relu: bool = True, out: torch.Tensor | None = None) -> torch.Tensor:
    """out = act(x + bias + residual) with per-channel bias; fp32 arithmetic, dtype of x."""
    _use_current_stream()
    if out is None:
        out = torch.empty_like(x)
    if bias is not None and (bias.dtype != x.dtype or bias.numel() != x.shape[1] or not bias.is_cuda):
        raise ValueError("bias must be a device vector [cols] of the dtype of x")
    xs, os_ = _as_ts(x), _as_ts(out)
    rs = ctypes.byref(_as_ts(residual)) if residual is not None else None
    _check(load_library().ts_bias_act(ctypes.byref(xs), bias.data_ptr() if bias is not None else None, rs,
                                      int(bool(relu)), ctypes.byref(os_)))
    return out


def ts_concat_cols(a: torch.Tensor, b: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    _use_current_stream()
    if out is None:
        out = torch.empty((a.shape[0], a.shape[1] + b.shape[1]), dtype=a.dtype, device=a.device)
    at, bt, ot = _as_ts(a), _as_ts(b), _as_ts(out)
    _check(load_library().ts_concat_cols(ctypes.byref(at), ctypes.byref(bt), ctypes.byref(ot)))
    return out


def ts_copy_bytes(dst: torch.Tensor, src: torch.Tensor):
    """Plain streaming copy of src into dst (same byte size), for bandwidth reference/calibration."""
    _use_current_stream()
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    _check(load_library().ts_copy_bytes(dst.data_ptr(), src.data_ptr(), nbytes))


def ts_profile_enable(on: bool, only: str | None = None):
    _check(load_library().ts_profile_enable(int(bool(on)), only.encode() if only else None))


def ts_profile_read() -> dict:
    """{kernel name: (launches, total_ms)} since the last read; synchronises the stream."""
    _use_current_stream()
    buf = ctypes.create_string_buffer(1 << 16)
    _check(load_library().ts_profile_read(buf, len(buf)))
    out = {}
    for line in buf.value.decode().splitlines():
        name, count, ms = line.split()
        out[name] = (int(count), float(ms))
    return out


class KMap:
    """Owner of a ``ts_kmap*``; freed by :func:`ts_free` or on garbage collection."""

    def __init__(self, handle: int):
        self._h = handle

    @property
    def handle(self):
        if not self._h:
            raise ValueError("kernel map already freed")
        return self._h

    num_in = property(lambda self: load_library().ts_kmap_num_in(self.handle))
    num_out = property(lambda self: load_library().ts_kmap_num_out(self.handle))
    num_pairs = property(lambda self: load_library().ts_kmap_num_pairs(self.handle))
    kernel_volume = property(lambda self: load_library().ts_kmap_kernel_volume(self.handle))

    def out_coords(self) -> torch.Tensor:
        return ts_kmap_out_coords(self)

    def in_coords(self) -> torch.Tensor:
        return ts_kmap_in_coords(self)

    def out_box(self):
        """(lo[3], hi[3], batches) holding every output coordinate, or None when the build bounded nothing."""
        lo, hi, b = (ctypes.c_int32 * 3)(), (ctypes.c_int32 * 3)(), ctypes.c_int32()
        rc = load_library().ts_kmap_out_box(self.handle, lo, hi, ctypes.byref(b))
        if rc == TS_ERR_UNSUPPORTED:
            return None
        _check(rc)
        return tuple(lo), tuple(hi), int(b.value)

    def sizes(self) -> np.ndarray:
        return ts_kmap_sizes(self)

    def pairs(self):
        return ts_kmap_pairs(self)

    def status(self):
        """Waits for an asynchronous build's verdict; raises TsError if the input was bad."""
        _check(load_library().ts_kmap_status(self.handle))
        return self

    def prepare(self):
        """Enqueues, without waiting, what an asynchronous build put off (ts_kmap_prepare)."""
        _use_current_stream()
        _check(load_library().ts_kmap_prepare(self.handle))
        return self

    def transpose(self) -> "KMap":
        return ts_kmap_transpose(self)

    def sort_rows(self):
        ts_kmap_sort_rows(self)
        return self

    def free(self):
        if self._h:
            load_library().ts_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def ts_build_kmap(coords: torch.Tensor, kernel_size: int, stride: int = 1, transposed: bool = False,
                  wait: bool = True, grid=None, boundary=None, search: int = TS_SEARCH_AUTO, box=None) -> KMap:
    """coords: device int32 [N,4] (batch, x, y, z).  wait=False: ts_build_kmap_async (errors of the input
    surface at ``KMap.status()`` or the first accessor that needs the map's sizes).
    grid=(lo[3], hi[3], batches): search through the coordinate grid over that box (ts_build_kmap_ex,
    TS_SEARCH_GRID).  search=TS_SEARCH_HASH keeps a strided build on the hash table.  boundary=(bx, by, bz): Alg. 3's boundary check for a strided map.
    box=(lo[3], hi[3], batches): a box holding the coordinates, stated so that a strided build on the default route
    need not measure one (ignored at stride 1)."""
    if coords.dtype != torch.int32 or coords.dim() != 2 or coords.shape[1] != 4:
        raise ValueError("coords must be int32 [N,4]")
    if not coords.is_cuda or not coords.is_contiguous():
        raise ValueError("coords must be a contiguous device tensor")
    _use_current_stream()
    h = ctypes.c_void_p()
    if grid is not None or boundary is not None or search != TS_SEARCH_AUTO or box is not None:
        opt = KMapOptions()
        opt.wait = int(bool(wait))
        opt.search = int(search)
        if box is not None and grid is None:
            lo, hi, batches = box
            opt.grid_lo = (ctypes.c_int32 * 3)(*[int(v) for v in lo])
            opt.grid_hi = (ctypes.c_int32 * 3)(*[int(v) for v in hi])
            opt.grid_batches = int(batches)
        if grid is not None:
            lo, hi, batches = grid
            opt.search = TS_SEARCH_GRID
            opt.grid_lo = (ctypes.c_int32 * 3)(*[int(v) for v in lo])
            opt.grid_hi = (ctypes.c_int32 * 3)(*[int(v) for v in hi])
            opt.grid_batches = int(batches)
        if boundary is not None:
            opt.has_boundary = 1
            opt.boundary = (ctypes.c_int32 * 3)(*[int(v) for v in boundary])
        rc = load_library().ts_build_kmap_ex(coords.data_ptr() if coords.numel() else None, coords.shape[0],
                                             int(kernel_size), int(stride), int(bool(transposed)), ctypes.byref(opt),
                                             ctypes.byref(h))
        _check(rc)
        return KMap(h.value)
    fn = load_library().ts_build_kmap if wait else load_library().ts_build_kmap_async
    rc = fn(coords.data_ptr() if coords.numel() else None, coords.shape[0], int(kernel_size), int(stride),
            int(bool(transposed)), ctypes.byref(h))
    _check(rc)
    return KMap(h.value)


def ts_identity_kmap(n: int) -> KMap:
    """The map of a 1x1x1, stride-1 convolution over n distinct points (output k <- input k); holds no coordinates."""
    _use_current_stream()
    handle = ctypes.c_void_p()
    _check(load_library().ts_identity_kmap(int(n), ctypes.byref(handle)))
    return KMap(handle.value)


def ts_kmap_transpose(forward: KMap) -> KMap:
    """The transposed map of a forward strided map, derived without another search."""
    _use_current_stream()
    handle = ctypes.c_void_p()
    _check(load_library().ts_kmap_transpose(forward.handle, ctypes.byref(handle)))
    return KMap(handle.value)


def ts_kmap_sort_rows(kmap: KMap):
    """Optional: order the map's output rows by offset bitmask (worth it for maps that serve several layers)."""
    _use_current_stream()
    _check(load_library().ts_kmap_sort_rows(kmap.handle))


def ts_free(kmap: KMap):
    kmap.free()


def ts_kmap_out_coords(kmap: KMap) -> torch.Tensor:
    _use_current_stream()
    dst = torch.empty((kmap.num_out, 4), dtype=torch.int32, device="cuda")
    _check(load_library().ts_kmap_out_coords(kmap.handle, dst.data_ptr() if dst.numel() else None))
    return dst


def ts_kmap_in_coords(kmap: KMap) -> torch.Tensor:
    _use_current_stream()
    dst = torch.empty((kmap.num_in, 4), dtype=torch.int32, device="cuda")
    _check(load_library().ts_kmap_in_coords(kmap.handle, dst.data_ptr() if dst.numel() else None))
    return dst


def ts_kmap_sizes(kmap: KMap) -> np.ndarray:
    dst = (ctypes.c_int64 * kmap.kernel_volume)()
    _check(load_library().ts_kmap_sizes(kmap.handle, dst))
    return np.array(list(dst), dtype=np.int64)


def ts_kmap_pairs(kmap: KMap):
    """(in_idx, out_idx): device int32 [num_pairs] each, offset-major."""
    _use_current_stream()
    m = kmap.num_pairs
    a = torch.empty((m,), dtype=torch.int32, device="cuda")
    b = torch.empty((m,), dtype=torch.int32, device="cuda")
    _check(load_library().ts_kmap_pairs(kmap.handle, a.data_ptr() if m else None, b.data_ptr() if m else None))
    return a, b


def _weights_ts(weights: torch.Tensor) -> ts_tensor:
    if weights.dim() != 3:
        raise ValueError("weights must be [K^3, C_in, C_out]")
    return _as_ts(weights, rows=weights.shape[0] * weights.shape[1], cols=weights.shape[2])


def ts_sparse_conv(feats: torch.Tensor, weights: torch.Tensor, kmap: KMap, out: torch.Tensor | None = None,
                   dataflow: int = TS_DATAFLOW_AUTO) -> torch.Tensor:
    """feats [num_in, C_in], weights [K^3, C_in, C_out] -> out [num_out, C_out] (same dtype)."""
    _use_current_stream()
    if out is None:
        out = torch.empty((kmap.num_out, weights.shape[2]), dtype=feats.dtype, device=feats.device)
    f, w, o = _as_ts(feats), _weights_ts(weights), _as_ts(out)
    lib = load_library()
    if dataflow == TS_DATAFLOW_AUTO:
        rc = lib.ts_sparse_conv(ctypes.byref(f), ctypes.byref(w), kmap.handle, ctypes.byref(o))
    else:
        rc = lib.ts_sparse_conv_ex(ctypes.byref(f), ctypes.byref(w), kmap.handle, ctypes.byref(o), int(dataflow))
    _check(rc)
    return out


def ts_sparse_conv_static(feats: torch.Tensor, weights: torch.Tensor, kmap: KMap, out: torch.Tensor) -> torch.Tensor:
    """ts_sparse_conv for callers that cannot allocate: ``out`` is required, and neither this wrapper nor the
    library allocates device memory (the library's staging area is a fixed array inside libts.so)."""
    _use_current_stream()
    f, w, o = _as_ts(feats), _weights_ts(weights), _as_ts(out)
    _check(load_library().ts_sparse_conv_static(ctypes.byref(f), ctypes.byref(w), kmap.handle, ctypes.byref(o)))
    return out


def ts_sparse_conv_act(feats: torch.Tensor, weights: torch.Tensor, kmap: KMap, bias: torch.Tensor | None = None,
                       residual: torch.Tensor | None = None, relu: bool = True,
                       out: torch.Tensor | None = None) -> torch.Tensor:
    """out = act(conv(feats) + bias + residual) in one call (fused epilogue for fp16)."""
    _use_current_stream()
    c_out = weights.shape[-1]
    if out is None:
        out = torch.empty((kmap.num_out, c_out), dtype=feats.dtype, device=feats.device)
    f, w, o = _as_ts(feats), _weights_ts(weights), _as_ts(out)
    r = _as_ts(residual) if residual is not None else None
    _check(load_library().ts_sparse_conv_act(ctypes.byref(f), ctypes.byref(w), kmap.handle,
                                             bias.data_ptr() if bias is not None else None,
                                             ctypes.byref(r) if r is not None else None, int(bool(relu)),
                                             ctypes.byref(o)))
    return out


class Weights:
    """Prepared weights of one layer (owned by the library until ``free`` / garbage collection)."""

    def __init__(self, handle: int, c_in: int, c_out: int, dtype: torch.dtype, device):
        self._h, self.c_in, self.c_out, self.dtype, self.device = handle, c_in, c_out, dtype, device

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("weights already freed")
        return self._h

    def free(self):
        if self._h is not None:
            load_library().ts_weights_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def ts_weights_prepare(weights: torch.Tensor) -> Weights:
    """weights [K^3, C_in, C_out] -> the same, repacked once for the layer kernels."""
    _use_current_stream()
    w = _weights_ts(weights)
    handle = ctypes.c_void_p()
    _check(load_library().ts_weights_prepare(ctypes.byref(w), int(weights.shape[0]), ctypes.byref(handle)))
    return Weights(handle.value, weights.shape[1], weights.shape[2], weights.dtype, weights.device)


def ts_sparse_conv_prepared(feats: torch.Tensor, weights: Weights, kmap: KMap, bias: torch.Tensor | None = None,
                            residual: torch.Tensor | None = None, relu: bool = False,
                            out: torch.Tensor | None = None) -> torch.Tensor:
    """ts_sparse_conv_act with weights from ts_weights_prepare."""
    _use_current_stream()
    if out is None:
        out = torch.empty((kmap.num_out, weights.c_out), dtype=feats.dtype, device=feats.device)
    f, o = _as_ts(feats), _as_ts(out)
    r = _as_ts(residual) if residual is not None else None
    _check(load_library().ts_sparse_conv_prepared(ctypes.byref(f), weights.handle, kmap.handle,
                                                  bias.data_ptr() if bias is not None else None,
                                                  ctypes.byref(r) if r is not None else None, int(bool(relu)),
                                                  ctypes.byref(o)))
    return out


def ts_sparse_conv_prepared2(feats: torch.Tensor, feats2: torch.Tensor | None, weights: Weights, kmap: KMap,
                             bias: torch.Tensor | None = None, residual: torch.Tensor | None = None,
                             relu: bool = False, out: torch.Tensor | None = None) -> torch.Tensor:
    """ts_sparse_conv_prepared on the channel concatenation [feats | feats2], which is never formed."""
    _use_current_stream()
    if out is None:
        out = torch.empty((kmap.num_out, weights.c_out), dtype=feats.dtype, device=feats.device)
    f, o = _as_ts(feats), _as_ts(out)
    f2 = _as_ts(feats2) if feats2 is not None else None
    r = _as_ts(residual) if residual is not None else None
    _check(load_library().ts_sparse_conv_prepared2(ctypes.byref(f), ctypes.byref(f2) if f2 is not None else None,
                                                   weights.handle, kmap.handle,
                                                   bias.data_ptr() if bias is not None else None,
                                                   ctypes.byref(r) if r is not None else None, int(bool(relu)),
                                                   ctypes.byref(o)))
    return out


_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_RELEASE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)
_allocator_refs = None      # keeps the callbacks alive while the library may call them


def ts_set_allocator(alloc=None, release=None):
    """``alloc(bytes) -> device address (int) or 0`` and ``release(address)``; both None: the library's own pool."""
    global _allocator_refs
    lib = load_library()
    if alloc is None and release is None:
        _check(lib.ts_set_allocator(None, None, None))
        return
    a = _ALLOC_FN(lambda n, ctx: alloc(n) or 0)
    r = _RELEASE_FN(lambda p, ctx: release(p))
    keep = (_allocator_refs, a, r)      # earlier callbacks stay alive: blocks they handed out may still come back
    _check(lib.ts_set_allocator(ctypes.cast(a, ctypes.c_void_p), ctypes.cast(r, ctypes.c_void_p), None))
    _allocator_refs = keep


def use_torch_allocator(on: bool = True):
    """Route the library's device memory through PyTorch's caching allocator (on the current stream)."""
    if not on:
        ts_set_allocator(None, None)
        return
    ts_set_allocator(lambda n: torch.cuda.caching_allocator_alloc(n), lambda p: torch.cuda.caching_allocator_delete(p))


def ts_sparse_conv_ex(feats, weights, kmap, out=None, dataflow: int = TS_DATAFLOW_AUTO):
    return ts_sparse_conv(feats, weights, kmap, out, dataflow)


TS_GATHER_AUTO, TS_GATHER_OUTPUT_ORDER, TS_GATHER_INPUT_STATIONARY = 0, 1, 2


def ts_gather(feats: torch.Tensor, kmap: KMap, F: torch.Tensor | None = None, order: int = TS_GATHER_AUTO) -> torch.Tensor:
    _use_current_stream()
    if F is None:
        F = torch.zeros((kmap.num_pairs, feats.shape[1]), dtype=feats.dtype, device=feats.device)
    f, b = _as_ts(feats), _as_ts(F)
    if order == TS_GATHER_AUTO:
        _check(load_library().ts_gather(ctypes.byref(f), kmap.handle, ctypes.byref(b)))
    else:
        _check(load_library().ts_gather_ex(ctypes.byref(f), kmap.handle, ctypes.byref(b), int(order)))
    return F


def ts_grouped_matmul(F: torch.Tensor, feats: torch.Tensor | None, weights: torch.Tensor, kmap: KMap,
                      G: torch.Tensor | None = None) -> torch.Tensor:
    _use_current_stream()
    if G is None:
        G = torch.empty((kmap.num_pairs, weights.shape[2]), dtype=torch.float32, device=F.device)
    a, w, g = _as_ts(F), _weights_ts(weights), _as_ts(G)
    x = ctypes.byref(_as_ts(feats)) if feats is not None else None
    _check(load_library().ts_grouped_matmul(ctypes.byref(a), x, ctypes.byref(w), kmap.handle, ctypes.byref(g)))
    return G


def ts_adaptive_groups(sizes, epsilon: float) -> list[int]:
    """Group number of every weight index (Appendix B, Alg. 4, first loop); host arithmetic only."""
    sizes = [int(v) for v in sizes]
    n = len(sizes)
    arr = (ctypes.c_int64 * max(n, 1))(*sizes)
    group_of = (ctypes.c_int32 * max(n, 1))()
    groups = ctypes.c_int32(0)
    _check(load_library().ts_adaptive_groups(arr, n, float(epsilon), group_of, ctypes.byref(groups)))
    return list(group_of[:n])


def ts_grouped_matmul_adaptive(F: torch.Tensor, feats: torch.Tensor | None, weights: torch.Tensor, kmap: KMap,
                               epsilon: float, S: int, G: torch.Tensor | None = None):
    """Returns (G, stats) with stats = dict(launches, groups, padded_rows, rows)."""
    _use_current_stream()
    if G is None:
        G = torch.empty((kmap.num_pairs, weights.shape[2]), dtype=torch.float32, device=F.device)
    a, w, g = _as_ts(F), _weights_ts(weights), _as_ts(G)
    x = ctypes.byref(_as_ts(feats)) if feats is not None else None
    stats = (ctypes.c_int64 * 4)()
    _check(load_library().ts_grouped_matmul_adaptive(ctypes.byref(a), x, ctypes.byref(w), kmap.handle,
                                                     float(epsilon), int(S), ctypes.byref(g), stats))
    return G, dict(launches=stats[0], groups=stats[1], padded_rows=stats[2], rows=stats[3])


def ts_scatter_reduce(G: torch.Tensor, kmap: KMap, out: torch.Tensor | None = None,
                      dtype: torch.dtype = torch.float16) -> torch.Tensor:
    _use_current_stream()
    if out is None:
        out = torch.empty((kmap.num_out, G.shape[1]), dtype=dtype, device=G.device)
    g, o = _as_ts(G), _as_ts(out)
    _check(load_library().ts_scatter_reduce(ctypes.byref(g), kmap.handle, ctypes.byref(o)))
    return out
