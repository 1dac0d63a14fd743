"""ctypes binding of libhch.so: the same names as the C entry points, arguments marshalled
from numpy arrays (HOST) and torch tensors (DEVICE).  No arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

__all__ = [
    "HchError", "Levels", "LevelInfo", "HCH_F32", "HCH_BF16",
    "HCH_WS_FWD", "HCH_WS_BWD_DATA", "HCH_WS_BWD_WEIGHT", "HCH_WS_MIN",
    "HCH_ALGO_COLUMNS", "HCH_ALGO_FUSED", "HCH_ALGO_COLUMNS_RESIDENT", "HCH_ALGO_FUSED_DENSE",
    "library_path", "load_library", "exported_symbols",
    "hch_build_levels", "hch_build_levels_device", "hch_build_tables_host", "hch_build_neighbours",
    "hch_build_neighbours_range", "hch_hash2col", "hch_col2hash", "hch_conv_workspace_bytes", "hch_conv_fwd", "hch_conv_bwd_data",
    "hch_conv_bwd_weight", "hch_pool_fwd", "hch_pool_bwd", "hch_relu_fwd", "hch_relu_bwd", "hch_relu_pool_fwd",
    "hch_pool_relu_bwd", "hch_pool_relu_bwd_pooled", "hch_deconv_fwd", "hch_deconv_bwd_data", "hch_deconv_bwd_weight",
    "hch_unpool_fwd", "hch_unpool_bwd", "hch_kernel_count", "hch_kernel_name", "hch_profile_enable", "hch_profile_read",
    "hch_profile_reset", "hch_field_build", "hch_sconv_workspace_bytes", "hch_sconv_fwd", "hch_sconv_bwd_weight",
    "hch_sconv_bwd_data", "hch_avgpool_fwd", "hch_avgpool_bwd", "hch_build_levels_ratios",
    "hch_spool_max_fwd", "hch_spool_max_bwd", "hch_spool_avg_fwd", "hch_spool_avg_bwd", "hch_build_tap_major",
    "hch_conv_bwd_weight_noalloc", "HCH_NOALLOC_SCRATCH_BYTES", "hch_probe_mfma", "hch_set_lean_loops",
]

HCH_F32, HCH_BF16 = 0, 1
HCH_WS_FWD, HCH_WS_BWD_DATA, HCH_WS_BWD_WEIGHT, HCH_WS_MIN = 0, 1, 2, 3
HCH_ALGO_COLUMNS, HCH_ALGO_FUSED, HCH_ALGO_COLUMNS_RESIDENT, HCH_ALGO_FUSED_DENSE = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "libhch.so")

# every symbol include/hch.h declares
exported_symbols = [
    "hch_last_error", "hch_build_levels", "hch_build_levels_device", "hch_build_tables_host", "hch_free_levels",
    "hch_num_levels", "hch_level_info", "hch_build_neighbours", "hch_build_neighbours_range", "hch_hash2col",
    "hch_col2hash",
    "hch_conv_workspace_bytes", "hch_conv_fwd", "hch_conv_bwd_data", "hch_conv_bwd_weight",
    "hch_pool_fwd", "hch_pool_bwd", "hch_relu_fwd", "hch_relu_bwd", "hch_relu_pool_fwd",
    "hch_pool_relu_bwd", "hch_pool_relu_bwd_pooled", "hch_deconv_fwd", "hch_deconv_bwd_data", "hch_deconv_bwd_weight",
    "hch_unpool_fwd", "hch_unpool_bwd", "hch_kernel_count", "hch_kernel_name", "hch_profile_enable", "hch_profile_read",
    "hch_profile_reset", "hch_field_build", "hch_sconv_workspace_bytes", "hch_sconv_fwd", "hch_sconv_bwd_weight",
    "hch_sconv_bwd_data", "hch_avgpool_fwd", "hch_avgpool_bwd", "hch_build_levels_ratios",
    "hch_spool_max_fwd", "hch_spool_max_bwd", "hch_spool_avg_fwd", "hch_spool_avg_bwd", "hch_build_tap_major",
    "hch_conv_bwd_weight_noalloc",
    "hch_probe_mfma", "hch_set_lean_loops",
]


class HchError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"hch status {status}: {message}")
        self.status = status


class _Desc(C.Structure):
    _fields_ = [("ubar", C.c_int32), ("batch", C.c_int32), ("n_total", C.c_int64),
                ("m_total", C.c_int64), ("r_total", C.c_int64), ("nbr_valid", C.c_int64),
                ("mbar", C.c_void_p), ("rbar", C.c_void_p), ("attempts", C.c_void_p),
                ("M", C.c_void_p), ("R", C.c_void_p), ("N", C.c_void_p),
                ("coords_host", C.c_void_p), ("H_host", C.c_void_p), ("T_host", C.c_void_p),
                ("Phi_host", C.c_void_p), ("V_host", C.c_void_p),
                ("H", C.c_void_p), ("T", C.c_void_p), ("Phi", C.c_void_p), ("V", C.c_void_p),
                ("coords", C.c_void_p), ("nbr27", C.c_void_p), ("child8", C.c_void_p),
                ("row_order", C.c_void_p), ("tile_taps", C.c_void_p)]


class _KernelStats(C.Structure):
    _fields_ = [("launches", C.c_int64), ("ms", C.c_double), ("bytes", C.c_double),
                ("flops", C.c_double)]


_lib = None


def library_path():
    return _LIBPATH


def load_library():
    """Load libhch.so (built by paper_1803_11385_amd.build.build_library).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIBPATH):
        raise ImportError(f"{_LIBPATH} is missing: run `python -c 'import __graft_entry__ as g; "
                          "g.build()'` (hipcc --offload-arch=gfx950) first; there is no fallback")
    L = C.CDLL(_LIBPATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.hch_last_error.restype = C.c_char_p
    L.hch_build_levels.argtypes = [vp, vp, i32, i32, i32, vp, C.POINTER(vp)]
    L.hch_build_levels_device.argtypes = [vp, vp, i32, i32, i32, vp, C.POINTER(vp)]
    L.hch_build_tables_host.argtypes = [vp, vp, i32, i32, i32, C.POINTER(vp)]
    L.hch_build_levels_ratios.argtypes = [vp, vp, i32, i32, i32, vp, i32, vp, C.POINTER(vp)]
    L.hch_spool_max_fwd.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, i32, vp]
    L.hch_spool_max_bwd.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp]
    L.hch_spool_avg_fwd.argtypes = [vp, i32, i32, i32, vp, vp, vp, i32, vp]
    L.hch_spool_avg_bwd.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, i32, vp]
    L.hch_free_levels.argtypes = [vp]
    L.hch_free_levels.restype = None
    L.hch_num_levels.argtypes = [vp]
    L.hch_num_levels.restype = i32
    L.hch_level_info.argtypes = [vp, i32, C.POINTER(_Desc)]
    L.hch_build_neighbours.argtypes = [vp, i32, vp]
    L.hch_build_neighbours_range.argtypes = [vp, i32, i32, vp]
    L.hch_build_tap_major.argtypes = [vp, i32, vp]
    L.hch_hash2col.argtypes = [vp, i32, C.c_int, vp, i32, i64, i64, vp, vp]
    L.hch_col2hash.argtypes = [vp, i32, vp, i32, vp, vp]
    L.hch_conv_workspace_bytes.argtypes = [vp, i32, i32, i32, C.c_int, C.c_int, C.c_int]
    L.hch_conv_workspace_bytes.restype = sz
    L.hch_field_build.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
    L.hch_sconv_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, i32, C.c_int, C.c_int]
    L.hch_sconv_workspace_bytes.restype = sz
    for name in ("hch_sconv_fwd", "hch_sconv_bwd_weight", "hch_sconv_bwd_data"):
        getattr(L, name).argtypes = [vp, i32, i32, i32, C.c_int, vp, vp, vp, vp, i32, i32, vp, sz, vp]
    L.hch_avgpool_fwd.argtypes = [vp, i32, vp, vp, i32, vp]
    L.hch_avgpool_bwd.argtypes = [vp, i32, vp, vp, i32, vp]
    L.hch_unpool_fwd.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    L.hch_unpool_bwd.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    for name in ("hch_conv_fwd", "hch_conv_bwd_data", "hch_conv_bwd_weight",
                 "hch_deconv_fwd", "hch_deconv_bwd_data", "hch_deconv_bwd_weight"):
        getattr(L, name).argtypes = [vp, i32, C.c_int, vp, vp, vp, i32, i32, vp, sz, C.c_int, vp]
    L.hch_conv_bwd_weight_noalloc.argtypes = [vp, i32, C.c_int, vp, vp, vp, i32, i32, vp]
    L.hch_pool_fwd.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    L.hch_pool_bwd.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    L.hch_relu_pool_fwd.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    L.hch_pool_relu_bwd.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    L.hch_pool_relu_bwd_pooled.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    L.hch_relu_fwd.argtypes = [vp, vp, i64, vp]
    L.hch_relu_bwd.argtypes = [vp, vp, vp, i64, vp]
    L.hch_probe_mfma.argtypes = [C.c_int, i32, i32, vp, vp]
    L.hch_set_lean_loops.argtypes = [i32]
    L.hch_set_lean_loops.restype = i32
    L.hch_kernel_count.restype = i32
    L.hch_kernel_name.argtypes = [i32]
    L.hch_kernel_name.restype = C.c_char_p
    L.hch_profile_enable.argtypes = [i32, i32]
    L.hch_profile_read.argtypes = [i32, C.POINTER(_KernelStats)]
    _lib = L
    return L


def _check(st):
    if st != 0:
        raise HchError(st, load_library().hch_last_error().decode())


def _host_array(ptr, shape, dtype):
    n = int(np.prod(shape))
    if n == 0 or not ptr:
        return np.zeros(shape, dtype)
    buf = (C.c_char * (n * np.dtype(dtype).itemsize)).from_address(ptr)
    return np.frombuffer(buf, dtype=dtype).reshape(shape).copy()


class LevelInfo:
    """Python view of hch_level_desc.  Host arrays are copied into numpy; device arrays are
    exposed as raw addresses (ints) plus `device_*()` helpers that copy them back via torch."""

    def __init__(self, d: _Desc):
        b = d.batch
        self.ubar, self.batch = d.ubar, b
        self.n_total, self.m_total, self.r_total = d.n_total, d.m_total, d.r_total
        self.nbr_valid = d.nbr_valid
        self.mbar = _host_array(d.mbar, (b,), np.int32)
        self.rbar = _host_array(d.rbar, (b,), np.int32)
        self.attempts = _host_array(d.attempts, (b,), np.int32)
        self.M = _host_array(d.M, (b + 1,), np.int64)
        self.R = _host_array(d.R, (b + 1,), np.int64)
        self.N = _host_array(d.N, (b + 1,), np.int64)
        self._d = d

    # host copies of the tables
    def coords_host(self):
        return _host_array(self._d.coords_host, (self.n_total, 3), np.int32)

    def H_host(self):
        return _host_array(self._d.H_host, (self.m_total,), np.int32)

    def T_host(self):
        return _host_array(self._d.T_host, (self.m_total, 3), np.uint16)

    def Phi_host(self):
        return _host_array(self._d.Phi_host, (self.r_total, 3), np.uint8)

    def V_host(self):
        return _host_array(self._d.V_host, (self.m_total,), np.int32)

    # device arrays copied back to numpy
    def _dev(self, ptr, shape, dtype):
        import torch
        n = int(np.prod(shape))
        out = np.empty(shape, dtype)
        if n == 0:
            return out
        if not ptr:
            raise HchError(1, "device table is NULL")
        nbytes = n * np.dtype(dtype).itemsize
        t = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        import ctypes
        hip = _hip()
        st = hip.hipMemcpy(C.c_void_p(t.data_ptr()), C.c_void_p(ptr), C.c_size_t(nbytes), 3)
        if st != 0:
            raise HchError(4, f"hipMemcpy failed ({st})")
        return np.frombuffer(t.cpu().numpy().tobytes(), dtype=dtype).reshape(shape).copy()

    def device_H(self):
        return self._dev(self._d.H, (self.m_total,), np.int32)

    def device_T(self):
        return self._dev(self._d.T, (self.m_total, 3), np.uint16)

    def device_Phi(self):
        return self._dev(self._d.Phi, (self.r_total, 3), np.uint8)

    def device_V(self):
        return self._dev(self._d.V, (self.m_total,), np.int32)

    def device_coords(self):
        return self._dev(self._d.coords, (self.n_total, 3), np.int32)

    def device_nbr27(self):
        return self._dev(self._d.nbr27, (self.n_total, 27), np.int32)

    def device_child8(self):
        return self._dev(self._d.child8, (self.n_total, 8), np.int32)

    def device_row_order(self):
        return self._dev(self._d.row_order, (self.n_total,), np.int32)

    def device_tile_taps(self):
        return self._dev(self._d.tile_taps, ((self.n_total + 63) // 64,), np.uint32)


_hiplib = None


def _hip():
    global _hiplib
    if _hiplib is None:
        for name in ("libamdhip64.so", "/opt/rocm/lib/libamdhip64.so"):
            try:
                _hiplib = C.CDLL(name)
                break
            except OSError:
                continue
        if _hiplib is None:
            raise ImportError("libamdhip64.so not found")
        _hiplib.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    return _hiplib


class Levels:
    """Owner of an hch_levels handle."""

    def __init__(self, handle):
        self._h = handle
        self._n = {}

    @property
    def handle(self):
        if not self._h:
            raise HchError(1, "levels already freed")
        return self._h

    @property
    def n_levels(self):
        return load_library().hch_num_levels(self.handle)

    def info(self, level):
        d = _Desc()
        _check(load_library().hch_level_info(self.handle, level, C.byref(d)))
        return LevelInfo(d)

    def n(self, level):
        """N_l, the number of voxels (rows of every feature tensor) of `level`."""
        if level not in self._n:
            self._n[level] = int(self.info(level).n_total)
        return self._n[level]

    def free(self):
        if self._h:
            load_library().hch_free_levels(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    return C.c_void_p(int(stream))


# Every DEVICE argument is checked here, on the host, before its address goes to the library: a
# CPU tensor, a wrong element type, a non-contiguous view or a buffer shorter than the call will
# read or write would otherwise become an out-of-bounds access on the GPU instead of an error.
_F32, _I32 = "f32", "i32"


def _dp(t, what="tensor", kind=None, numel=0):
    """Address of a DEVICE tensor (None -> NULL).  kind: _F32, _I32, an hch_dtype (HCH_F32 / HCH_BF16:
    float32, or any 2-byte element type holding bfloat16 bit patterns), or None (bytes)."""
    if t is None:
        return C.c_void_p(None)
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise HchError(1, f"{what}: must be a torch tensor in GPU memory")
    if not t.is_contiguous():
        raise HchError(1, f"{what}: must be contiguous")
    if kind == _F32 or kind == HCH_F32:
        ok = t.dtype == torch.float32
    elif kind == _I32:
        ok = t.dtype == torch.int32
    elif kind == HCH_BF16:
        ok = t.element_size() == 2
    else:
        ok = True
    if not ok:
        raise HchError(1, f"{what}: wrong element type {t.dtype}")
    if t.numel() < numel:
        raise HchError(1, f"{what}: {t.numel()} elements, the call needs {int(numel)}")
    return C.c_void_p(t.data_ptr())


def _nbytes(ws):
    return ws.numel() * ws.element_size() if ws is not None else 0


def _in_dtype(dtype):
    if dtype not in (HCH_F32, HCH_BF16):
        raise HchError(1, "unknown dtype")
    return dtype


def _level_n(levels, level, what="level"):
    if not isinstance(level, int) or level < 0 or level >= levels.n_levels:
        raise HchError(1, f"{what} out of range")
    return levels.n(level)


def _out_level(levels, level_in, stride):
    """Rows of the level a field of this stride writes, for the argument checks only; the library
    decides (and rejects a stride that no level matches)."""
    n_in = _level_n(levels, level_in, "level_in")
    if stride == 1:
        return n_in, n_in
    u = levels.info(level_in).ubar
    for l in range(level_in + 1, levels.n_levels):
        if levels.info(l).ubar * stride >= u > (levels.info(l).ubar - 1) * stride:
            return n_in, levels.n(l)
    raise HchError(1, "no level of this set is `stride` times coarser than level_in")


def _host_inputs(coords, model_offsets):
    coords = np.ascontiguousarray(coords, dtype=np.int32)
    offs = np.ascontiguousarray(model_offsets, dtype=np.int64)
    if coords.ndim != 2 or coords.shape[1] != 3 or offs.ndim != 1 or offs.size < 2:
        raise HchError(1, "coords must be [n,3] and model_offsets [b+1]")
    if coords.shape[0] != offs[-1]:
        raise HchError(1, "model_offsets[-1] must equal the number of coordinates")
    return coords, offs


def hch_build_levels(coords, model_offsets, resolution, n_levels, stream=None):
    coords, offs = _host_inputs(coords, model_offsets)
    h = C.c_void_p()
    _check(load_library().hch_build_levels(coords.ctypes.data, offs.ctypes.data, offs.size - 1,
                                           int(resolution), int(n_levels), _stream(stream),
                                           C.byref(h)))
    return Levels(h)


def hch_build_levels_device(coords, model_offsets, resolution, n_levels, stream=None):
    coords, offs = _host_inputs(coords, model_offsets)
    h = C.c_void_p()
    _check(load_library().hch_build_levels_device(coords.ctypes.data, offs.ctypes.data, offs.size - 1,
                                                  int(resolution), int(n_levels), _stream(stream),
                                                  C.byref(h)))
    return Levels(h)


def hch_build_levels_ratios(coords, model_offsets, resolution, ratios, device_tables=False, stream=None):
    """Levels 0 .. len(ratios): level l+1 is ratios[l] times coarser than level l."""
    coords, offs = _host_inputs(coords, model_offsets)
    r = np.ascontiguousarray(np.asarray(ratios, dtype=np.int32).reshape(-1))
    h = C.c_void_p()
    _check(load_library().hch_build_levels_ratios(coords.ctypes.data, offs.ctypes.data, offs.size - 1,
                                                  int(resolution), int(r.size) + 1,
                                                  r.ctypes.data if r.size else None,
                                                  1 if device_tables else 0, _stream(stream), C.byref(h)))
    return Levels(h)


def hch_build_tables_host(coords, model_offsets, resolution, n_levels):
    coords, offs = _host_inputs(coords, model_offsets)
    h = C.c_void_p()
    _check(load_library().hch_build_tables_host(coords.ctypes.data, offs.ctypes.data,
                                                offs.size - 1, int(resolution), int(n_levels),
                                                C.byref(h)))
    return Levels(h)


def hch_build_neighbours(levels, level, stream=None):
    _check(load_library().hch_build_neighbours(levels.handle, level, _stream(stream)))


def hch_build_tap_major(levels, level=-1, stream=None):
    _check(load_library().hch_build_tap_major(levels.handle, level, _stream(stream)))


def hch_build_neighbours_range(levels, first, count, stream=None):
    _check(load_library().hch_build_neighbours_range(levels.handle, first, count, _stream(stream)))


def hch_hash2col(levels, level, dtype, X, c_in, row_begin, row_count, col, stream=None):
    n, dt = _level_n(levels, level), _in_dtype(dtype)
    _check(load_library().hch_hash2col(levels.handle, level, dtype, _dp(X, "X", dt, n * c_in), c_in, row_begin,
                                       row_count, _dp(col, "col", dt, max(0, row_count) * 27 * c_in), _stream(stream)))


def hch_col2hash(levels, level, dcol, c_in, dX, stream=None):
    n = _level_n(levels, level)
    _check(load_library().hch_col2hash(levels.handle, level, _dp(dcol, "dcol", _F32, n * 27 * c_in), c_in,
                                       _dp(dX, "dX", _F32, n * c_in), _stream(stream)))


def hch_conv_workspace_bytes(levels, level, c_in, c_out, dtype, kind, algo=HCH_ALGO_COLUMNS):
    return int(load_library().hch_conv_workspace_bytes(levels.handle, level, c_in, c_out, dtype,
                                                       kind, algo))


def _conv_like(name, levels, level, dtype, a, a_c, b, b_c, out, out_c, c_in, c_out, workspace, algo, stream):
    """a, b: inputs of `dtype`; out: float32.  *_c: channels per voxel row, or None for a weight
    tensor of 27 * c_in * c_out elements."""
    n, dt = _level_n(levels, level), _in_dtype(dtype)
    wn = 27 * c_in * c_out
    size = lambda c: wn if c is None else n * c
    _check(getattr(load_library(), name)(levels.handle, level, dtype, _dp(a, "first input", dt, size(a_c)),
                                         _dp(b, "second input", dt, size(b_c)), _dp(out, "output", _F32, size(out_c)),
                                         c_in, c_out, _dp(workspace, "workspace"), _nbytes(workspace), algo,
                                         _stream(stream)))


def hch_conv_fwd(levels, level, dtype, X, W, Y, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS, stream=None):
    _conv_like("hch_conv_fwd", levels, level, dtype, X, c_in, W, None, Y, c_out, c_in, c_out, workspace, algo, stream)


def hch_conv_bwd_data(levels, level, dtype, dY, W, dX, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS, stream=None):
    _conv_like("hch_conv_bwd_data", levels, level, dtype, dY, c_out, W, None, dX, c_in, c_in, c_out, workspace, algo, stream)


def hch_conv_bwd_weight(levels, level, dtype, X, dY, dW, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS, stream=None):
    _conv_like("hch_conv_bwd_weight", levels, level, dtype, X, c_in, dY, c_out, dW, None, c_in, c_out, workspace, algo, stream)


HCH_NOALLOC_SCRATCH_BYTES = 32 << 20


def hch_conv_bwd_weight_noalloc(levels, level, dtype, X, dY, dW, c_in, c_out, stream=None):
    n, dt = _level_n(levels, level), _in_dtype(dtype)
    _check(load_library().hch_conv_bwd_weight_noalloc(levels.handle, level, dtype, _dp(X, "X", dt, n * c_in),
                                                      _dp(dY, "dY", dt, n * c_out),
                                                      _dp(dW, "dW", _F32, 27 * c_in * c_out), c_in, c_out,
                                                      _stream(stream)))


def hch_deconv_fwd(levels, level, dtype, X, W, Y, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS, stream=None):
    _conv_like("hch_deconv_fwd", levels, level, dtype, X, c_in, W, None, Y, c_out, c_in, c_out, workspace, algo, stream)


def hch_deconv_bwd_data(levels, level, dtype, dY, W, dX, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS,
                        stream=None):
    _conv_like("hch_deconv_bwd_data", levels, level, dtype, dY, c_out, W, None, dX, c_in, c_in, c_out, workspace, algo, stream)


def hch_deconv_bwd_weight(levels, level, dtype, X, dY, dW, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS,
                          stream=None):
    _conv_like("hch_deconv_bwd_weight", levels, level, dtype, X, c_in, dY, c_out, dW, None, c_in, c_out, workspace, algo, stream)


def _pool_rows(levels, level_in):
    """(N_fine, N_coarse) of a pooling between level_in and level_in + 1."""
    return _level_n(levels, level_in, "level_in"), _level_n(levels, level_in + 1, "level_in + 1")


def hch_unpool_fwd(levels, level_out, Xc, argmax, Y, c, stream=None):
    nf, nc = _pool_rows(levels, level_out)
    _check(load_library().hch_unpool_fwd(levels.handle, level_out, _dp(Xc, "Xc", _F32, nc * c),
                                         _dp(argmax, "argmax", _I32, nc * c), _dp(Y, "Y", _F32, nf * c), c,
                                         _stream(stream)))


def hch_unpool_bwd(levels, level_out, dY, argmax, dXc, c, stream=None):
    nf, nc = _pool_rows(levels, level_out)
    _check(load_library().hch_unpool_bwd(levels.handle, level_out, _dp(dY, "dY", _F32, nf * c),
                                         _dp(argmax, "argmax", _I32, nc * c), _dp(dXc, "dXc", _F32, nc * c), c,
                                         _stream(stream)))


def hch_pool_fwd(levels, level_in, X, Y, argmax, c, stream=None):
    nf, nc = _pool_rows(levels, level_in)
    _check(load_library().hch_pool_fwd(levels.handle, level_in, _dp(X, "X", _F32, nf * c), _dp(Y, "Y", _F32, nc * c),
                                       _dp(argmax, "argmax", _I32, nc * c), c, _stream(stream)))


def hch_pool_bwd(levels, level_in, dY, argmax, dX, c, stream=None):
    nf, nc = _pool_rows(levels, level_in)
    _check(load_library().hch_pool_bwd(levels.handle, level_in, _dp(dY, "dY", _F32, nc * c),
                                       _dp(argmax, "argmax", _I32, nc * c), _dp(dX, "dX", _F32, nf * c), c,
                                       _stream(stream)))


def hch_relu_pool_fwd(levels, level_in, Y, A, P, argmax, c, stream=None):
    nf, nc = _pool_rows(levels, level_in)
    _check(load_library().hch_relu_pool_fwd(levels.handle, level_in, _dp(Y, "Y", _F32, nf * c), _dp(A, "A", _F32, nf * c),
                                            _dp(P, "P", _F32, nc * c), _dp(argmax, "argmax", _I32, nc * c), c,
                                            _stream(stream)))


def hch_pool_relu_bwd(levels, level_in, dP, argmax, A, dY, c, stream=None):
    nf, nc = _pool_rows(levels, level_in)
    _check(load_library().hch_pool_relu_bwd(levels.handle, level_in, _dp(dP, "dP", _F32, nc * c),
                                            _dp(argmax, "argmax", _I32, nc * c), _dp(A, "A", _F32, nf * c),
                                            _dp(dY, "dY", _F32, nf * c), c, _stream(stream)))


def hch_pool_relu_bwd_pooled(levels, level_in, dP, argmax, P, dY, c, stream=None):
    nf, nc = _pool_rows(levels, level_in)
    _check(load_library().hch_pool_relu_bwd_pooled(levels.handle, level_in, _dp(dP, "dP", _F32, nc * c),
                                                   _dp(argmax, "argmax", _I32, nc * c), _dp(P, "P", _F32, nc * c),
                                                   _dp(dY, "dY", _F32, nf * c), c, _stream(stream)))


def hch_field_build(levels, level_in, F, stride, pad, field, field_t, stream=None):
    n_in, n_out = _out_level(levels, level_in, stride)
    _check(load_library().hch_field_build(levels.handle, level_in, F, stride, pad,
                                          _dp(field, "field", _I32, n_out * F ** 3),
                                          _dp(field_t, "field_t", _I32, n_in * F ** 3), _stream(stream)))


def hch_sconv_workspace_bytes(levels, level_in, F, stride, c_in, c_out, dtype, kind):
    return int(load_library().hch_sconv_workspace_bytes(levels.handle, level_in, F, stride, c_in, c_out, dtype, kind))


def _sconv(name, levels, level_in, F, stride, dtype, a, a_n, b, b_n, out, out_n, idx, idx_n, c_in, c_out, workspace,
           stream):
    dt = _in_dtype(dtype)
    _check(getattr(load_library(), name)(levels.handle, level_in, F, stride, dtype, _dp(a, "first input", dt, a_n),
                                         _dp(b, "second input", dt, b_n), _dp(out, "output", _F32, out_n),
                                         _dp(idx, "index rows", _I32, idx_n), c_in, c_out, _dp(workspace, "workspace"),
                                         _nbytes(workspace), _stream(stream)))


def hch_sconv_fwd(levels, level_in, F, stride, dtype, X, W, Y, field, c_in, c_out, workspace, stream=None):
    n_in, n_out = _out_level(levels, level_in, stride)
    _sconv("hch_sconv_fwd", levels, level_in, F, stride, dtype, X, n_in * c_in, W, F ** 3 * c_in * c_out, Y,
           n_out * c_out, field, n_out * F ** 3, c_in, c_out, workspace, stream)


def hch_sconv_bwd_weight(levels, level_in, F, stride, dtype, X, dY, dW, field, c_in, c_out, workspace, stream=None):
    n_in, n_out = _out_level(levels, level_in, stride)
    _sconv("hch_sconv_bwd_weight", levels, level_in, F, stride, dtype, X, n_in * c_in, dY, n_out * c_out, dW,
           F ** 3 * c_in * c_out, field, n_out * F ** 3, c_in, c_out, workspace, stream)


def hch_sconv_bwd_data(levels, level_in, F, stride, dtype, dY, W, dX, field_t, c_in, c_out, workspace, stream=None):
    n_in, n_out = _out_level(levels, level_in, stride)
    _sconv("hch_sconv_bwd_data", levels, level_in, F, stride, dtype, dY, n_out * c_out, W, F ** 3 * c_in * c_out, dX,
           n_in * c_in, field_t, n_in * F ** 3, c_in, c_out, workspace, stream)


def hch_avgpool_fwd(levels, level_in, X, Y, c, stream=None):
    nf, nc = _pool_rows(levels, level_in)
    _check(load_library().hch_avgpool_fwd(levels.handle, level_in, _dp(X, "X", _F32, nf * c), _dp(Y, "Y", _F32, nc * c),
                                          c, _stream(stream)))


def hch_avgpool_bwd(levels, level_in, dY, dX, c, stream=None):
    nf, nc = _pool_rows(levels, level_in)
    _check(load_library().hch_avgpool_bwd(levels.handle, level_in, _dp(dY, "dY", _F32, nc * c),
                                          _dp(dX, "dX", _F32, nf * c), c, _stream(stream)))


def hch_spool_max_fwd(levels, level_in, F, stride, X, field, Y, argmax, c, stream=None):
    n_in, n_out = _out_level(levels, level_in, stride)
    _check(load_library().hch_spool_max_fwd(levels.handle, level_in, F, stride, _dp(X, "X", _F32, n_in * c),
                                            _dp(field, "field", _I32, n_out * F ** 3), _dp(Y, "Y", _F32, n_out * c),
                                            _dp(argmax, "argmax", _I32, n_out * c), c, _stream(stream)))


def hch_spool_max_bwd(levels, level_in, F, stride, pad, dY, argmax, field, field_t, dX, c, stream=None):
    n_in, n_out = _out_level(levels, level_in, stride)
    _check(load_library().hch_spool_max_bwd(levels.handle, level_in, F, stride, pad, _dp(dY, "dY", _F32, n_out * c),
                                            _dp(argmax, "argmax", _I32, n_out * c),
                                            _dp(field, "field", _I32, n_out * F ** 3),
                                            _dp(field_t, "field_t", _I32, n_in * F ** 3), _dp(dX, "dX", _F32, n_in * c),
                                            c, _stream(stream)))


def hch_spool_avg_fwd(levels, level_in, F, stride, X, field, Y, c, stream=None):
    n_in, n_out = _out_level(levels, level_in, stride)
    _check(load_library().hch_spool_avg_fwd(levels.handle, level_in, F, stride, _dp(X, "X", _F32, n_in * c),
                                            _dp(field, "field", _I32, n_out * F ** 3), _dp(Y, "Y", _F32, n_out * c), c,
                                            _stream(stream)))


def hch_spool_avg_bwd(levels, level_in, F, stride, pad, dY, field, field_t, dX, c, stream=None):
    n_in, n_out = _out_level(levels, level_in, stride)
    _check(load_library().hch_spool_avg_bwd(levels.handle, level_in, F, stride, pad, _dp(dY, "dY", _F32, n_out * c),
                                            _dp(field, "field", _I32, n_out * F ** 3),
                                            _dp(field_t, "field_t", _I32, n_in * F ** 3), _dp(dX, "dX", _F32, n_in * c),
                                            c, _stream(stream)))


def hch_relu_fwd(x, y, n, stream=None):
    _check(load_library().hch_relu_fwd(_dp(x, "x", _F32, n), _dp(y, "y", _F32, n), n, _stream(stream)))


def hch_relu_bwd(y, dy, dx, n, stream=None):
    _check(load_library().hch_relu_bwd(_dp(y, "y", _F32, n), _dp(dy, "dy", _F32, n), _dp(dx, "dx", _F32, n), n,
                                       _stream(stream)))


def hch_probe_mfma(dtype, iters, workgroups, sink, stream=None):
    _check(load_library().hch_probe_mfma(_in_dtype(dtype), int(iters), int(workgroups),
                                         _dp(sink, "sink", _F32, workgroups * 256), _stream(stream)))


def hch_set_lean_loops(enabled):
    return int(load_library().hch_set_lean_loops(1 if enabled else 0))


def hch_kernel_count():
    return int(load_library().hch_kernel_count())


def hch_kernel_name(kernel_id):
    return load_library().hch_kernel_name(kernel_id).decode()


def hch_profile_enable(kernel_id, on):
    _check(load_library().hch_profile_enable(int(kernel_id), int(bool(on))))


def hch_profile_read(kernel_id):
    st = _KernelStats()
    _check(load_library().hch_profile_read(kernel_id, C.byref(st)))
    return dict(launches=st.launches, ms=st.ms, bytes=st.bytes, flops=st.flops)


def hch_profile_reset():
    _check(load_library().hch_profile_reset())


load_library()
