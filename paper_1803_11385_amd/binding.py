"""ctypes binding of libhch.so: the same names as the C entry points, arguments marshalled
from numpy arrays (HOST) and torch tensors (DEVICE).  No arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

__all__ = [
    "HchError", "Levels", "LevelInfo", "HCH_F32", "HCH_BF16",
    "HCH_WS_FWD", "HCH_WS_BWD_DATA", "HCH_WS_BWD_WEIGHT", "HCH_WS_MIN",
    "HCH_ALGO_COLUMNS", "HCH_ALGO_FUSED", "HCH_ALGO_COLUMNS_RESIDENT",
    "library_path", "load_library", "exported_symbols",
    "hch_build_levels", "hch_build_levels_device", "hch_build_tables_host", "hch_build_neighbours",
    "hch_build_neighbours_range", "hch_hash2col", "hch_col2hash", "hch_conv_workspace_bytes", "hch_conv_fwd", "hch_conv_bwd_data",
    "hch_conv_bwd_weight", "hch_pool_fwd", "hch_pool_bwd", "hch_relu_fwd", "hch_relu_bwd", "hch_relu_pool_fwd",
    "hch_pool_relu_bwd", "hch_deconv_fwd", "hch_deconv_bwd_data", "hch_deconv_bwd_weight",
    "hch_unpool_fwd", "hch_unpool_bwd", "hch_kernel_count", "hch_kernel_name", "hch_profile_enable", "hch_profile_read",
    "hch_profile_reset", "hch_field_build", "hch_sconv_workspace_bytes", "hch_sconv_fwd", "hch_sconv_bwd_weight",
    "hch_sconv_bwd_data", "hch_avgpool_fwd", "hch_avgpool_bwd", "hch_build_levels_ratios",
    "hch_spool_max_fwd", "hch_spool_max_bwd", "hch_spool_avg_fwd", "hch_spool_avg_bwd", "hch_build_tap_major",
]

HCH_F32, HCH_BF16 = 0, 1
HCH_WS_FWD, HCH_WS_BWD_DATA, HCH_WS_BWD_WEIGHT, HCH_WS_MIN = 0, 1, 2, 3
HCH_ALGO_COLUMNS, HCH_ALGO_FUSED, HCH_ALGO_COLUMNS_RESIDENT = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBPATH = os.path.join(_HERE, "libhch.so")

# every symbol include/hch.h declares
exported_symbols = [
    "hch_last_error", "hch_build_levels", "hch_build_levels_device", "hch_build_tables_host", "hch_free_levels",
    "hch_num_levels", "hch_level_info", "hch_build_neighbours", "hch_build_neighbours_range", "hch_hash2col",
    "hch_col2hash",
    "hch_conv_workspace_bytes", "hch_conv_fwd", "hch_conv_bwd_data", "hch_conv_bwd_weight",
    "hch_pool_fwd", "hch_pool_bwd", "hch_relu_fwd", "hch_relu_bwd", "hch_relu_pool_fwd",
    "hch_pool_relu_bwd", "hch_deconv_fwd", "hch_deconv_bwd_data", "hch_deconv_bwd_weight",
    "hch_unpool_fwd", "hch_unpool_bwd", "hch_kernel_count", "hch_kernel_name", "hch_profile_enable", "hch_profile_read",
    "hch_profile_reset", "hch_field_build", "hch_sconv_workspace_bytes", "hch_sconv_fwd", "hch_sconv_bwd_weight",
    "hch_sconv_bwd_data", "hch_avgpool_fwd", "hch_avgpool_bwd", "hch_build_levels_ratios",
    "hch_spool_max_fwd", "hch_spool_max_bwd", "hch_spool_avg_fwd", "hch_spool_avg_bwd", "hch_build_tap_major",
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
                ("coords", C.c_void_p), ("nbr27", C.c_void_p), ("child8", C.c_void_p)]


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
    L.hch_spool_max_bwd.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp]
    L.hch_spool_avg_fwd.argtypes = [vp, i32, i32, i32, vp, vp, vp, i32, vp]
    L.hch_spool_avg_bwd.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, i32, vp]
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
    L.hch_pool_fwd.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    L.hch_pool_bwd.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    L.hch_relu_pool_fwd.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    L.hch_pool_relu_bwd.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    L.hch_relu_fwd.argtypes = [vp, vp, i64, vp]
    L.hch_relu_bwd.argtypes = [vp, vp, vp, i64, vp]
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
        return self.info(level).n_total

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


def _dp(t):
    return C.c_void_p(t.data_ptr() if t is not None else None)


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
    _check(load_library().hch_hash2col(levels.handle, level, dtype, _dp(X), c_in, row_begin,
                                       row_count, _dp(col), _stream(stream)))


def hch_col2hash(levels, level, dcol, c_in, dX, stream=None):
    _check(load_library().hch_col2hash(levels.handle, level, _dp(dcol), c_in, _dp(dX),
                                       _stream(stream)))


def hch_conv_workspace_bytes(levels, level, c_in, c_out, dtype, kind, algo=HCH_ALGO_COLUMNS):
    return int(load_library().hch_conv_workspace_bytes(levels.handle, level, c_in, c_out, dtype,
                                                       kind, algo))


def hch_conv_fwd(levels, level, dtype, X, W, Y, c_in, c_out, workspace,
                 algo=HCH_ALGO_COLUMNS, stream=None):
    _check(load_library().hch_conv_fwd(levels.handle, level, dtype, _dp(X), _dp(W), _dp(Y), c_in,
                                       c_out, _dp(workspace),
                                       workspace.numel() * workspace.element_size(), algo,
                                       _stream(stream)))


def hch_conv_bwd_data(levels, level, dtype, dY, W, dX, c_in, c_out, workspace,
                      algo=HCH_ALGO_COLUMNS, stream=None):
    _check(load_library().hch_conv_bwd_data(levels.handle, level, dtype, _dp(dY), _dp(W), _dp(dX),
                                            c_in, c_out, _dp(workspace),
                                            workspace.numel() * workspace.element_size(), algo,
                                            _stream(stream)))


def hch_conv_bwd_weight(levels, level, dtype, X, dY, dW, c_in, c_out, workspace,
                        algo=HCH_ALGO_COLUMNS, stream=None):
    _check(load_library().hch_conv_bwd_weight(levels.handle, level, dtype, _dp(X), _dp(dY),
                                              _dp(dW), c_in, c_out, _dp(workspace),
                                              workspace.numel() * workspace.element_size(), algo,
                                              _stream(stream)))


def _conv_like(name, levels, level, dtype, a, b, out, c_in, c_out, workspace, algo, stream):
    _check(getattr(load_library(), name)(levels.handle, level, dtype, _dp(a), _dp(b), _dp(out), c_in,
                                         c_out, _dp(workspace),
                                         workspace.numel() * workspace.element_size(), algo,
                                         _stream(stream)))


def hch_deconv_fwd(levels, level, dtype, X, W, Y, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS, stream=None):
    _conv_like("hch_deconv_fwd", levels, level, dtype, X, W, Y, c_in, c_out, workspace, algo, stream)


def hch_deconv_bwd_data(levels, level, dtype, dY, W, dX, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS,
                        stream=None):
    _conv_like("hch_deconv_bwd_data", levels, level, dtype, dY, W, dX, c_in, c_out, workspace, algo, stream)


def hch_deconv_bwd_weight(levels, level, dtype, X, dY, dW, c_in, c_out, workspace, algo=HCH_ALGO_COLUMNS,
                          stream=None):
    _conv_like("hch_deconv_bwd_weight", levels, level, dtype, X, dY, dW, c_in, c_out, workspace, algo, stream)


def hch_unpool_fwd(levels, level_out, Xc, argmax, Y, c, stream=None):
    _check(load_library().hch_unpool_fwd(levels.handle, level_out, _dp(Xc), _dp(argmax), _dp(Y), c,
                                         _stream(stream)))


def hch_unpool_bwd(levels, level_out, dY, argmax, dXc, c, stream=None):
    _check(load_library().hch_unpool_bwd(levels.handle, level_out, _dp(dY), _dp(argmax), _dp(dXc), c,
                                         _stream(stream)))


def hch_pool_fwd(levels, level_in, X, Y, argmax, c, stream=None):
    _check(load_library().hch_pool_fwd(levels.handle, level_in, _dp(X), _dp(Y), _dp(argmax), c,
                                       _stream(stream)))


def hch_pool_bwd(levels, level_in, dY, argmax, dX, c, stream=None):
    _check(load_library().hch_pool_bwd(levels.handle, level_in, _dp(dY), _dp(argmax), _dp(dX), c,
                                       _stream(stream)))


def hch_relu_pool_fwd(levels, level_in, Y, A, P, argmax, c, stream=None):
    _check(load_library().hch_relu_pool_fwd(levels.handle, level_in, _dp(Y), _dp(A), _dp(P),
                                            _dp(argmax), c, _stream(stream)))


def hch_pool_relu_bwd(levels, level_in, dP, argmax, A, dY, c, stream=None):
    _check(load_library().hch_pool_relu_bwd(levels.handle, level_in, _dp(dP), _dp(argmax), _dp(A),
                                            _dp(dY), c, _stream(stream)))


def hch_field_build(levels, level_in, F, stride, pad, field, field_t, stream=None):
    _check(load_library().hch_field_build(levels.handle, level_in, F, stride, pad, _dp(field), _dp(field_t),
                                          _stream(stream)))


def hch_sconv_workspace_bytes(levels, level_in, F, stride, c_in, c_out, dtype, kind):
    return int(load_library().hch_sconv_workspace_bytes(levels.handle, level_in, F, stride, c_in, c_out, dtype, kind))


def _sconv(name, levels, level_in, F, stride, dtype, a, b, out, idx, c_in, c_out, workspace, stream):
    _check(getattr(load_library(), name)(levels.handle, level_in, F, stride, dtype, _dp(a), _dp(b), _dp(out),
                                         _dp(idx), c_in, c_out, _dp(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)))


def hch_sconv_fwd(levels, level_in, F, stride, dtype, X, W, Y, field, c_in, c_out, workspace, stream=None):
    _sconv("hch_sconv_fwd", levels, level_in, F, stride, dtype, X, W, Y, field, c_in, c_out, workspace, stream)


def hch_sconv_bwd_weight(levels, level_in, F, stride, dtype, X, dY, dW, field, c_in, c_out, workspace, stream=None):
    _sconv("hch_sconv_bwd_weight", levels, level_in, F, stride, dtype, X, dY, dW, field, c_in, c_out, workspace, stream)


def hch_sconv_bwd_data(levels, level_in, F, stride, dtype, dY, W, dX, field_t, c_in, c_out, workspace, stream=None):
    _sconv("hch_sconv_bwd_data", levels, level_in, F, stride, dtype, dY, W, dX, field_t, c_in, c_out, workspace, stream)


def hch_avgpool_fwd(levels, level_in, X, Y, c, stream=None):
    _check(load_library().hch_avgpool_fwd(levels.handle, level_in, _dp(X), _dp(Y), c, _stream(stream)))


def hch_avgpool_bwd(levels, level_in, dY, dX, c, stream=None):
    _check(load_library().hch_avgpool_bwd(levels.handle, level_in, _dp(dY), _dp(dX), c, _stream(stream)))


def hch_spool_max_fwd(levels, level_in, F, stride, X, field, Y, argmax, c, stream=None):
    _check(load_library().hch_spool_max_fwd(levels.handle, level_in, F, stride, _dp(X), _dp(field), _dp(Y),
                                            _dp(argmax), c, _stream(stream)))


def hch_spool_max_bwd(levels, level_in, F, stride, dY, argmax, field, field_t, dX, c, stream=None):
    _check(load_library().hch_spool_max_bwd(levels.handle, level_in, F, stride, _dp(dY), _dp(argmax),
                                            _dp(field), _dp(field_t), _dp(dX), c, _stream(stream)))


def hch_spool_avg_fwd(levels, level_in, F, stride, X, field, Y, c, stream=None):
    _check(load_library().hch_spool_avg_fwd(levels.handle, level_in, F, stride, _dp(X), _dp(field), _dp(Y), c,
                                            _stream(stream)))


def hch_spool_avg_bwd(levels, level_in, F, stride, dY, field, field_t, dX, c, stream=None):
    _check(load_library().hch_spool_avg_bwd(levels.handle, level_in, F, stride, _dp(dY), _dp(field), _dp(field_t),
                                            _dp(dX), c, _stream(stream)))


def hch_relu_fwd(x, y, n, stream=None):
    _check(load_library().hch_relu_fwd(_dp(x), _dp(y), n, _stream(stream)))


def hch_relu_bwd(y, dy, dx, n, stream=None):
    _check(load_library().hch_relu_bwd(_dp(y), _dp(dy), _dp(dx), n, _stream(stream)))


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
