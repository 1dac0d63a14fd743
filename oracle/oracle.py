"""ctypes front end of the CPU oracle (oracle/hch_oracle.c) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
module.  It knows nothing of the GPU library and shares no code with it.

Layouts are the paper's (Section 3.2): a level's data array is a row-major
c x N float64 matrix; W is c_out x (c_in*27) with column index i_c*27 + k.
Helpers `to_paper_X` / `to_paper_W` convert from the voxel-major rows and the
[27][c_in][c_out] weights the input generators produce.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hch_oracle.c")
# HCH_ORACLE_LIB names another build of the same source (the sanitizer run of the test suite)
_LIB = os.environ.get("HCH_ORACLE_LIB") or os.path.join(_HERE, "liboracle.so")

ORC_OK, ORC_EINVAL, ORC_ECAP, ORC_EBUILD, ORC_EUNSUPPORTED = 0, 1, 2, 3, 5


def build(force=False, out=None, extra_flags=("-O2",)):
    """Compile the oracle with gcc (plain C, OpenMP on the outer loops).  No -march=native: the
    library is built in one container and also run on another machine."""
    out = out or _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *extra_flags, "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-Wall", "-o", out, _SRC, "-lm"])
    return out


class _Level(C.Structure):
    _fields_ = [("b", C.c_int32), ("ubar", C.c_int32),
                ("mbar", C.c_void_p), ("rbar", C.c_void_p),
                ("M", C.c_void_p), ("R", C.c_void_p), ("N", C.c_void_p),
                ("H", C.c_void_p), ("T", C.c_void_p), ("Phi", C.c_void_p), ("V", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_mbar.restype = C.c_int
        L.orc_mbar.argtypes = [C.c_int64]
        L.orc_rbar0.restype = C.c_int
        L.orc_rbar0.argtypes = [C.c_int64, C.c_int]
        L.orc_rbar_next.restype = C.c_int
        L.orc_rbar_next.argtypes = [C.c_int, C.c_int]
        L.orc_psh_build.restype = C.c_int
        L.orc_lookup.restype = C.c_int64
        L.orc_lookup.argtypes = [C.POINTER(_Level), C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_hash_slot.restype = C.c_int64
        L.orc_hash_slot.argtypes = [C.POINTER(_Level), C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_threads.restype = C.c_int
        _lib = L
    return _lib


def _p(a):
    return C.c_void_p(a.ctypes.data)


def mbar(n):
    return lib().orc_mbar(int(n))


def rbar0(n, m):
    return lib().orc_rbar0(int(n), int(m))


def rbar_next(r, m):
    return lib().orc_rbar_next(int(r), int(m))


def threads():
    return lib().orc_threads()


def set_threads(n):
    """Threads of the oracle's OpenMP loops from now on (timing only; results do not depend on it)."""
    lib().orc_set_threads(C.c_int(int(n)))


def psh_build(coords, ubar):
    """PSH of one model (Section 3.1, 5.2).  Returns dict(m, r, H, T, Phi, attempts)."""
    coords = np.ascontiguousarray(coords, dtype=np.int32)
    n = coords.shape[0]
    m = mbar(n)
    H = np.empty(m ** 3, np.int32)
    T = np.empty((m ** 3, 3), np.uint16)
    r = rbar0(n, m)
    cap = max(8, 4 * r ** 3)
    while True:
        Phi = np.zeros((cap, 3), np.uint8)
        r_out, att = C.c_int(0), C.c_int(0)
        st = lib().orc_psh_build(_p(coords), C.c_int64(n), C.c_int(ubar), _p(H), _p(T), _p(Phi),
                                 C.c_int64(cap), C.byref(r_out), C.byref(att))
        if st == ORC_ECAP:
            cap = max(cap * 4, r_out.value ** 3)
            continue
        if st != ORC_OK:
            raise RuntimeError(f"orc_psh_build failed with status {st}")
        r = r_out.value
        return dict(m=m, r=r, H=H, T=T, Phi=Phi[: r ** 3].copy(), attempts=att.value)


class Level:
    """One resolution level of the mini-batch super-PSH (Section 3.2)."""

    def __init__(self, coords, model_offsets, ubar, tables=None):
        self.coords = np.ascontiguousarray(coords, dtype=np.int32)
        self.model_offsets = np.ascontiguousarray(model_offsets, dtype=np.int64)
        self.ubar = int(ubar)
        self.b = len(self.model_offsets) - 1
        n = np.diff(self.model_offsets).astype(np.int64)
        if tables is None:
            tables = [psh_build(self.coords[self.model_offsets[i]: self.model_offsets[i + 1]], ubar)
                      for i in range(self.b)]
        self.attempts = [t.get("attempts", 1) for t in tables]
        self.n = n
        self.mbar = np.array([t["m"] for t in tables], np.int32)
        self.rbar = np.array([t["r"] for t in tables], np.int32)
        self.M = np.zeros(self.b + 1, np.int64)
        self.R = np.zeros(self.b + 1, np.int64)
        self.N = np.zeros(self.b + 1, np.int64)
        lib().orc_super_prefix(C.c_int32(self.b), _p(self.mbar), _p(self.rbar), _p(self.n),
                               _p(self.M), _p(self.R), _p(self.N))
        # super tables: the per-model tables flattened and attached one after another
        self.H = np.ascontiguousarray(np.concatenate([t["H"] for t in tables]))
        self.T = np.ascontiguousarray(np.concatenate([t["T"] for t in tables], axis=0))
        self.Phi = np.ascontiguousarray(np.concatenate([t["Phi"] for t in tables], axis=0))
        self.V = np.empty(int(self.M[-1]), np.int32)
        lib().orc_fill_V(C.c_int32(self.b), _p(self.M), _p(self.V))
        self.model = np.repeat(np.arange(self.b, dtype=np.int32), n)
        self._c = _Level(self.b, self.ubar, self.mbar.ctypes.data, self.rbar.ctypes.data,
                         self.M.ctypes.data, self.R.ctypes.data, self.N.ctypes.data,
                         self.H.ctypes.data, self.T.ctypes.data, self.Phi.ctypes.data,
                         self.V.ctypes.data)

    @property
    def Ntot(self):
        return int(self.N[-1])

    @property
    def ref(self):
        return C.byref(self._c)

    def lookup(self, v, p):
        return int(lib().orc_lookup(self.ref, int(v), int(p[0]), int(p[1]), int(p[2])))

    def hash_slot(self, v, p):
        return int(lib().orc_hash_slot(self.ref, int(v), int(p[0]), int(p[1]), int(p[2])))


def coarsen(coords, model_offsets, ubar, ratio=2):
    """Next coarser level of the hierarchy.  Section 5.1: each level halves the resolution
    (ratio 2); Section 4: a PSH can be generated on a grid of arbitrary resolution, so any
    integer ratio is possible: the grid has side ceil(ubar / ratio), a coarse voxel is occupied
    iff one of the ratio^3 positions below it is; per model the coarse voxels are ordered by
    their linear index (x*u+y)*u+z, ascending."""
    uc = -(-ubar // ratio)
    out, offs = [], [0]
    for i in range(len(model_offsets) - 1):
        c = coords[model_offsets[i]: model_offsets[i + 1]].astype(np.int64) // ratio
        lin = np.unique((c[:, 0] * uc + c[:, 1]) * uc + c[:, 2])
        cc = np.stack([lin // (uc * uc), (lin // uc) % uc, lin % uc], axis=1).astype(np.int32)
        out.append(cc)
        offs.append(offs[-1] + cc.shape[0])
    return np.concatenate(out, axis=0), np.asarray(offs, np.int64), uc


def build_hierarchy(coords, model_offsets, ubar, n_levels, ratios=None):
    """Level 0 = finest (caller's voxel order); level l+1 is ratios[l] times coarser than level l
    (2 everywhere when ratios is None: resolution ubar / 2^l)."""
    levels = []
    c, o, u = np.ascontiguousarray(coords, np.int32), np.asarray(model_offsets, np.int64), ubar
    for l in range(n_levels):
        levels.append(Level(c, o, u))
        if l + 1 < n_levels:
            c, o, u = coarsen(c, o, u, 2 if ratios is None else int(ratios[l]))
    return levels


# ---------------------------------------------------------------------------
# layout helpers (pure transposes)
# ---------------------------------------------------------------------------

def to_paper_X(X):
    """voxel-major [N, c] -> the paper's c x N float64 data matrix."""
    return np.ascontiguousarray(np.asarray(X, dtype=np.float64).T)


def from_paper_X(D):
    return np.ascontiguousarray(np.asarray(D).T)


def to_paper_W(W):
    """[27, c_in, c_out] -> c_out x (c_in*27) with column index i_c*27 + k."""
    W = np.asarray(W, dtype=np.float64)
    k, ci, co = W.shape
    return np.ascontiguousarray(W.transpose(2, 1, 0).reshape(co, ci * k))


def from_paper_W(Wp, c_in):
    co = Wp.shape[0]
    return np.ascontiguousarray(Wp.reshape(co, c_in, 27).transpose(2, 1, 0))


# ---------------------------------------------------------------------------
# operators
# ---------------------------------------------------------------------------

def hash2col(Li, Lo, Din, F=3, Ss=1, Sp=0):
    Din = np.ascontiguousarray(Din, np.float64)
    c = Din.shape[0]
    assert Din.shape[1] == Li.Ntot
    Dt = np.zeros((c * F ** 3, Lo.Ntot), np.float64)
    lib().orc_hash2col(Li.ref, Lo.ref, C.c_int(c), _p(Din), C.c_int(F), C.c_int(Ss), C.c_int(Sp),
                       _p(Dt))
    return Dt


def col2hash(Li, Lo, dDt, c, F=3, Ss=1, Sp=0):
    dDt = np.ascontiguousarray(dDt, np.float64)
    assert dDt.shape == (c * F ** 3, Lo.Ntot)
    dD = np.empty((c, Li.Ntot), np.float64)
    lib().orc_col2hash(Li.ref, Lo.ref, C.c_int(c), _p(dDt), C.c_int(F), C.c_int(Ss), C.c_int(Sp),
                       _p(dD))
    return dD


def field_indices(Li, Lo, F=3, Ss=1, Sp=0):
    """N_o x F^3 int32: global input data index of every field position, or -1."""
    out = np.full((Lo.Ntot, F ** 3), -2, np.int32)
    lib().orc_field_indices(Li.ref, Lo.ref, C.c_int(F), C.c_int(Ss), C.c_int(Sp), _p(out))
    return out


def neighbours(L):
    """27 neighbour indices of every voxel (3x3x3, stride 1)."""
    return field_indices(L, L, 3, 1, 0)


def children(Lfine, Lcoarse):
    """8 child indices of every coarse voxel (2x2x2, stride 2, no padding)."""
    return field_indices(Lfine, Lcoarse, 2, 2, 0)


def matmul(A, B, ta=False, tb=False):
    A = np.ascontiguousarray(A, np.float64)
    B = np.ascontiguousarray(B, np.float64)
    m = A.shape[1] if ta else A.shape[0]
    k = A.shape[0] if ta else A.shape[1]
    n = B.shape[0] if tb else B.shape[1]
    assert (B.shape[1] if tb else B.shape[0]) == k
    Cm = np.empty((m, n), np.float64)
    lib().orc_matmul(_p(A), _p(B), _p(Cm), C.c_int64(m), C.c_int64(k), C.c_int64(n),
                     C.c_int(int(ta)), C.c_int(int(tb)))
    return Cm


def conv_fwd(L, Din, Wp):
    """D_o = W * hash2col(D_i) (Eq.3); Din c_in x N, Wp c_out x (c_in*27)."""
    Din = np.ascontiguousarray(Din, np.float64)
    Wp = np.ascontiguousarray(Wp, np.float64)
    c_in, c_out = Din.shape[0], Wp.shape[0]
    assert Wp.shape[1] == c_in * 27 and Din.shape[1] == L.Ntot
    Dt = np.zeros((c_in * 27, L.Ntot), np.float64)
    Dout = np.empty((c_out, L.Ntot), np.float64)
    lib().orc_conv_fwd(L.ref, L.ref, C.c_int(c_in), C.c_int(c_out), _p(Din), _p(Wp),
                       C.c_int(3), C.c_int(1), C.c_int(0), _p(Dt), _p(Dout))
    return Dout


def conv_bwd_weight(L, Din, dDout):
    """dW = dD_o * hash2col(D_i)^T (Eq.7)."""
    Din = np.ascontiguousarray(Din, np.float64)
    dDout = np.ascontiguousarray(dDout, np.float64)
    c_in, c_out = Din.shape[0], dDout.shape[0]
    Dt = np.zeros((c_in * 27, L.Ntot), np.float64)
    dW = np.empty((c_out, c_in * 27), np.float64)
    lib().orc_conv_bwd_weight(L.ref, L.ref, C.c_int(c_in), C.c_int(c_out), _p(Din), _p(dDout),
                              C.c_int(3), C.c_int(1), C.c_int(0), _p(Dt), _p(dW))
    return dW


def conv_bwd_data(L, dDout, Wp, c_in):
    """dD_i = col2hash(W^T * dD_o) (Eq.8, Algorithm 2)."""
    dDout = np.ascontiguousarray(dDout, np.float64)
    Wp = np.ascontiguousarray(Wp, np.float64)
    c_out = dDout.shape[0]
    dDt = np.empty((c_in * 27, L.Ntot), np.float64)
    dD = np.empty((c_in, L.Ntot), np.float64)
    lib().orc_conv_bwd_data(L.ref, L.ref, C.c_int(c_in), C.c_int(c_out), _p(dDout), _p(Wp),
                            C.c_int(3), C.c_int(1), C.c_int(0), _p(dDt), _p(dD))
    return dD


def conv_fwd_at(L, Din, Wp, idx):
    Din = np.ascontiguousarray(Din, np.float64)
    Wp = np.ascontiguousarray(Wp, np.float64)
    idx = np.ascontiguousarray(idx, np.int64)
    c_in, c_out = Din.shape[0], Wp.shape[0]
    out = np.empty((idx.size, c_out), np.float64)
    lib().orc_conv_fwd_at(L.ref, C.c_int(c_in), C.c_int(c_out), _p(Din), _p(Wp), _p(L.coords),
                          _p(L.model), _p(idx), C.c_int64(idx.size), _p(out))
    return out


def conv_bwd_data_at(L, dDout, Wp, c_in, idx):
    dDout = np.ascontiguousarray(dDout, np.float64)
    Wp = np.ascontiguousarray(Wp, np.float64)
    idx = np.ascontiguousarray(idx, np.int64)
    c_out = dDout.shape[0]
    out = np.empty((idx.size, c_in), np.float64)
    lib().orc_conv_bwd_data_at(L.ref, C.c_int(c_in), C.c_int(c_out), _p(dDout), _p(Wp),
                               _p(L.coords), _p(L.model), _p(idx), C.c_int64(idx.size), _p(out))
    return out


def conv_bwd_weight_at(L, Din, dDout, triples):
    """dW[o, ci*27+k] for rows (o, ci, k) of `triples`."""
    Din = np.ascontiguousarray(Din, np.float64)
    dDout = np.ascontiguousarray(dDout, np.float64)
    tr = np.ascontiguousarray(triples, np.int32)
    out = np.empty(tr.shape[0], np.float64)
    lib().orc_conv_bwd_weight_at(L.ref, C.c_int(Din.shape[0]), C.c_int(dDout.shape[0]), _p(Din),
                                 _p(dDout), _p(L.coords), _p(L.model), _p(tr),
                                 C.c_int64(tr.shape[0]), _p(out))
    return out


# general kernel side F, stride Ss, padding Sp between an input level Li and an output level Lo
# (Algorithm 1 / 2 as stated: field [p*Ss - Sp, p*Ss - Sp + F - 1]^3, centred when Ss = 1);
# weights c_out x (c_in*F^3) with column index i_c*F^3 + row, row = (fx*F + fy)*F + fz

def sconv_fwd(Li, Lo, Din, Wp, F, Ss, Sp):
    Din = np.ascontiguousarray(Din, np.float64)
    Wp = np.ascontiguousarray(Wp, np.float64)
    c_in, c_out = Din.shape[0], Wp.shape[0]
    assert Wp.shape[1] == c_in * F ** 3 and Din.shape[1] == Li.Ntot
    Dt = np.zeros((c_in * F ** 3, Lo.Ntot), np.float64)
    Dout = np.empty((c_out, Lo.Ntot), np.float64)
    lib().orc_conv_fwd(Li.ref, Lo.ref, C.c_int(c_in), C.c_int(c_out), _p(Din), _p(Wp),
                       C.c_int(F), C.c_int(Ss), C.c_int(Sp), _p(Dt), _p(Dout))
    return Dout


def sconv_bwd_weight(Li, Lo, Din, dDout, F, Ss, Sp):
    Din = np.ascontiguousarray(Din, np.float64)
    dDout = np.ascontiguousarray(dDout, np.float64)
    c_in, c_out = Din.shape[0], dDout.shape[0]
    assert Din.shape[1] == Li.Ntot and dDout.shape[1] == Lo.Ntot
    Dt = np.zeros((c_in * F ** 3, Lo.Ntot), np.float64)
    dW = np.empty((c_out, c_in * F ** 3), np.float64)
    lib().orc_conv_bwd_weight(Li.ref, Lo.ref, C.c_int(c_in), C.c_int(c_out), _p(Din), _p(dDout),
                              C.c_int(F), C.c_int(Ss), C.c_int(Sp), _p(Dt), _p(dW))
    return dW


def sconv_bwd_data(Li, Lo, dDout, Wp, c_in, F, Ss, Sp):
    dDout = np.ascontiguousarray(dDout, np.float64)
    Wp = np.ascontiguousarray(Wp, np.float64)
    c_out = dDout.shape[0]
    assert dDout.shape[1] == Lo.Ntot and Wp.shape == (c_out, c_in * F ** 3)
    dDt = np.empty((c_in * F ** 3, Lo.Ntot), np.float64)
    dD = np.empty((c_in, Li.Ntot), np.float64)
    lib().orc_conv_bwd_data(Li.ref, Lo.ref, C.c_int(c_in), C.c_int(c_out), _p(dDout), _p(Wp),
                            C.c_int(F), C.c_int(Ss), C.c_int(Sp), _p(dDt), _p(dD))
    return dD


def avgpool_fwd(Lfine, Lcoarse, Din, F=2, Ss=2, Sp=0):
    """Average pooling (Section 4): the strided convolution whose weights all equal 1/F^3, applied
    channel by channel: the mean of the column matrix over the F^3 field rows."""
    Din = np.ascontiguousarray(Din, np.float64)
    c = Din.shape[0]
    Dt = hash2col(Lfine, Lcoarse, Din, F, Ss, Sp)
    return Dt.reshape(c, F ** 3, Lcoarse.Ntot).sum(axis=1) / F ** 3


def avgpool_bwd(Lfine, Lcoarse, dDout, F=2, Ss=2, Sp=0):
    """Its adjoint = average-unpooling (Section 4): the coarse value spread evenly over the field."""
    dDout = np.ascontiguousarray(dDout, np.float64)
    c = dDout.shape[0]
    dDt = np.repeat(dDout[:, None, :] / F ** 3, F ** 3, axis=1).reshape(c * F ** 3, Lcoarse.Ntot)
    return col2hash(Lfine, Lcoarse, dDt, c, F, Ss, Sp)


def pool_max_fwd(Lfine, Lcoarse, Din, F=2, Ss=2, Sp=0):
    Din = np.ascontiguousarray(Din, np.float64)
    c = Din.shape[0]
    assert Din.shape[1] == Lfine.Ntot
    Dout = np.zeros((c, Lcoarse.Ntot), np.float64)
    sw = np.full((c, Lcoarse.Ntot), -1, np.int32)
    lib().orc_pool_max_fwd(Lfine.ref, Lcoarse.ref, C.c_int(c), _p(Din), C.c_int(F), C.c_int(Ss),
                           C.c_int(Sp), _p(Dout), _p(sw))
    return Dout, sw


def pool_max_bwd(Ni, dDout, sw):
    dDout = np.ascontiguousarray(dDout, np.float64)
    sw = np.ascontiguousarray(sw, np.int32)
    c, No = dDout.shape
    dD = np.empty((c, Ni), np.float64)
    lib().orc_pool_max_bwd(C.c_int(c), C.c_int64(Ni), C.c_int64(No), _p(dDout), _p(sw), _p(dD))
    return dD


def deconv_fwd(L, Din, Wp):
    """Transposed convolution (Section 4): col2hash(W^T * D_i).  Din c_i x N; Wp c_i x (c_o*27) is
    the weight matrix of the forward convolution c_o -> c_i being transposed; returns c_o x N."""
    Din = np.ascontiguousarray(Din, np.float64)
    Wp = np.ascontiguousarray(Wp, np.float64)
    c_i = Din.shape[0]
    assert Wp.shape[0] == c_i and Wp.shape[1] % 27 == 0
    c_o = Wp.shape[1] // 27
    Dt = np.empty((c_o * 27, L.Ntot), np.float64)
    Dout = np.empty((c_o, L.Ntot), np.float64)
    lib().orc_deconv_fwd(L.ref, C.c_int(c_i), C.c_int(c_o), _p(Din), _p(Wp), C.c_int(3), _p(Dt), _p(Dout))
    return Dout


def unpool_max_fwd(Nfine, Dcoarse, sw):
    """Max-unpooling (Section 4): zero everywhere except at the recorded switches."""
    return pool_max_bwd(Nfine, Dcoarse, sw)


def unpool_max_bwd(dDfine, sw):
    dDfine = np.ascontiguousarray(dDfine, np.float64)
    sw = np.ascontiguousarray(sw, np.int32)
    c, Nf = dDfine.shape
    Nc = sw.shape[1]
    out = np.empty((c, Nc), np.float64)
    lib().orc_unpool_max_bwd(C.c_int(c), C.c_int64(Nf), C.c_int64(Nc), _p(dDfine), _p(sw), _p(out))
    return out
