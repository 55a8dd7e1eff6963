"""ctypes loader for the float64 CPU oracle in s2_oracle.c.

TEST INFRASTRUCTURE ONLY (see the header of s2_oracle.c).  Argument
marshalling only: every number comes out of the C functions.  All arrays are
float64 numpy, C-contiguous, in the layouts documented in s2_oracle.c.
"""
import ctypes
import os
import subprocess

import numpy as np

EQUIANGULAR = 0
LEGENDRE_GAUSS = 1
LEGENDRE_GAUSS_LOBATTO = 3  # Gauss-Lobatto nodes in cos(colat): a Gaussian-type grid with both poles
EQUIANGULAR_TRAPEZOID = 2   # the grid exactly as App. A.1 prints it (no south pole, zero weight at the pole)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "s2_oracle.c")
# S2_ORACLE_LIB: load another build of the same source instead (the sanitizer test points it at an ASan/UBSan build)
_LIB = os.environ.get("S2_ORACLE_LIB") or os.path.join(_HERE, "liboracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_bp = ctypes.POINTER(ctypes.c_uint8)


def build(force=False):
    """Compile s2_oracle.c into liboracle.so next to it (gcc, OpenMP)."""
    if os.environ.get("S2_ORACLE_LIB"):
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.s2o_geodesic.restype = ctypes.c_double
        _lib.s2o_geodesic.argtypes = [ctypes.c_double] * 4
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


def grid(grid_type, nlat):
    """(colat[nlat], wlat[nlat]); wlat integrates f(colat) sin(colat) over [0, pi]."""
    colat = np.empty(nlat, np.float64)
    wlat = np.empty(nlat, np.float64)
    rc = _load().s2o_grid(int(grid_type), int(nlat), colat.ctypes.data_as(_dp), wlat.ctypes.data_as(_dp))
    if rc:
        raise ValueError("s2o_grid failed (%d)" % rc)
    return colat, wlat


def omega(grid_type, nlat, nlon):
    """Quadrature weight per latitude, longitude spacing included."""
    return grid(grid_type, nlat)[1] * (2.0 * np.pi / nlon)


def geodesic(colat1, lon1, colat2, lon2):
    return _load().s2o_geodesic(float(colat1), float(lon1), float(colat2), float(lon2))


def indicator(grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta):
    """uint8 mask[nlat_out][nlat_in][nlon_in] for the output point at longitude 0."""
    m = np.zeros((nlat_out, nlat_in, nlon_in), np.uint8)
    rc = _load().s2o_indicator(
        int(grid_type), int(nlat_in), int(nlon_in), int(nlat_out), int(nlon_out),
        ctypes.c_double(theta), m.ctypes.data_as(_bp))
    if rc:
        raise ValueError("s2o_indicator failed (%d)" % rc)
    return m


def indicator_point(grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta, h, w):
    """uint8 row[nlat_in][nlon_in]: brute-force disk membership for output point (h, w)."""
    m = np.zeros((nlat_in, nlon_in), np.uint8)
    rc = _load().s2o_indicator_point(
        int(grid_type), int(nlat_in), int(nlon_in), int(nlat_out), int(nlon_out),
        ctypes.c_double(theta), int(h), int(w), m.ctypes.data_as(_bp))
    if rc:
        raise ValueError("s2o_indicator_point failed (%d)" % rc)
    return m


def neighbor_csr(grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta):
    """Canonical neighbor lists from the indicator: row_ptr int64[nlat_out+1],
    col int32[] = h'*nlon_in + w', ascending within each output latitude."""
    m = indicator(grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta)
    flat = m.reshape(nlat_out, -1)
    counts = flat.sum(axis=1, dtype=np.int64)
    row_ptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    col = np.nonzero(flat)[1].astype(np.int32)
    return row_ptr, col


def _grid_args(g):
    return [int(g["grid_type"]), int(g["nlat_in"]), int(g["nlon_in"]), int(g["nlat_out"]), int(g["nlon_out"]),
            ctypes.c_double(g["theta"])]


def nattn_fwd(g, q, k, v, scale, brute=False):
    """g: dict(grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta).
    brute: False = shift-invariant indicator of App. B.3; True (1) = eq. (5) per (output, input) pair, mask stored;
    2 = eq. (5) per pair evaluated on the fly (no N_out * N_in bytes: any grid size).
    q [nbh,d,Ho,Wo], k [nbh,d,Hi,Wi], v [nbh,e,Hi,Wi] -> out [nbh,e,Ho,Wo], lse [nbh,Ho,Wo]."""
    q, qp = _d(q); k, kp = _d(k); v, vp = _d(v)
    nbh, d = q.shape[0], q.shape[1]
    e = v.shape[1]
    assert q.shape[2:] == (g["nlat_out"], g["nlon_out"]) and k.shape == (nbh, d, g["nlat_in"], g["nlon_in"])
    assert v.shape == (nbh, e, g["nlat_in"], g["nlon_in"])
    out = np.empty((nbh, e, g["nlat_out"], g["nlon_out"]), np.float64)
    lse = np.empty((nbh, g["nlat_out"], g["nlon_out"]), np.float64)
    rc = _load().s2o_nattn_fwd(*_grid_args(g), int(brute), nbh, d, e, ctypes.c_double(scale),
                               qp, kp, vp, out.ctypes.data_as(_dp), lse.ctypes.data_as(_dp))
    if rc:
        raise ValueError("s2o_nattn_fwd failed (%d)" % rc)
    return out, lse


def nattn_bwd(g, q, k, v, dout, scale, brute=False):
    """Gradients of sum(dout*out): returns dq, dk, dv shaped like q, k, v."""
    q, qp = _d(q); k, kp = _d(k); v, vp = _d(v); dout, gp = _d(dout)
    nbh, d = q.shape[0], q.shape[1]
    e = v.shape[1]
    assert dout.shape == (nbh, e, g["nlat_out"], g["nlon_out"])
    dq = np.empty_like(q); dk = np.empty_like(k); dv = np.empty_like(v)
    rc = _load().s2o_nattn_bwd(*_grid_args(g), int(brute), nbh, d, e, ctypes.c_double(scale),
                               qp, kp, vp, gp, dq.ctypes.data_as(_dp), dk.ctypes.data_as(_dp),
                               dv.ctypes.data_as(_dp))
    if rc:
        raise ValueError("s2o_nattn_bwd failed (%d)" % rc)
    return dq, dk, dv


def nattn_cond(g, q, k, v, dout, scale, brute=False):
    """Rounding sensitivities (sums of absolute terms, see s2o_nattn_cond) of out, lse, dq, dk, dv."""
    q, qp = _d(q); k, kp = _d(k); v, vp = _d(v); dout, gp = _d(dout)
    nbh, d = q.shape[0], q.shape[1]
    e = v.shape[1]
    assert dout.shape == (nbh, e, g["nlat_out"], g["nlon_out"])
    c_out = np.empty_like(dout); c_lse = np.empty((nbh, g["nlat_out"], g["nlon_out"]), np.float64)
    c_dq = np.empty_like(q); c_dk = np.empty_like(k); c_dv = np.empty_like(v)
    rc = _load().s2o_nattn_cond(*_grid_args(g), int(brute), nbh, d, e, ctypes.c_double(scale),
                                qp, kp, vp, gp, c_out.ctypes.data_as(_dp), c_lse.ctypes.data_as(_dp),
                                c_dq.ctypes.data_as(_dp), c_dk.ctypes.data_as(_dp), c_dv.ctypes.data_as(_dp))
    if rc:
        raise ValueError("s2o_nattn_cond failed (%d)" % rc)
    return c_out, c_lse, c_dq, c_dk, c_dv


def global_fwd(grid_type, nlat, nlon, q, k, v, scale):
    """Token-major q,k [nbh,N,d], v [nbh,N,e] -> out [nbh,N,e], lse [nbh,N]."""
    q, qp = _d(q); k, kp = _d(k); v, vp = _d(v)
    nbh, N, d = q.shape
    e = v.shape[2]
    assert N == nlat * nlon and k.shape == (nbh, N, d) and v.shape == (nbh, N, e)
    out = np.empty((nbh, N, e), np.float64)
    lse = np.empty((nbh, N), np.float64)
    rc = _load().s2o_global_fwd(int(grid_type), int(nlat), int(nlon), nbh, d, e, ctypes.c_double(scale),
                                qp, kp, vp, out.ctypes.data_as(_dp), lse.ctypes.data_as(_dp))
    if rc:
        raise ValueError("s2o_global_fwd failed (%d)" % rc)
    return out, lse


def global_bwd(grid_type, nlat, nlon, q, k, v, dout, scale):
    q, qp = _d(q); k, kp = _d(k); v, vp = _d(v); dout, gp = _d(dout)
    nbh, N, d = q.shape
    e = v.shape[2]
    assert N == nlat * nlon and dout.shape == (nbh, N, e)
    dq = np.empty_like(q); dk = np.empty_like(k); dv = np.empty_like(v)
    rc = _load().s2o_global_bwd(int(grid_type), int(nlat), int(nlon), nbh, d, e, ctypes.c_double(scale),
                                qp, kp, vp, gp, dq.ctypes.data_as(_dp), dk.ctypes.data_as(_dp),
                                dv.ctypes.data_as(_dp))
    if rc:
        raise ValueError("s2o_global_bwd failed (%d)" % rc)
    return dq, dk, dv
