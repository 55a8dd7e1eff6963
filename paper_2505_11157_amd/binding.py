"""Thin ctypes binding of libs2attn.so: same names as the C ABI (include/s2attn.h).

Argument marshalling only.  Tensors are torch tensors used as device-memory
handles (data_ptr) and the current torch stream is passed as the HIP stream;
nothing is computed here.  There is no fallback: a missing library raises.
"""
import ctypes
import os

import numpy as np

S2_GRID_EQUIANGULAR = 0
S2_GRID_LEGENDRE_GAUSS = 1
S2_GRID_EQUIANGULAR_TRAPEZOID = 2
S2_GRID_LEGENDRE_GAUSS_LOBATTO = 3
S2_F32 = 0
S2_BF16 = 1
S2_OK = 0
S2_ERR_INVALID_ARG = -1
S2_ERR_UNSUPPORTED = -2
S2_ERR_EMPTY_NEIGHBORHOOD = -3
S2_ERR_ALLOC = -4
S2_ERR_DEVICE = -5
S2_ERR_WORKSPACE = -6
S2_ERR_AMBIGUOUS_CUTOFF = -7
S2_DEBUG_NO_MFMA = 1
S2_DEBUG_NO_STREAM = 2
S2_DEBUG_NO_ROW_GROUPS = 4
S2_DEBUG_FAIL_LAUNCH = 8
S2_DEBUG_FORCE_BAND = 16
S2_DEBUG_NO_BAND = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libs2attn.so")
_lib = None

_vp = ctypes.c_void_p
_i = ctypes.c_int


class S2Error(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("s2attn error %d: %s" % (code, msg))
        self.code = code


def lib():
    """Load libs2attn.so (built in-tree by paper_2505_11157_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libs2attn.so is not built: run `python -m paper_2505_11157_amd.build` "
                              "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        L.s2_grid_init.argtypes = [_i, _i, _i, _i, _i, ctypes.c_double, ctypes.POINTER(_vp)]
        L.s2_grid_init.restype = _i
        L.s2_grid_destroy.argtypes = [_vp]
        L.s2_grid_destroy.restype = None
        L.s2_grid_get_weights.argtypes = [_vp, _vp, _vp]
        L.s2_grid_get_weights.restype = _i
        L.s2_grid_device_flags.argtypes = [_vp, ctypes.POINTER(ctypes.c_uint)]
        L.s2_grid_device_flags.restype = _i
        L.s2_grid_num_neighbors.argtypes = [_vp]
        L.s2_grid_num_neighbors.restype = ctypes.c_int64
        L.s2_grid_get_neighbors.argtypes = [_vp, _vp, _vp]
        L.s2_grid_get_neighbors.restype = _i
        L.s2_grid_get_neighbors_at.argtypes = [_vp, _i, _i, _vp, _vp]
        L.s2_grid_get_neighbors_at.restype = _i
        L.s2_nattn_bwd_workspace_bytes.argtypes = [_vp, _i, _i, _i, _i, _i]
        L.s2_nattn_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.s2_nattn_fwd.argtypes = [_vp, _i, _i, _i, _i, _i, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp]
        L.s2_nattn_fwd.restype = _i
        L.s2_nattn_bwd.argtypes = [_vp, _i, _i, _i, _i, _i, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp,
                                   _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.s2_nattn_bwd.restype = _i
        L.s2_nattn_bwd_static.argtypes = [_vp, _i, _i, _i, _i, _i, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp,
                                          _vp, _vp, _vp, _vp]
        L.s2_nattn_bwd_static.restype = _i
        L.s2_nattn_bwd_static_max_points.argtypes = []
        L.s2_nattn_bwd_static_max_points.restype = ctypes.c_size_t
        L.s2_mha_workspace_bytes.argtypes = [_vp, _i, _i, _i]
        L.s2_mha_workspace_bytes.restype = ctypes.c_size_t
        L.s2_mha_fwd.argtypes = [_vp, _i, _i, _i, ctypes.c_float, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.s2_mha_fwd.restype = _i
        L.s2_mha_bwd.argtypes = [_vp, _i, _i, _i, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.s2_mha_bwd.restype = _i
        L.s2_disco_init.argtypes = [_vp, _i, ctypes.POINTER(_vp)]
        L.s2_disco_init.restype = _i
        L.s2_disco_destroy.argtypes = [_vp]
        L.s2_disco_destroy.restype = None
        L.s2_disco_workspace_bytes.argtypes = [_vp, _i, _i, _i]
        L.s2_disco_workspace_bytes.restype = ctypes.c_size_t
        L.s2_disco_fwd.argtypes = [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.s2_disco_fwd.restype = _i
        L.s2_disco_bwd.argtypes = [_vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.s2_disco_bwd.restype = _i
        L.s2_attn_global_fwd_workspace_bytes.argtypes = [_vp, _i, _i, _i, _i]
        L.s2_attn_global_fwd_workspace_bytes.restype = ctypes.c_size_t
        L.s2_attn_global_bwd_workspace_bytes.argtypes = [_vp, _i, _i, _i, _i]
        L.s2_attn_global_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.s2_attn_global_fwd.argtypes = [_vp, _i, _i, _i, _i, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp,
                                         ctypes.c_size_t, _vp]
        L.s2_attn_global_fwd.restype = _i
        L.s2_attn_global_bwd.argtypes = [_vp, _i, _i, _i, _i, ctypes.c_float, _vp, _vp, _vp, _vp, _vp, _vp,
                                         _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.s2_attn_global_bwd.restype = _i
        L.s2_trace_enable.argtypes = [_i]
        L.s2_trace_enable.restype = _i
        L.s2_trace_count.argtypes = []
        L.s2_trace_count.restype = _i
        L.s2_trace_get.argtypes = [_i, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float),
                                   ctypes.POINTER(ctypes.c_double)]
        L.s2_trace_get.restype = _i
        L.s2_trace_reset.argtypes = []
        L.s2_trace_reset.restype = None
        L.s2_peak_measure.argtypes = [_i, ctypes.POINTER(ctypes.c_double)]
        L.s2_peak_measure.restype = _i
        L.s2_debug_control.argtypes = [ctypes.c_uint, ctypes.c_uint]
        L.s2_debug_control.restype = ctypes.c_uint
        L.s2_last_error.argtypes = []
        L.s2_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def s2_last_error():
    return lib().s2_last_error().decode()


def _check(rc):
    if rc != S2_OK:
        raise S2Error(rc, s2_last_error())


class Grid:
    """Owner of an s2_grid_t* (released on garbage collection)."""

    def __init__(self, handle, grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta):
        self.handle = handle
        self.grid_type, self.theta = grid_type, theta
        self.nlat_in, self.nlon_in, self.nlat_out, self.nlon_out = nlat_in, nlon_in, nlat_out, nlon_out

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.s2_grid_destroy(self.handle)
            self.handle = None


def s2_grid_init(grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta_cutoff):
    h = _vp()
    _check(lib().s2_grid_init(int(grid_type), int(nlat_in), int(nlon_in), int(nlat_out), int(nlon_out),
                              float(theta_cutoff), ctypes.byref(h)))
    return Grid(h, grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta_cutoff)


def s2_grid_get_weights(g):
    colat = np.empty(g.nlat_in, np.float64)
    om = np.empty(g.nlat_in, np.float64)
    _check(lib().s2_grid_get_weights(g.handle, colat.ctypes.data, om.ctypes.data))
    return colat, om


def s2_grid_device_flags(g):
    """Synchronise and return the device-side flag word of the handle (0 = healthy); clears it."""
    flags = ctypes.c_uint(0)
    _check(lib().s2_grid_device_flags(g.handle, ctypes.byref(flags)))
    return int(flags.value)


def s2_grid_num_neighbors(g):
    return int(lib().s2_grid_num_neighbors(g.handle))


def s2_grid_get_neighbors_at(g, h, w):
    """Neighbor list of output point (h, w): absolute input indices h'*nlon_in + w_in, ascending."""
    n = ctypes.c_int(0)
    _check(lib().s2_grid_get_neighbors_at(g.handle, int(h), int(w), None, ctypes.byref(n)))
    col = np.empty(n.value, np.int32)
    _check(lib().s2_grid_get_neighbors_at(g.handle, int(h), int(w), col.ctypes.data, ctypes.byref(n)))
    return col


def s2_grid_get_neighbors(g):
    row_ptr = np.empty(g.nlat_out + 1, np.int64)
    col = np.empty(s2_grid_num_neighbors(g), np.int32)
    _check(lib().s2_grid_get_neighbors(g.handle, row_ptr.ctypes.data, col.ctypes.data))
    return row_ptr, col


def _stream():
    import torch
    return _vp(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return S2_F32
    if t.dtype == torch.bfloat16:
        return S2_BF16
    raise TypeError("unsupported tensor dtype %s" % t.dtype)


def _dev(*ts):
    for t in ts:
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def s2_nattn_bwd_workspace_bytes(g, batch, heads, d_qk, d_v, dtype=S2_F32):
    return int(lib().s2_nattn_bwd_workspace_bytes(g.handle, batch, heads, d_qk, d_v, dtype))


def s2_nattn_fwd(g, q, k, v, scale, out=None, lse=None):
    """q [B,H,d,nlat_out,nlon_out], k [B,H,d,nlat_in,nlon_in], v [B,H,e,nlat_in,nlon_in] -> out, lse."""
    import torch
    _dev(q, k, v)
    B, H, d = q.shape[:3]
    e = v.shape[2]
    if q.shape[3:] != (g.nlat_out, g.nlon_out) or k.shape != (B, H, d, g.nlat_in, g.nlon_in) \
            or v.shape != (B, H, e, g.nlat_in, g.nlon_in):
        raise ValueError("tensor shapes do not match the grid handle")
    if out is None:
        out = torch.empty((B, H, e, g.nlat_out, g.nlon_out), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((B, H, g.nlat_out, g.nlon_out), dtype=torch.float32, device=q.device)
    _dev(out, lse)
    _check(lib().s2_nattn_fwd(g.handle, B, H, d, e, _dtype_code(q), float(scale), q.data_ptr(), k.data_ptr(),
                              v.data_ptr(), out.data_ptr(), lse.data_ptr(), _stream()))
    return out, lse


def s2_nattn_bwd(g, q, k, v, out, lse, dout, scale, dq=None, dk=None, dv=None, workspace=None):
    import torch
    _dev(q, k, v, out, lse, dout)
    B, H, d = q.shape[:3]
    e = v.shape[2]
    if out.shape != (B, H, e, g.nlat_out, g.nlon_out) or dout.shape != out.shape \
            or lse.shape != (B, H, g.nlat_out, g.nlon_out) or k.shape != (B, H, d, g.nlat_in, g.nlon_in):
        raise ValueError("tensor shapes do not match the grid handle")
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = s2_nattn_bwd_workspace_bytes(g, B, H, d, e, _dtype_code(q))
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    _dev(dq, dk, dv, workspace)
    _check(lib().s2_nattn_bwd(g.handle, B, H, d, e, _dtype_code(q), float(scale), q.data_ptr(), k.data_ptr(),
                              v.data_ptr(), out.data_ptr(), lse.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                              dk.data_ptr(), dv.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()))
    return dq, dk, dv


def s2_nattn_bwd_static_max_points():
    return int(lib().s2_nattn_bwd_static_max_points())


def s2_nattn_bwd_static(g, q, k, v, out, lse, dout, scale, dq, dk, dv):
    """s2_nattn_bwd on the library's static device scratch: allocates nothing, so the gradients are passed in."""
    _dev(q, k, v, out, lse, dout, dq, dk, dv)
    B, H, d = q.shape[:3]
    e = v.shape[2]
    if out.shape != (B, H, e, g.nlat_out, g.nlon_out) or dout.shape != out.shape \
            or lse.shape != (B, H, g.nlat_out, g.nlon_out) or k.shape != (B, H, d, g.nlat_in, g.nlon_in) \
            or dq.shape != q.shape or dk.shape != k.shape or dv.shape != v.shape:
        raise ValueError("tensor shapes do not match the grid handle")
    _check(lib().s2_nattn_bwd_static(g.handle, B, H, d, e, _dtype_code(q), float(scale), q.data_ptr(), k.data_ptr(),
                                     v.data_ptr(), out.data_ptr(), lse.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                     dk.data_ptr(), dv.data_ptr(), _stream()))
    return dq, dk, dv


MHA_FIELDS = ("gamma", "beta", "pos", "Wq", "bq", "Wk", "bk", "Wv", "bv", "Wo", "bo")


class _MhaPointers(ctypes.Structure):
    """s2_mha_params_t / s2_mha_grads_t: eleven device pointers."""
    _fields_ = [(f, ctypes.c_void_p) for f in MHA_FIELDS]


def _mha_struct(tensors):
    st = _MhaPointers()
    for f in MHA_FIELDS:
        t = tensors.get(f)
        if t is not None:
            _dev(t)
        setattr(st, f, t.data_ptr() if t is not None else None)
    return st


def s2_mha_workspace_bytes(g, batch, channels, heads):
    return int(lib().s2_mha_workspace_bytes(g.handle, batch, channels, heads))


def s2_mha_fwd(g, x, params, heads, eps=1e-5, y=None, workspace=None):
    """x [B, C, nlat, nlon] float32; params: dict of device tensors (MHA_FIELDS; optional ones may be missing).
    Returns y and the workspace (which s2_mha_bwd needs back)."""
    import torch
    _dev(x)
    B, C = x.shape[:2]
    y = torch.empty_like(x) if y is None else y
    if workspace is None:
        workspace = torch.empty(max(s2_mha_workspace_bytes(g, B, C, heads), 1), dtype=torch.uint8, device=x.device)
    st = _mha_struct(params)
    _check(lib().s2_mha_fwd(g.handle, B, C, heads, float(eps), x.data_ptr(), ctypes.byref(st), y.data_ptr(),
                            workspace.data_ptr(), workspace.numel(), _stream()))
    return y, workspace


def s2_mha_bwd(g, x, params, heads, dy, workspace, eps=1e-5, want=MHA_FIELDS):
    """Gradients of sum(dy * y): returns dx and a dict of parameter gradients (for the names in `want` that exist in
    params)."""
    import torch
    _dev(x, dy, workspace)
    B, C = x.shape[:2]
    dx = torch.empty_like(x)
    grads = {f: torch.empty_like(params[f]) for f in want if params.get(f) is not None}
    st, gs = _mha_struct(params), _mha_struct(grads)
    _check(lib().s2_mha_bwd(g.handle, B, C, heads, float(eps), x.data_ptr(), ctypes.byref(st), dy.data_ptr(),
                            dx.data_ptr(), ctypes.byref(gs), workspace.data_ptr(), workspace.numel(), _stream()))
    return dx, grads


class Disco:
    """Owner of an s2_disco_t* (keeps its grid handle alive; released on garbage collection)."""

    def __init__(self, handle, grid, nbasis):
        self.handle, self.grid, self.nbasis = handle, grid, nbasis

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.s2_disco_destroy(self.handle)
            self.handle = None


def s2_disco_init(g, nbasis):
    h = _vp()
    _check(lib().s2_disco_init(g.handle, int(nbasis), ctypes.byref(h)))
    return Disco(h, g, nbasis)


def s2_disco_workspace_bytes(dc, batch, cin, cout):
    return int(lib().s2_disco_workspace_bytes(dc.handle, batch, cin, cout))


def s2_disco_fwd(dc, x, weight, bias=None, y=None, workspace=None):
    """x [B, cin, nlat_in, nlon_in], weight [cout, cin, nbasis] -> y [B, cout, nlat_out, nlon_out], workspace."""
    import torch
    _dev(x, weight)
    B, cin = x.shape[:2]
    cout = weight.shape[0]
    g = dc.grid
    if x.shape[2:] != (g.nlat_in, g.nlon_in) or weight.shape != (cout, cin, dc.nbasis):
        raise ValueError("tensor shapes do not match the handles")
    y = torch.empty((B, cout, g.nlat_out, g.nlon_out), dtype=x.dtype, device=x.device) if y is None else y
    if workspace is None:
        workspace = torch.empty(max(s2_disco_workspace_bytes(dc, B, cin, cout), 1), dtype=torch.uint8, device=x.device)
    _check(lib().s2_disco_fwd(dc.handle, B, cin, cout, x.data_ptr(), weight.data_ptr(),
                              bias.data_ptr() if bias is not None else None, y.data_ptr(), workspace.data_ptr(),
                              workspace.numel(), _stream()))
    return y, workspace


def s2_disco_bwd(dc, x, weight, dy, workspace, with_bias=True):
    import torch
    _dev(x, weight, dy, workspace)
    B, cin = x.shape[:2]
    cout = weight.shape[0]
    dx, dw = torch.empty_like(x), torch.empty_like(weight)
    db = torch.empty(cout, dtype=x.dtype, device=x.device) if with_bias else None
    _check(lib().s2_disco_bwd(dc.handle, B, cin, cout, x.data_ptr(), weight.data_ptr(), dy.data_ptr(), dx.data_ptr(),
                              dw.data_ptr(), db.data_ptr() if db is not None else None, workspace.data_ptr(),
                              workspace.numel(), _stream()))
    return dx, dw, db


def s2_attn_global_fwd_workspace_bytes(g, batch, heads, d, dtype=S2_BF16):
    return int(lib().s2_attn_global_fwd_workspace_bytes(g.handle, batch, heads, d, dtype))


def s2_attn_global_bwd_workspace_bytes(g, batch, heads, d, dtype=S2_BF16):
    return int(lib().s2_attn_global_bwd_workspace_bytes(g.handle, batch, heads, d, dtype))


def s2_attn_global_fwd(g, q, k, v, scale, out=None, lse=None, workspace=None):
    """Token-major q, k, v [B,H,N,d] -> out [B,H,N,d], lse float32 [B,H,N]."""
    import torch
    _dev(q, k, v)
    B, H, N, d = q.shape
    if N != g.nlat_in * g.nlon_in or k.shape != q.shape or v.shape != q.shape:
        raise ValueError("tensor shapes do not match the grid handle")
    out = torch.empty_like(q) if out is None else out
    lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device) if lse is None else lse
    if workspace is None:
        need = s2_attn_global_fwd_workspace_bytes(g, B, H, d, _dtype_code(q))
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    _dev(out, lse, workspace)
    _check(lib().s2_attn_global_fwd(g.handle, B, H, d, _dtype_code(q), float(scale), q.data_ptr(), k.data_ptr(),
                                    v.data_ptr(), out.data_ptr(), lse.data_ptr(), workspace.data_ptr(),
                                    workspace.numel(), _stream()))
    return out, lse


def s2_attn_global_bwd(g, q, k, v, out, lse, dout, scale, dq=None, dk=None, dv=None, workspace=None):
    import torch
    _dev(q, k, v, out, lse, dout)
    B, H, N, d = q.shape
    if N != g.nlat_in * g.nlon_in or out.shape != q.shape or dout.shape != q.shape or lse.shape != (B, H, N):
        raise ValueError("tensor shapes do not match the grid handle")
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = s2_attn_global_bwd_workspace_bytes(g, B, H, d, _dtype_code(q))
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    _dev(dq, dk, dv, workspace)
    _check(lib().s2_attn_global_bwd(g.handle, B, H, d, _dtype_code(q), float(scale), q.data_ptr(), k.data_ptr(),
                                    v.data_ptr(), out.data_ptr(), lse.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                    dk.data_ptr(), dv.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()))
    return dq, dk, dv


S2_PEAK_COPY, S2_PEAK_FMA_F32, S2_PEAK_MFMA_F32, S2_PEAK_MFMA_BF16, S2_PEAK_LDS_READ = range(5)


def s2_peak_measure(kind):
    """Measured ceiling of the current device (see include/s2attn.h for kinds and units)."""
    val = ctypes.c_double(0.0)
    _check(lib().s2_peak_measure(int(kind), ctypes.byref(val)))
    return float(val.value)


def s2_debug_control(set_bits=0, clear_bits=0):
    """Test-only dispatch switches (S2_DEBUG_*): returns the new flag word."""
    return int(lib().s2_debug_control(int(set_bits), int(clear_bits)))


def s2_trace_enable(on):
    return int(lib().s2_trace_enable(1 if on else 0))


def s2_trace_reset():
    lib().s2_trace_reset()


def s2_trace_entries():
    """[(kernel name, ms, pairs)] of every launch recorded since the last reset (waits for them)."""
    L = lib()
    out = []
    for i in range(L.s2_trace_count()):
        name, ms, pairs = ctypes.c_char_p(), ctypes.c_float(), ctypes.c_double()
        _check(L.s2_trace_get(i, ctypes.byref(name), ctypes.byref(ms), ctypes.byref(pairs)))
        out.append((name.value.decode(), ms.value, pairs.value))
    return out
