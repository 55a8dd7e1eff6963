"""GPU parity of the neighborhood attention on bf16 tensors (through the C ABI) against the float64 oracle.

Inputs are rounded to bf16 before either side sees them.  Tolerance for the bf16 tensors (out, dq, dk, dv):
|x - ref| <= 2e-2 |ref| + 2e-2 rms(ref) elementwise (a pure relative bound is meaningless at zero crossings); the
float32 logsumexp is held to |x - ref| <= 1e-5 + 1e-5 |ref| (it is a float32 sum of exact bf16 products).
dq and dk get one derived allowance on top: the backward forms D_i = dout_i . out_i from the bf16 `out` tensor the
caller hands back, whose elements carry a rounding of up to 2^-9 |out|, so |dD_i| <= 2^-9 sum_c |dout_ic out_ic|; that
error enters dS_ij = p_ij (dout_i.v_j - D_i) for every j at once and propagates linearly:
|d dq_il| <= |scale| dD_i sum_j p_ij |k_jl|,  |d dk_jl| <= |scale| sum_i p_ij dD_i |q_il|  (both sums come from the
oracle: its forward with |k| in place of v, and the dv output of its backward with dD_i |q_i| in place of dout).
It matters only where the softmax is nearly one-hot (a handful of elements per million on the workloads).
Shapes with equal grids, d = e = 32 and a longitude count that is a multiple of 64 run on the bf16 matrix cores
(band tiles); d = e = 16, 32, 64 on other multiples of 16 on the fp32 band tiles with bf16 loads and stores; every other
shape on the shape-agnostic kernels with bf16 loads and stores.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle as O
import paper_2505_11157_amd as S
from paper_2505_11157_amd.workloads import grid_dict, make_inputs, round_to_bf16

pytestmark = pytest.mark.gpu
_REPORT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "parity_report.jsonl")


def _close(x, ref, what, case, f32=False, rel=2e-2, extra=0.0):
    err = np.abs(x - ref)
    rms = np.sqrt((ref ** 2).mean())
    tol = 1e-5 + 1e-5 * np.abs(ref) if f32 else rel * np.abs(ref) + rel * rms + extra
    rec = dict(case=case, what=what, n=int(err.size), max_abs=float(err.max()),
               max_rel_to_ref_plus_rms=float((err / (np.abs(ref) + rms)).max()), rms_ref=float(rms),
               n_over_plain=int((err > rel * np.abs(ref) + rel * rms).sum()) if not f32 else 0)
    print("parity %-24s %-4s max|err| %.3e  max err/(|ref|+rms) %.3e  over the plain bound %d/%d" % (
        case, what, rec["max_abs"], rec["max_rel_to_ref_plus_rms"], rec["n_over_plain"], rec["n"]), flush=True)
    try:
        with open(_REPORT, "a") as f:
            f.write(json.dumps(rec) + "\n")
    except OSError:
        pass
    assert np.isfinite(x).all(), "%s %s: non-finite values" % (case, what)
    assert (err <= tol).all(), "%s %s: max err %.3e, max excess %.3e, %d elements over" % (
        case, what, err.max(), (err - tol).max(), int((err > tol).sum()))


def run_bf16(c, arrs, slices, case, backward=True, scale=None):
    gd = grid_dict(c)
    g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
    B, H, d = c["batch"], c["heads"], c["d"]
    scale = 1 / math.sqrt(d) if scale is None else scale
    arrs = [round_to_bf16(a) for a in arrs]
    dev = torch.device("cuda:0")
    fold = lambda a: torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).to(torch.bfloat16).contiguous()
    q, k, v, dout = (fold(a) for a in arrs)
    out, lse = S.s2_nattn_fwd(g, q, k, v, scale)
    assert out.dtype == torch.bfloat16 and lse.dtype == torch.float32
    res = [out, lse]
    if backward:
        res += list(S.s2_nattn_bwd(g, q, k, v, out, lse, dout, scale))
    torch.cuda.synchronize()
    assert S.s2_grid_device_flags(g) == 0
    res = [t.float().reshape((B * H,) + t.shape[2:]).cpu().numpy().astype(np.float64) for t in res]
    for s in slices:
        sl = slice(s, s + 1)
        a64 = [a[sl].astype(np.float64) for a in arrs]
        brute = gd["nlon_in"] % gd["nlon_out"] != 0
        r_out, r_lse = O.nattn_fwd(gd, a64[0], a64[1], a64[2], scale, brute=brute)
        cs = "%s[%d]" % (case, s)
        _close(res[1][sl], r_lse, "lse", cs, f32=True)
        _close(res[0][sl], r_out, "out", cs)
        if backward:
            r_dq, r_dk, r_dv = O.nattn_bwd(gd, *a64, scale, brute=brute)
            # allowance for D_i formed from the bf16-rounded `out` (see the module docstring)
            dD = 2.0 ** -9 * np.abs(a64[3] * r_out).sum(axis=1, keepdims=True)
            a_dq = abs(scale) * dD * O.nattn_fwd(gd, a64[0], a64[1], np.abs(a64[1]), scale, brute=brute)[0]
            a_dk = abs(scale) * O.nattn_bwd(gd, a64[0], a64[1], a64[1], dD * np.abs(a64[0]), scale, brute=brute)[2]
            _close(res[2][sl], r_dq, "dq", cs, extra=a_dq)
            _close(res[3][sl], r_dk, "dk", cs, extra=a_dk)
            _close(res[4][sl], r_dv, "dv", cs)
    return res


def _c(gt, nlat, nlon, theta, B=1, H=2, d=32, nlat_out=None, nlon_out=None):
    return dict(kind="nattn", grid_type=gt, nlat_in=nlat, nlon_in=nlon, nlat_out=nlat_out or nlat,
                nlon_out=nlon_out or nlon, theta=theta, batch=B, heads=H, d=d, dtype="f32")


# matrix-core path: one and several 256-longitude groups, partial last group (320, 192), arcs from one to dozens of
# offsets and whole circles, all four grid types (the App. A.1 grid has a zero-weight pole row), a disk that covers
# the sphere
FAST = [
    _c(0, 17, 64, 0.5), _c(1, 16, 128, 0.3, B=2, H=1), _c(0, 33, 192, 0.3, H=3), _c(0, 21, 320, 0.25),
    _c(2, 32, 128, 0.3), _c(3, 17, 64, 0.45), _c(0, 9, 64, math.pi), _c(1, 24, 256, 0.12), _c(0, 65, 256, 2 * math.pi / 64),
    _c(0, 13, 512, 0.2, H=1),
]
# shape-agnostic kernels on bf16 tensors: other head widths, 2:1 grids, upsampling, ragged longitude counts
GENERIC = [
    _c(0, 12, 15, 1.1, B=2, H=1, d=5, nlat_out=7, nlon_out=5), _c(1, 24, 70, 0.4, H=1, d=64),
    _c(0, 19, 152, 0.3, H=3, nlat_out=10, nlon_out=76), _c(0, 9, 16, 0.5, d=8, nlat_out=17, nlon_out=32),
    _c(0, 33, 100, 0.3, H=2), _c(2, 16, 32, 0.45, d=8),
]


@pytest.mark.parametrize("ci", range(len(FAST)))
def test_bf16_matrix_core_path(ci):
    c, arrs = make_inputs(FAST[ci], seed=800 + ci)
    S.s2_trace_reset()
    S.s2_trace_enable(True)
    try:
        run_bf16(c, arrs, range(c["batch"] * c["heads"]), "bf16-mc%d" % ci)
        names = {n for n, _, _ in S.s2_trace_entries()}
    finally:
        S.s2_trace_enable(False)
        S.s2_trace_reset()
    assert names and all(n.split("<")[0] in ("nattn_fwd_bf16", "nattn_bwd_dq_bf16", "nattn_bwd_dkdv_bf16") for n in names), names


# fp32 band tiles with bf16 loads and stores: head widths 16 and 64, and d = 32 on longitude counts that are multiples of
# 16 but not of 64 (whole circles near the poles, short arcs, a ragged last group, the zero-weight pole row)
BAND = [
    _c(0, 17, 64, 0.5, d=16), _c(0, 33, 192, 0.3, H=2, d=64), _c(1, 16, 128, 0.3, B=2, H=1, d=16), _c(0, 21, 80, 0.4, d=32),
    _c(2, 32, 144, 0.3, d=64), _c(0, 9, 64, math.pi, d=64),
]


@pytest.mark.parametrize("ci", range(len(BAND)))
def test_bf16_band_tile_path(ci):
    c, arrs = make_inputs(BAND[ci], seed=870 + ci)
    S.s2_trace_reset()
    S.s2_trace_enable(True)
    try:
        run_bf16(c, arrs, range(c["batch"] * c["heads"]), "bf16-band%d" % ci)
        names = {n for n, _, _ in S.s2_trace_entries()}
    finally:
        S.s2_trace_enable(False)
        S.s2_trace_reset()
    assert names == {"nattn_fwd_band<bf16>", "nattn_bwd_dq_band<bf16>", "nattn_bwd_dkdv_band<bf16>"}, names


@pytest.mark.parametrize("ci", range(len(GENERIC)))
def test_bf16_shape_agnostic_path(ci):
    c, arrs = make_inputs(GENERIC[ci], seed=850 + ci)
    run_bf16(c, arrs, range(c["batch"] * c["heads"]), "bf16-gen%d" % ci)


@pytest.mark.parametrize("cfg,slices", [(2, range(8)), (3, [0, 9, 18, 27, 4, 13, 22, 31])])
def test_bf16_workload_shapes(cfg, slices):
    # workloads 2 and 3 with bf16 tensors: all 8 slices, resp. one slice per residue mod 8
    c, arrs = make_inputs(cfg)
    r1 = run_bf16(c, arrs, slices, "bf16-cfg%d" % cfg)
    r2 = run_bf16(c, arrs, [], "bf16-cfg%d" % cfg)
    for a, b in zip(r1, r2):
        assert np.array_equal(a, b)          # no atomics: bit-reproducible


def test_bf16_matches_shape_agnostic_kernels():
    # the two bf16 paths against each other on a matrix-core shape (test-only switch keeps the matrix cores out)
    c, arrs = make_inputs(FAST[2], seed=802)
    r1 = run_bf16(c, arrs, [], "")
    S.s2_debug_control(S.S2_DEBUG_NO_MFMA, 0)
    try:
        r2 = run_bf16(c, arrs, [1], "bf16-gen-on-mc-shape")
    finally:
        S.s2_debug_control(0, S.S2_DEBUG_NO_MFMA)
    for a, b, what in zip(r1, r2, ("out", "lse", "dq", "dk", "dv")):
        rms = np.sqrt((b ** 2).mean())
        assert (np.abs(a - b) <= 3e-2 * np.abs(b) + 3e-2 * rms).all(), what


@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_bf16_peaked_softmax_forward(sign):
    # q and k scaled by 6: nearly one-hot probabilities, the shared reference maximum of an output's four lanes
    # moves many times.  Forward only: with a one-hot softmax dS = p (dout.v - D) cancels to the rounding of the
    # bf16 `out` that D is computed from, and the 2e-2 bound does not apply to the gradients.
    for ci in (2, 4, 8):
        c, arrs = make_inputs(FAST[ci], seed=870 + ci)
        arrs = [arrs[0] * np.float32(6.0), arrs[1] * np.float32(6.0), arrs[2], arrs[3]]
        gd = grid_dict(c)
        B, H, d = c["batch"], c["heads"], c["d"]
        scale = sign / math.sqrt(d)
        arrs = [round_to_bf16(a) for a in arrs]
        g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
        dev = torch.device("cuda:0")
        fold = lambda a: torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).to(torch.bfloat16).contiguous()
        out, lse = S.s2_nattn_fwd(g, fold(arrs[0]), fold(arrs[1]), fold(arrs[2]), scale)
        torch.cuda.synchronize()
        a64 = [a[:1].astype(np.float64) for a in arrs]
        r_out, r_lse = O.nattn_fwd(gd, a64[0], a64[1], a64[2], scale)
        x_lse = lse.reshape((B * H,) + lse.shape[2:])[:1].cpu().numpy().astype(np.float64)
        x_out = out.float().reshape((B * H,) + out.shape[2:])[:1].cpu().numpy().astype(np.float64)
        assert np.isfinite(x_out).all() and np.isfinite(x_lse).all()
        assert np.abs(x_lse - r_lse).max() <= 1e-4 * max(1.0, np.abs(r_lse).max())
        _close(x_out, r_out, "out", "bf16-peaked%d%s" % (ci, "+" if sign > 0 else "-"))


def test_bf16_errors():
    g = S.s2_grid_init(0, 17, 64, 17, 64, 0.5)
    dev = torch.device("cuda:0")
    q = torch.zeros((1, 1, 32, 17, 64), device=dev, dtype=torch.bfloat16)
    out, lse = S.s2_nattn_fwd(g, q, q, q, 1.0)
    with pytest.raises(S.S2Error) as ei:
        S.s2_nattn_bwd(g, q, q, q, out, lse, q, 1.0, workspace=torch.empty(16, dtype=torch.uint8, device=dev))
    assert ei.value.code == S.S2_ERR_WORKSPACE
    torch.cuda.synchronize()
