"""Host logic of the HIP library (no GPU needed): quadrature, neighbor lists, errors, exported symbols."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import oracle as O
import paper_2505_11157_amd as S
from paper_2505_11157_amd.workloads import grid_dict

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

EXTRA = [
    dict(grid_type=0, nlat_in=17, nlon_in=32, nlat_out=9, nlon_out=16, theta=0.45),
    dict(grid_type=1, nlat_in=12, nlon_in=24, nlat_out=12, nlon_out=24, theta=0.6),
    dict(grid_type=1, nlat_in=16, nlon_in=36, nlat_out=8, nlon_out=12, theta=0.5),
    dict(grid_type=0, nlat_in=9, nlon_in=16, nlat_out=9, nlon_out=16, theta=math.pi),
    dict(grid_type=0, nlat_in=12, nlon_in=15, nlat_out=7, nlon_out=5, theta=1.1),
    dict(grid_type=0, nlat_in=33, nlon_in=64, nlat_out=33, nlon_out=1, theta=0.3),
    dict(grid_type=1, nlat_in=2, nlon_in=1, nlat_out=2, nlon_out=1, theta=0.2),
    # the equiangular grid exactly as the paper prints it (no south pole, trapezoid weights)
    dict(grid_type=2, nlat_in=16, nlon_in=32, nlat_out=16, nlon_out=32, theta=0.45),
    dict(grid_type=2, nlat_in=128, nlon_in=256, nlat_out=128, nlon_out=256, theta=0.1),
    dict(grid_type=2, nlat_in=64, nlon_in=128, nlat_out=32, nlon_out=64, theta=0.2),
    # Gauss-Lobatto nodes in cos(colat): a Gaussian-type grid with both poles
    dict(grid_type=3, nlat_in=17, nlon_in=32, nlat_out=17, nlon_out=32, theta=0.45),
    dict(grid_type=3, nlat_in=129, nlon_in=256, nlat_out=129, nlon_out=256, theta=0.1),
    dict(grid_type=3, nlat_in=65, nlon_in=128, nlat_out=33, nlon_out=64, theta=0.2),
]


def _init(gd):
    return S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])


@pytest.mark.parametrize("gd", [grid_dict(c) for c in (1, 2, 3, 4)] + EXTRA)
def test_neighbor_lists_bit_exact_and_weights(gd):
    g = _init(gd)
    row_ptr, col = S.s2_grid_get_neighbors(g)
    want_ptr, want_col = O.neighbor_csr(**gd)
    assert row_ptr.dtype == np.int64 and col.dtype == np.int32
    assert np.array_equal(row_ptr, want_ptr)
    assert np.array_equal(col, want_col)
    assert S.s2_grid_num_neighbors(g) == len(want_col)
    colat, om = S.s2_grid_get_weights(g)
    ocolat, _ = O.grid(gd["grid_type"], gd["nlat_in"])
    assert np.allclose(colat, ocolat, rtol=0, atol=4e-15)
    assert np.allclose(om, O.omega(gd["grid_type"], gd["nlat_in"], gd["nlon_in"]), rtol=1e-10, atol=0)
    if gd["grid_type"] != 2:
        assert abs(om.sum() * gd["nlon_in"] - 4 * math.pi) < 1e-12
    else:   # the grid of App. A.1: zero weight at the pole, sum only close to 4 pi
        assert om[0] == 0.0 and (om[1:] > 0).all()
        assert abs(om.sum() * gd["nlon_in"] - 4 * math.pi) < 11.0 / gd["nlat_in"] ** 2


def test_init_errors():
    bad = [
        ((5, 17, 32, 17, 32, 0.3), S.S2_ERR_INVALID_ARG),
        ((0, 1, 32, 17, 32, 0.3), S.S2_ERR_INVALID_ARG),
        ((0, 17, 0, 17, 32, 0.3), S.S2_ERR_INVALID_ARG),
        ((0, 17, 32, 17, 32, 0.0), S.S2_ERR_INVALID_ARG),
        ((0, 17, 32, 17, 32, -1.0), S.S2_ERR_INVALID_ARG),
        ((0, 17, 32, 17, 32, 3.5), S.S2_ERR_INVALID_ARG),
        ((0, 17, 32, 17, 32, float("nan")), S.S2_ERR_INVALID_ARG),
        ((0, 17, 32, 17, 24, 0.3), S.S2_ERR_UNSUPPORTED),
        ((1, 4, 8, 64, 8, 0.01), S.S2_ERR_EMPTY_NEIGHBORHOOD),
    ]
    for args, code in bad:
        with pytest.raises(S.S2Error) as ei:
            S.s2_grid_init(*args)
        assert ei.value.code == code, args
        assert S.s2_last_error() != ""


def test_ambiguous_cutoff_rejected():
    # theta chosen so that the equator neighbour at 2 grid steps sits exactly on the inclusion threshold
    with pytest.raises(S.S2Error) as ei:
        S.s2_grid_init(0, 17, 32, 17, 32, math.pi / 8 - 1e-9)
    assert ei.value.code == S.S2_ERR_AMBIGUOUS_CUTOFF


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "s2attn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(s2_[a-z0-9_]+)\s*\(", hdr))
    assert {"s2_grid_init", "s2_grid_destroy", "s2_nattn_fwd", "s2_nattn_bwd", "s2_attn_global_fwd",
            "s2_attn_global_bwd", "s2_last_error"} <= names
    L = ctypes.CDLL(S.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def test_null_arguments_return_codes():
    L = S.lib()
    assert L.s2_grid_init(0, 17, 32, 17, 32, 0.3, None) == S.S2_ERR_INVALID_ARG
    assert L.s2_nattn_fwd(None, 1, 1, 8, 8, 0, 1.0, None, None, None, None, None, None) == S.S2_ERR_INVALID_ARG
    assert L.s2_grid_num_neighbors(None) == 0
    L.s2_grid_destroy(None)


def test_neighborhood_of_zero_weight_points_only_is_rejected():
    # trapezoid grid: the pole row has weight zero; a cutoff below the latitude spacing leaves the pole outputs
    # with pole points only
    with pytest.raises(S.S2Error) as ei:
        S.s2_grid_init(2, 16, 32, 16, 32, 0.1)
    assert ei.value.code == S.S2_ERR_EMPTY_NEIGHBORHOOD
    S.s2_grid_init(2, 16, 32, 16, 32, 0.3)


@pytest.mark.parametrize("gd", [
    dict(grid_type=0, nlat_in=9, nlon_in=16, nlat_out=17, nlon_out=32, theta=0.5),      # upsampling x2
    dict(grid_type=1, nlat_in=8, nlon_in=12, nlat_out=12, nlon_out=36, theta=0.6),      # upsampling x3
    dict(grid_type=0, nlat_in=6, nlon_in=10, nlat_out=9, nlon_out=40, theta=math.pi),   # x4, whole sphere
    dict(grid_type=2, nlat_in=8, nlon_in=16, nlat_out=8, nlon_out=32, theta=0.45),      # x2 on the trapezoid grid
    dict(grid_type=0, nlat_in=17, nlon_in=32, nlat_out=9, nlon_out=16, theta=0.45),     # downsampling
    dict(grid_type=1, nlat_in=12, nlon_in=24, nlat_out=12, nlon_out=24, theta=0.6),     # equal grids
])
def test_neighbor_lists_at_every_output_point(gd):
    # eq. (5) evaluated by the oracle for every (output, input) pair against the library's shift-reused lists
    g = _init(gd)
    for h in range(gd["nlat_out"]):
        for w in range(gd["nlon_out"]):
            want = np.flatnonzero(O.indicator_point(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"],
                                                    gd["nlon_out"], gd["theta"], h, w).reshape(-1))
            got = S.s2_grid_get_neighbors_at(g, h, w)
            assert got.dtype == np.int32 and np.array_equal(got, want), (h, w)


def test_incommensurate_longitudes_rejected():
    with pytest.raises(S.S2Error) as ei:
        S.s2_grid_init(0, 9, 16, 9, 24, 0.5)
    assert ei.value.code == S.S2_ERR_UNSUPPORTED


@pytest.mark.parametrize("seed", range(120))
def test_random_grids_neighbor_lists(seed):
    # seeded random grids (all types, equal / downsampling / upsampling ratios, unequal latitude counts): the library's
    # arc tables, expanded for every output point, against eq. (5) evaluated per pair by the oracle
    rng = np.random.default_rng(5000 + seed)
    gt = int(rng.integers(0, 4))
    nlon_lo = int(rng.integers(1, 14))
    ratio = int(rng.choice([1, 2, 3, 4, 5]))
    up = bool(rng.integers(0, 2))
    nlon_in, nlon_out = (nlon_lo, nlon_lo * ratio) if up else (nlon_lo * ratio, nlon_lo)
    gd = dict(grid_type=gt, nlat_in=int(rng.integers(2, 16)), nlon_in=nlon_in, nlat_out=int(rng.integers(2, 16)),
              nlon_out=nlon_out, theta=float(rng.uniform(0.05, math.pi)))
    masks = [[O.indicator_point(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"],
                                gd["theta"], h, w).reshape(-1) for w in range(nlon_out)] for h in range(gd["nlat_out"])]
    om = O.omega(gt, gd["nlat_in"], nlon_in)
    tok_w = np.repeat(om, nlon_in)
    every_output_sees_weight = all((tok_w[m.astype(bool)] > 0).any() for row in masks for m in row)
    try:
        g = _init(gd)
    except S.S2Error as err:
        assert err.code == S.S2_ERR_EMPTY_NEIGHBORHOOD and not every_output_sees_weight
        return
    assert every_output_sees_weight
    for h in range(gd["nlat_out"]):
        for w in range(nlon_out):
            assert np.array_equal(S.s2_grid_get_neighbors_at(g, h, w), np.flatnonzero(masks[h][w])), (h, w)


def test_debug_switches_and_host_only_handle():
    # the test-only dispatch switches are plain bits; without a HIP device a handle is host-only and every
    # attention call reports S2_ERR_DEVICE instead of launching (or falling back to) anything
    assert S.s2_debug_control(0, 0xFFFFFFFF) == 0
    assert S.s2_debug_control(S.S2_DEBUG_NO_MFMA | S.S2_DEBUG_FAIL_LAUNCH, 0) == 9
    assert S.s2_debug_control(S.S2_DEBUG_NO_STREAM, S.S2_DEBUG_NO_MFMA) == 10
    assert S.s2_debug_control(0, 0xFFFFFFFF) == 0
    import torch
    if torch.cuda.is_available():
        pytest.skip("a device is present: the handle is not host-only")
    g = S.s2_grid_init(0, 9, 16, 9, 16, 0.5)
    L = S.lib()
    buf = (ctypes.c_float * 64)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert L.s2_nattn_fwd(g.handle, 1, 1, 4, 4, S.S2_F32, 1.0, p, p, p, p, p, None) == S.S2_ERR_DEVICE
    assert "no device tables" in S.s2_last_error()
    assert L.s2_nattn_bwd(g.handle, 1, 1, 4, 4, S.S2_F32, 1.0, p, p, p, p, p, p, p, p, p, p, 1 << 20, None) == S.S2_ERR_DEVICE
