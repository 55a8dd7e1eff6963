"""GPU parity of the fp32 band-tile matrix-core kernels (head dimensions 16 and 64 on equal grids; 32 when a test
switch routes it there) against the float64 oracle, through the C ABI, at the stated bound
|x - ref| <= 1e-6 + 1e-5 |ref| (plus the derived rounding allowance of test_gpu_nattn on the peaked cases)."""
import math

import numpy as np
import pytest
import torch

import paper_2505_11157_amd as S
from paper_2505_11157_amd.workloads import make_inputs
from test_gpu_nattn import C_DERIVED, debug_switches, run_case

pytestmark = pytest.mark.gpu


def _c(grid_type, nlat, nlon, theta, batch, heads, d):
    return dict(kind="nattn", grid_type=grid_type, nlat_in=nlat, nlon_in=nlon, nlat_out=nlat, nlon_out=nlon, theta=theta,
                batch=batch, heads=heads, d=d, dtype="f32")


# (grid type, nlat, nlon, theta): whole circles and long arcs on most rows / short arcs with a few polar rows /
# Gauss grid / a ragged last segment of latitudes (nlat not a multiple of four) / one segment only / the grid of
# App. A.1 with its zero-weight pole row / a window that wraps several times around 64 longitudes / bands of 3 rows
SHAPES = [
    (0, 17, 64, 0.9), (0, 33, 192, 0.3), (1, 16, 128, 0.45), (0, 41, 256, 4 * math.pi / 40), (1, 3, 64, 0.7),
    (2, 32, 128, 0.4), (0, 9, 64, math.pi), (0, 9, 256, 0.5), (3, 33, 128, 0.35), (0, 65, 256, 2 * math.pi / 64),
    # longitude counts that leave the last group of a latitude ragged (16, 16 and 48 owners of 64; 16 of 32 at d = 64)
    (0, 21, 80, 0.5), (1, 18, 144, 0.3), (0, 25, 240, 0.2),
]


@pytest.mark.parametrize("d", [16, 64, 32])
@pytest.mark.parametrize("i", range(len(SHAPES)))
def test_band_kernels(i, d):
    gt, nlat, nlon, theta = SHAPES[i]
    c, arrs = make_inputs(_c(gt, nlat, nlon, theta, 1, 3, d), seed=900 + i)
    with debug_switches(S.S2_DEBUG_FORCE_BAND if d == 32 else 0):
        run_case(c, arrs, [0, 2], case="band%d[d%d]" % (i, d))


@pytest.mark.parametrize("i", [1, 12])
def test_band_kernels_d32_many_slices(i):
    # 20 slices (more than two workgroups per compute unit; d = 16 switches from two to four owner tiles per wavefront
    # at that point, see the random shapes): three of them against the oracle
    gt, nlat, nlon, theta = SHAPES[i]
    c, arrs = make_inputs(_c(gt, nlat, nlon, theta, 4, 5, 32), seed=930 + i)
    with debug_switches(S.S2_DEBUG_FORCE_BAND):
        run_case(c, arrs, [0, 7, 19], case="band%d[d32,20 slices]" % i)


@pytest.mark.parametrize("seed", range(30))
def test_band_kernels_random_shapes(seed):
    # seeded random equal grids (all grid types, 5 to 40 latitudes, longitude counts that are multiples of 16 from 64 to
    # 320, random cutoffs, 1 to 24 slices: few and many workgroups, ragged last groups and segments, short arcs, long
    # arcs and whole circles in whatever mix comes up) for d = 16, 32 (routed to the band tiles) and 64; one random slice
    # against the oracle
    rng = np.random.default_rng(8100 + seed)
    d = (16, 32, 64)[seed % 3]
    gt = int(rng.integers(0, 4))
    nlat = int(rng.integers(5, 41))
    nlon = 16 * int(rng.integers(4, 21))
    theta = float(rng.uniform(1.2, 7.0)) * math.pi / nlat
    batch, heads = int(rng.integers(1, 5)), int(rng.integers(1, 7))
    c = _c(gt, nlat, nlon, theta, batch, heads, d)
    try:
        S.s2_grid_init(gt, nlat, nlon, nlat, nlon, theta)
    except S.S2Error as err:
        assert err.code in (S.S2_ERR_EMPTY_NEIGHBORHOOD, S.S2_ERR_AMBIGUOUS_CUTOFF)
        pytest.skip("cutoff rejected for this random grid")
    c, arrs = make_inputs(c, seed=8200 + seed)
    with debug_switches(S.S2_DEBUG_FORCE_BAND if d == 32 else 0):
        run_case(c, arrs, [int(rng.integers(0, batch * heads))], case="band-random%d[d%d]" % (seed, d))


@pytest.mark.parametrize("d", [16, 64])
@pytest.mark.parametrize("factor,sign", [(6.0, 1.0), (6.0, -1.0)])
def test_band_kernels_peaked(d, factor, sign):
    # nearly one-hot softmax (q and k scaled by 6) and a negative scale: the lazy reference maximum moves repeatedly
    for i in (1, 3, 0):
        gt, nlat, nlon, theta = SHAPES[i]
        c, arrs = make_inputs(_c(gt, nlat, nlon, theta, 1, 2, d), seed=950 + i)
        arrs = [arrs[0] * np.float32(factor), arrs[1] * np.float32(factor), arrs[2], arrs[3]]
        c = dict(c, scale=sign / math.sqrt(d))
        run_case(c, arrs, [1], C=C_DERIVED, case="band-peaked%d[d%d,%+g]" % (i, d, sign * factor))


@pytest.mark.parametrize("d", [16, 64])
def test_band_kernels_workload_grid(d):
    # the 129 x 256 grid of the headline workload with other head dimensions: two slices against the oracle
    c, arrs = make_inputs(_c(0, 129, 256, 0.09817477042468103, 1, 3, d), seed=77)
    run_case(c, arrs, [0, 2], case="band129x256[d%d]" % d)


def test_band_kernels_bit_reproducible():
    c, arrs = make_inputs(_c(0, 33, 192, 0.3, 1, 3, 64), seed=5)
    g = S.s2_grid_init(0, 33, 192, 33, 192, 0.3)
    dev = torch.device("cuda:0")
    q, k, v, go = (torch.from_numpy(a).to(dev).reshape((1, 3) + a.shape[1:]).contiguous() for a in arrs)
    ref = None
    for _ in range(20):
        out, lse = S.s2_nattn_fwd(g, q, k, v, 0.125)
        res = (out, lse) + tuple(S.s2_nattn_bwd(g, q, k, v, out, lse, go, 0.125))
        torch.cuda.synchronize()
        if ref is None:
            ref = [r.clone() for r in res]
        else:
            assert all(torch.equal(a, b) for a, b in zip(ref, res))
