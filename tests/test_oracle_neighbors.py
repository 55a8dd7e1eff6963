"""Pins for the oracle's geodesic distance and disk indicator (Sec. 3.2 eq. (5), App. B.3)."""
import math
import os

import numpy as np
import pytest

import oracle as O
from indep import dense_mask
from paper_2505_11157_amd.workloads import CONFIGS, grid_dict

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_geodesic_closed_forms():
    assert abs(O.geodesic(0.0, 1.3, 0.7, 2.9) - 0.7) < 1e-15                 # from the pole: the colatitude
    assert abs(O.geodesic(0.4, 1.0, 1.5, 1.0) - 1.1) < 1e-15                 # same meridian
    assert abs(O.geodesic(math.pi / 2, 0.2, math.pi / 2, 1.0) - 0.8) < 1e-15  # along the equator
    assert abs(O.geodesic(0.3, 0.5, math.pi - 0.3, 0.5 + math.pi) - math.pi) < 1e-15  # antipodes
    assert O.geodesic(0.9, 2.0, 0.9, 2.0) == 0.0


def test_geodesic_vs_haversine_and_acos():
    rng = np.random.default_rng(0)
    for _ in range(200):
        t1, t2 = rng.uniform(0, math.pi, 2); p1, p2 = rng.uniform(0, 2 * math.pi, 2)
        d = O.geodesic(t1, p1, t2, p2)
        assert abs(d - O.geodesic(t2, p2, t1, p1)) < 1e-15
        lat1, lat2 = math.pi / 2 - t1, math.pi / 2 - t2
        hav = math.sin((lat2 - lat1) / 2) ** 2 + math.cos(lat1) * math.cos(lat2) * math.sin((p2 - p1) / 2) ** 2
        assert abs(d - 2 * math.asin(math.sqrt(hav))) < 1e-12
        c = math.cos(t1) * math.cos(t2) + math.sin(t1) * math.sin(t2) * math.cos(p1 - p2)
        if abs(c) < 0.999:
            assert abs(d - math.acos(c)) < 1e-12


def test_config1_row_lengths_golden():
    with open(os.path.join(GOLDEN, "config1_row_lengths.txt")) as f:
        want = [int(x) for x in [l for l in f if not l.startswith("#")][0].split()]
    row_ptr, _ = O.neighbor_csr(**grid_dict(1))
    assert list(np.diff(row_ptr)) == want


def test_pole_and_equator_rows_analytic():
    # output at the north pole: member iff colat' <= theta; equator: same-row offsets |w'| <= theta/dlon.
    m = O.indicator(0, 129, 256, 129, 256, 4 * math.pi / 128)
    assert m[0, :5].all() and not m[0, 5:].any()
    eq = m[64, 64]
    assert eq[[0, 1, 2, 3, 4, 252, 253, 254, 255]].all() and eq.sum() == 9
    assert m[64, 60].sum() == 1 and m[64, 60, 0] == 1 and m[64, 59].sum() == 0
    m4 = O.indicator(0, 257, 512, 129, 256, 2 * math.pi / 128)
    assert m4[0, :5].all() and not m4[0, 5:].any()          # input spacing pi/256: 4 rows + pole


@pytest.mark.parametrize("cfg,count,pairs", [(1, 647, 20704), (2, 22170, 2837760), (3, 22439, 5744384),
                                            (4, 26783, 6856448)])
def test_counts_and_structure(cfg, count, pairs):
    g = grid_dict(cfg)
    m = O.indicator(**g)
    assert int(m.sum()) == count
    assert int(m.sum()) * g["nlon_out"] == pairs
    nlon = g["nlon_in"]
    # symmetric in +-w'
    assert (m == np.roll(m[:, :, ::-1], 1, axis=2)).all()
    # each (h, h') segment is one circular interval centred on w' = 0
    cnt = m.sum(axis=2)
    hw = (cnt - 1) // 2
    wp = np.minimum(np.arange(nlon), nlon - np.arange(nlon))
    rebuilt = (wp[None, None, :] <= hw[:, :, None]) & (cnt[:, :, None] > 0)
    rebuilt |= (cnt[:, :, None] == nlon)
    assert (rebuilt == m.astype(bool)).all()
    assert ((cnt % 2 == 1) | (cnt == 0) | (cnt == nlon)).all()
    if g["nlat_in"] == g["nlat_out"] and g["nlon_in"] == g["nlon_out"]:
        assert m[np.arange(g["nlat_out"]), np.arange(g["nlat_out"]), 0].all()          # self
        assert (m == m.transpose(1, 0, 2)).all()     # (h',w') in list(h) <=> (h,-w') in list(h'), with +-w' symmetry


@pytest.mark.parametrize("g", [grid_dict(1),
                               dict(grid_type=0, nlat_in=17, nlon_in=32, nlat_out=9, nlon_out=16, theta=0.45),
                               dict(grid_type=1, nlat_in=12, nlon_in=24, nlat_out=12, nlon_out=24, theta=0.6),
                               dict(grid_type=1, nlat_in=16, nlon_in=36, nlat_out=8, nlon_out=12, theta=0.5)])
def test_shift_form_equals_brute_force_and_chord_formula(g):
    m = O.indicator(**g).astype(bool)
    ps = g["nlon_in"] // g["nlon_out"]
    dm = dense_mask(g).reshape(g["nlat_out"], g["nlon_out"], g["nlat_in"], g["nlon_in"])
    for h in range(g["nlat_out"]):
        for w in range(g["nlon_out"]):
            row = O.indicator_point(h=h, w=w, **g).astype(bool)
            assert (row == np.roll(m[h], w * ps, axis=1)).all()
            assert (row == dm[h, w]).all()


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_formula_independence_full_configs(cfg):
    # shift form (atan2 of cross/dot) against the chord formula, output longitude 0 only.
    g = grid_dict(cfg)
    m = O.indicator(**g).astype(bool)
    from indep import colat_weights, unit_vectors
    ci, _ = colat_weights(g["grid_type"], g["nlat_in"]); co, _ = colat_weights(g["grid_type"], g["nlat_out"])
    xi = unit_vectors(ci, g["nlon_in"]); xo = unit_vectors(co, 1)[:, 0]
    chord2 = ((xo[:, None, None, :] - xi[None]) ** 2).sum(-1)
    assert ((chord2 <= (2 * math.sin((g["theta"] + 1e-9) / 2)) ** 2) == m).all()
    # guard band: nothing sits between the tie tolerance and a visible gap
    d = 2 * np.arcsin(np.minimum(np.sqrt(chord2) / 2, 1.0))
    gap = np.abs(d - g["theta"])
    assert not ((gap > 1e-10) & (gap < 1e-8)).any()


def test_theta_pi_covers_everything():
    m = O.indicator(0, 9, 16, 9, 16, math.pi)
    assert m.all()
    m = O.indicator(1, 8, 16, 8, 16, math.pi)
    assert m.all()


def test_cap_area_sanity():
    g = grid_dict(3)
    m = O.indicator(**g)
    om = O.omega(0, 129, 256)
    area = (m * om[None, :, None]).sum(axis=(1, 2))
    cap = 2 * math.pi * (1 - math.cos(g["theta"]))
    assert np.all(np.abs(area / cap - 1) < 0.3)      # boundary points count in full: not exact
    assert abs(area[20:110].mean() / cap - 1) < 0.08
