"""Pins for the oracle's grids and quadrature weights (App. A.1, Sec. 3.3)."""
import math

import numpy as np
import pytest

import oracle as O
from indep import colat_weights


@pytest.mark.parametrize("gt,nlat,nlon", [(0, 17, 32), (0, 129, 256), (0, 257, 512), (0, 65, 128), (0, 18, 7),
                                          (1, 64, 128), (1, 5, 8), (1, 33, 64)])
def test_weights_sum_to_4pi(gt, nlat, nlon):
    om = O.omega(gt, nlat, nlon)
    assert abs(om.sum() * nlon - 4 * math.pi) < 1e-13 * 4 * math.pi * 4
    assert (om > 0).all()
    assert np.allclose(om, om[::-1], rtol=1e-13, atol=0)   # north-south symmetry


@pytest.mark.parametrize("nlat", [17, 65, 129, 257])
def test_clenshaw_curtis_pole_weight_closed_form(nlat):
    n = nlat - 1
    _, w = O.grid(O.EQUIANGULAR, nlat)
    assert abs(w[0] - 1.0 / (n * n - 1)) < 1e-16 + 1e-13 / (n * n - 1)
    assert abs(w[-1] - 1.0 / (n * n - 1)) < 1e-16 + 1e-13 / (n * n - 1)


@pytest.mark.parametrize("nlat", [5, 6, 17, 33])
def test_clenshaw_curtis_exact_on_polynomials(nlat):
    # int_0^pi cos^m(t) sin(t) dt = 2/(m+1) for even m, 0 for odd m; exact up to degree n.
    t, w = O.grid(O.EQUIANGULAR, nlat)
    assert np.allclose(t, np.pi * np.arange(nlat) / (nlat - 1), rtol=0, atol=1e-15)
    for m in range(nlat):
        exact = 2.0 / (m + 1) if m % 2 == 0 else 0.0
        assert abs((w * np.cos(t) ** m).sum() - exact) < 1e-13, m


@pytest.mark.parametrize("nlat", [4, 17, 129])
def test_clenshaw_curtis_vs_moment_solve(nlat):
    t, w = O.grid(O.EQUIANGULAR, nlat)
    t2, w2 = colat_weights(0, nlat)
    assert np.allclose(t, t2, rtol=0, atol=1e-15)
    assert np.allclose(w, w2, rtol=1e-9, atol=1e-13)


def test_legendre_gauss_textbook_small():
    t, w = O.grid(O.LEGENDRE_GAUSS, 2)
    assert np.allclose(np.cos(t), [1 / math.sqrt(3), -1 / math.sqrt(3)], atol=1e-15)
    assert np.allclose(w, [1, 1], atol=1e-15)
    t, w = O.grid(O.LEGENDRE_GAUSS, 3)
    assert np.allclose(np.cos(t), [math.sqrt(0.6), 0, -math.sqrt(0.6)], atol=1e-15)
    assert np.allclose(w, [5 / 9, 8 / 9, 5 / 9], atol=1e-15)
    t, w = O.grid(O.LEGENDRE_GAUSS, 4)
    a = math.sqrt(3 / 7 - 2 / 7 * math.sqrt(6 / 5)); b = math.sqrt(3 / 7 + 2 / 7 * math.sqrt(6 / 5))
    assert np.allclose(np.cos(t), [b, a, -a, -b], atol=1e-15)
    wa = (18 + math.sqrt(30)) / 36; wb = (18 - math.sqrt(30)) / 36
    assert np.allclose(w, [wb, wa, wa, wb], atol=1e-15)


@pytest.mark.parametrize("nlat", [8, 64, 128])
def test_legendre_gauss_vs_numpy_and_exactness(nlat):
    t, w = O.grid(O.LEGENDRE_GAUSS, nlat)
    t2, w2 = colat_weights(1, nlat)
    assert np.allclose(t, t2, rtol=0, atol=1e-14)
    assert np.allclose(w, w2, rtol=1e-10, atol=0)   # numpy's eigenvalue route is the looser of the two
    assert (np.diff(t) > 0).all()             # north first
    x = np.cos(t)
    for m in range(0, min(2 * nlat, 40)):     # exact to degree 2n-1
        exact = 2.0 / (m + 1) if m % 2 == 0 else 0.0
        assert abs((w * x ** m).sum() - exact) < 1e-13


def test_bad_grid_rejected():
    with pytest.raises(ValueError):
        O.grid(0, 1)
    with pytest.raises(ValueError):
        O.grid(7, 16)


@pytest.mark.parametrize("nlat,nlon", [(8, 16), (65, 128), (128, 256), (257, 7)])
def test_trapezoid_grid_of_the_paper(nlat, nlon):
    # App. A.1: colat_i = pi i / nlat for i < nlat, q_ij = 2 pi^2 / (nlat nlon) sin(colat_i).
    # Closed form of the sum: sum_i sin(pi i / n) = cot(pi / (2n)), so the weights add up to
    # (2 pi^2 / n) cot(pi / (2n)) = 4 pi - pi^3 / (3 n^2) + O(n^-4): "approximately 4 pi".
    colat, w = O.grid(O.EQUIANGULAR_TRAPEZOID, nlat)
    om = O.omega(O.EQUIANGULAR_TRAPEZOID, nlat, nlon)
    assert colat[0] == 0.0 and om[0] == 0.0                      # north pole, weight zero
    assert np.allclose(np.diff(colat), math.pi / nlat, rtol=0, atol=1e-15)
    assert abs(colat[-1] - math.pi * (nlat - 1) / nlat) < 1e-15   # the south pole is not a grid point
    i = np.arange(nlat)
    assert np.allclose(om, 2 * math.pi ** 2 / (nlat * nlon) * np.sin(math.pi * i / nlat), rtol=1e-14, atol=0)
    total = om.sum() * nlon
    assert abs(total - 2 * math.pi ** 2 / nlat / math.tan(math.pi / (2 * nlat))) < 1e-12
    assert abs(total - (4 * math.pi - math.pi ** 3 / (3 * nlat ** 2))) < 2.0 / nlat ** 4 * 10
    # trapezoid rule in colatitude: exact for the first cosine mode only up to O(n^-2)
    assert abs((w * np.cos(colat) ** 2).sum() - 2.0 / 3.0) < 3.0 / nlat ** 2


def test_gauss_lobatto_textbook_small():
    # n = 3: nodes 1, 0, -1, weights 1/3, 4/3, 1/3 (Simpson); n = 4: +-1, +-1/sqrt(5), weights 1/6, 5/6;
    # n = 5: +-1, +-sqrt(3/7), 0, weights 1/10, 49/90, 32/45
    table = {3: ([1, 0, -1], [1 / 3, 4 / 3, 1 / 3]),
             4: ([1, 1 / math.sqrt(5), -1 / math.sqrt(5), -1], [1 / 6, 5 / 6, 5 / 6, 1 / 6]),
             5: ([1, math.sqrt(3 / 7), 0, -math.sqrt(3 / 7), -1], [1 / 10, 49 / 90, 32 / 45, 49 / 90, 1 / 10])}
    for n, (x, w) in table.items():
        colat, wl = O.grid(O.LEGENDRE_GAUSS_LOBATTO, n)
        assert np.allclose(np.cos(colat), x, rtol=0, atol=1e-15)
        assert np.allclose(wl, w, rtol=1e-14, atol=0)


@pytest.mark.parametrize("nlat", [6, 33, 128])
def test_gauss_lobatto_exactness_and_independent_construction(nlat):
    from indep import colat_weights
    colat, w = O.grid(O.LEGENDRE_GAUSS_LOBATTO, nlat)
    x = np.cos(colat)
    assert colat[0] == 0.0 and abs(colat[-1] - math.pi) < 1e-15 and (np.diff(colat) > 0).all()
    assert abs(w.sum() - 2.0) < 1e-13 and (w > 0).all()
    assert abs(w[0] - 2.0 / (nlat * (nlat - 1))) < 1e-16            # pole weight, closed form
    assert np.allclose(w, w[::-1], rtol=1e-12) and np.allclose(x, -x[::-1], atol=1e-15)
    # exact for polynomials up to degree 2n - 3, and not beyond
    for k in range(0, 2 * nlat - 2):
        exact = 2.0 / (k + 1) if k % 2 == 0 else 0.0
        assert abs((w * x ** k).sum() - exact) < 1e-13, k
    k = 2 * nlat - 2
    assert abs((w * x ** k).sum() - 2.0 / (k + 1)) > (1e-9 if nlat < 20 else 0.0)
    ic, iw = colat_weights(3, nlat)      # numpy's root finder + a moment solve in the Legendre basis
    assert np.allclose(ic, colat, rtol=0, atol=1e-10) and np.allclose(iw, w, rtol=0, atol=1e-10)
    om = O.omega(O.LEGENDRE_GAUSS_LOBATTO, nlat, 24)
    assert abs(om.sum() * 24 - 4 * math.pi) < 1e-12
