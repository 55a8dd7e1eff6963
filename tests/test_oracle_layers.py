"""Pins for the oracle's layer functions (Sec. 3.4 attention sub-block; App. B.3 DISCO convolution): an independent
dense formulation in torch float64 (own quadrature weights, own disk membership from chord lengths, own distances)
with gradients from autograd, plus closed-form special cases."""
import math

import numpy as np
import pytest
import torch

import oracle as O
from indep import colat_weights, dense_mask, log_omega_tokens, unit_vectors

GRIDS = [
    dict(grid_type=0, nlat_in=9, nlon_in=16, nlat_out=9, nlon_out=16, theta=0.6),
    dict(grid_type=1, nlat_in=8, nlon_in=12, nlat_out=8, nlon_out=12, theta=0.9),
]


def _mha_params(rng, C):
    w = lambda: rng.standard_normal((C, C)) / math.sqrt(C)
    b = lambda: 0.3 * rng.standard_normal(C)
    return dict(gamma=1 + 0.2 * rng.standard_normal(C), beta=b(), Wq=w(), bq=b(), Wk=w(), bk=b(), Wv=w(), bv=b(), Wo=w(), bo=b())


def dense_mha(g, heads, x, pos, p, dy=None, eps=1e-5):
    """The attention sub-block in torch float64: explicit moments, channel matrices as matmuls, dense masked softmax."""
    T = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    xt, post = T(x), T(pos)
    pt = {k: T(v) for k, v in p.items()}
    B, C, H, W = x.shape
    N = H * W
    d = C // heads
    xf = xt.reshape(B, C, N)
    mu = xf.mean(-1, keepdim=True)
    var = ((xf - mu) ** 2).mean(-1, keepdim=True)
    xhat = (xf - mu) / torch.sqrt(var + eps)
    xn = pt["gamma"][None, :, None] * xhat + pt["beta"][None, :, None] + post.reshape(C, N)[None]
    proj = lambda Wn, bn, t: torch.matmul(pt[Wn], t) + pt[bn][None, :, None]
    q, k, v = proj("Wq", "bq", xn), proj("Wk", "bk", xn), proj("Wv", "bv", xn)
    hd = lambda t: t.reshape(B, heads, d, N).transpose(2, 3)            # [B, heads, N, d]
    bias = torch.tensor(log_omega_tokens(g))[None, None, None, :]
    neg = torch.where(torch.tensor(dense_mask(g)), 0.0, -np.inf).to(torch.float64)[None, None]
    logits = hd(q) @ hd(k).transpose(2, 3) / math.sqrt(d) + bias + neg
    a = (torch.softmax(logits, -1) @ hd(v)).transpose(2, 3).reshape(B, C, N)
    y = xf + proj("Wo", "bo", a)
    res = {"y": y.detach().numpy().reshape(x.shape)}
    if dy is not None:
        (y * torch.tensor(np.asarray(dy, np.float64)).reshape(B, C, N)).sum().backward()
        res["dx"], res["dpos"] = xt.grad.numpy(), post.grad.numpy()
        for k_, v_ in pt.items():
            res["d" + k_] = v_.grad.numpy()
    return res


@pytest.mark.parametrize("gi", range(len(GRIDS)))
def test_mha_block_vs_dense_torch(gi):
    g = GRIDS[gi]
    rng = np.random.default_rng(50 + gi)
    B, C, heads = 2, 8, 2
    shp = (B, C, g["nlat_in"], g["nlon_in"])
    x, dy = rng.standard_normal(shp), rng.standard_normal(shp)
    pos = 0.5 * rng.standard_normal(shp[1:])
    p = _mha_params(rng, C)
    args = (p["gamma"], p["beta"], p["Wq"], p["bq"], p["Wk"], p["bk"], p["Wv"], p["bv"], p["Wo"], p["bo"])
    y, _ = O.mha_fwd(g, heads, x, pos, *args)
    grads = O.mha_bwd(g, heads, x, pos, *args, dy)
    ref = dense_mha(g, heads, x, pos, p, dy)
    assert np.allclose(y, ref["y"], rtol=1e-10, atol=1e-11)
    for name in ("dx", "dpos", "dgamma", "dbeta", "dWq", "dbq", "dWk", "dbk", "dWv", "dbv", "dWo", "dbo"):
        assert np.allclose(grads[name], ref[name], rtol=1e-9, atol=1e-10), name


def test_mha_block_special_cases():
    # Wo = 0, bo = 0: the block is the identity; Wq = Wk = 0: uniform logits, the attention output is the local
    # omega-weighted mean of v, so with v constant over the grid (Wv = 0, bv = c) y = x + Wo c + bo
    g = GRIDS[0]
    rng = np.random.default_rng(7)
    B, C, heads = 1, 4, 2
    shp = (B, C, g["nlat_in"], g["nlon_in"])
    x, pos = rng.standard_normal(shp), rng.standard_normal(shp[1:])
    p = _mha_params(rng, C)
    z = np.zeros((C, C))
    y, _ = O.mha_fwd(g, heads, x, pos, p["gamma"], p["beta"], p["Wq"], p["bq"], p["Wk"], p["bk"], p["Wv"], p["bv"], z, np.zeros(C))
    assert np.array_equal(y, x)
    y, _ = O.mha_fwd(g, heads, x, pos, p["gamma"], p["beta"], z, p["bq"], z, p["bk"], z, p["bv"], p["Wo"], p["bo"])
    want = x + (p["Wo"] @ p["bv"] + p["bo"])[None, :, None, None]
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------------------------------------------- DISCO

def dense_disco(g, K, x, weight, bias, dy=None):
    """Dense DISCO convolution in torch float64: Psi[k, i, j] from pairwise angles of unit vectors."""
    ci, wl = colat_weights(g["grid_type"], g["nlat_in"])
    co, _ = colat_weights(g["grid_type"], g["nlat_out"])
    xi = unit_vectors(ci, g["nlon_in"]).reshape(-1, 3)
    xo = unit_vectors(co, g["nlon_out"]).reshape(-1, 3)
    chord = np.sqrt(((xo[:, None, :] - xi[None, :, :]) ** 2).sum(-1))
    r = 2.0 * np.arcsin(np.clip(chord / 2.0, 0.0, 1.0))                # angle from the chord length
    om = np.repeat(wl * 2.0 * np.pi / g["nlon_in"], g["nlon_in"])
    dr = g["theta"] / K
    inside = dense_mask(g)
    Psi = np.stack([np.where(inside, np.maximum(0.0, 1.0 - np.abs(r / dr - k)), 0.0) * om[None, :] for k in range(K)])
    B, C = x.shape[:2]
    xt = torch.tensor(np.asarray(x, np.float64).reshape(B, C, -1), requires_grad=True)
    wt = torch.tensor(np.asarray(weight, np.float64), requires_grad=True)
    bt = torch.tensor(np.asarray(bias, np.float64), requires_grad=True)
    z = torch.einsum("kij,bcj->bcki", torch.tensor(Psi), xt)
    y = torch.einsum("ock,bcki->boi", wt, z) + bt[None, :, None]
    so = (g["nlat_out"], g["nlon_out"])
    res = {"y": y.detach().numpy().reshape((B, -1) + so)}
    if dy is not None:
        (y * torch.tensor(np.asarray(dy, np.float64).reshape(B, -1, so[0] * so[1]))).sum().backward()
        res.update(dx=xt.grad.numpy().reshape(x.shape), dweight=wt.grad.numpy(), dbias=bt.grad.numpy())
    return res


DISCO_GRIDS = GRIDS + [dict(grid_type=0, nlat_in=13, nlon_in=24, nlat_out=7, nlon_out=12, theta=0.7)]


@pytest.mark.parametrize("gi", range(len(DISCO_GRIDS)))
def test_disco_vs_dense_torch(gi):
    g = DISCO_GRIDS[gi]
    rng = np.random.default_rng(70 + gi)
    B, C, Oc, K = 2, 3, 4, 3
    x = rng.standard_normal((B, C, g["nlat_in"], g["nlon_in"]))
    dy = rng.standard_normal((B, Oc, g["nlat_out"], g["nlon_out"]))
    weight, bias = rng.standard_normal((Oc, C, K)), rng.standard_normal(Oc)
    y, _ = O.disco_fwd(g, K, x, weight, bias)
    dx, dw, db = O.disco_bwd(g, K, x, weight, bias, dy)
    ref = dense_disco(g, K, x, weight, bias, dy)
    assert np.allclose(y, ref["y"], rtol=1e-9, atol=1e-11)       # distances: atan2 form vs chord form
    assert np.allclose(dx, ref["dx"], rtol=1e-9, atol=1e-11)
    assert np.allclose(dw, ref["dweight"], rtol=1e-9, atol=1e-10)
    assert np.allclose(db, ref["dbias"], rtol=1e-12, atol=1e-12)


def test_disco_constant_field_and_partition_of_unity():
    # the hats sum to one for r <= theta - dr, so with all basis weights equal to one a constant field x = c gives
    # y(h, w) = c * sum over the disk of omega * s(r), s = 1 inside radius theta (K-1)/K, falling linearly to 0 at theta;
    # for a small disk that is c * [cap area of the inner radius + the linear rim], up to quadrature error
    g = dict(grid_type=1, nlat_in=48, nlon_in=96, nlat_out=48, nlon_out=96, theta=0.5)
    K, c = 4, 1.7
    x = np.full((1, 1, 48, 96), c)
    y, z = O.disco_fwd(g, K, x, np.ones((1, 1, K)), np.zeros(1))
    th, r0 = g["theta"], g["theta"] * (K - 1) / K
    # integral over the sphere of s(r): 2 pi [ (1 - cos r0) + int_{r0}^{th} (th - r)/(th - r0) sin r dr ]
    rim = ((th - r0) * math.cos(r0) - (math.sin(th) - math.sin(r0))) / (th - r0)
    exact = c * 2 * math.pi * ((1 - math.cos(r0)) + rim)
    mid = y[0, 0, 8:40]          # away from the poles the quadrature of the non-smooth integrand is accurate to a few %
    assert np.abs(mid - exact).max() < 0.04 * exact
    # exact longitude invariance of a constant field, and the k = 0 hat alone sees only r < dr
    assert np.abs(y - y[..., :1]).max() < 1e-13
    assert (z[0, 0, 0] > 0).all() and z[0, 0, 0].max() < c * 2 * math.pi * (1 - math.cos(th / K)) * 1.3


def test_disco_longitude_shift_equivariance():
    g = DISCO_GRIDS[2]
    rng = np.random.default_rng(3)
    x = rng.standard_normal((1, 2, g["nlat_in"], g["nlon_in"]))
    weight, bias = rng.standard_normal((3, 2, 2)), rng.standard_normal(3)
    y, _ = O.disco_fwd(g, 2, x, weight, bias)
    ps = g["nlon_in"] // g["nlon_out"]
    y2, _ = O.disco_fwd(g, 2, np.roll(x, ps, axis=3), weight, bias)
    assert np.allclose(y2, np.roll(y, 1, axis=3), rtol=0, atol=1e-13)
