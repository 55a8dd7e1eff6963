"""CPU oracle for the layers around the attention kernels: the spherical multi-head attention sub-block
(Sec. 3.4, "Spherical attention blocks") and the discrete-continuous (DISCO) convolution (App. B.3, first equation).

TEST INFRASTRUCTURE ONLY (see the header of s2_oracle.c).  Plain numpy float64 written from the definitions, one
step per line, with the attention itself delegated to the C oracle.  Gradients are written out by the chain rule;
tests pin them against torch autograd through an independent dense formulation.

Attention sub-block (pre-norm, residual; Sec. 3.4), x: [B, C, nlat, nlon], self-attention on one grid:
    xhat = (x - mean_hw x) / sqrt(var_hw x + eps)                  instance normalisation per (b, c); the paper names
                                                                   the operation only: plain (unweighted) moments over
                                                                   the grid points, biased variance, affine gamma/beta
    xn   = gamma xhat + beta + pos                                 position embedding added before the attention
    q, k, v = Wq xn + bq, Wk xn + bk, Wv xn + bv                   1x1 convolutions = channel matrices
    a    = attention per head (C = heads * d, head i takes channels i d .. (i+1) d - 1), logits q.k / sqrt(d)
    y    = x + Wo a + bo

DISCO convolution (App. B.3): psi_k[h, h', w'] are K basis functions supported on the geodesic disk of radius
theta_cutoff around the output point (h, longitude 0), multiplied by the quadrature weight of the input point:
    z[b, c, k, h, w] = sum_{h', w'} psi_k[h, h', w'] omega[h'] x[b, c, h', (w' + w pscale) mod nlon_in]
    y[b, o, h, w]    = sum_{c, k} weight[o, c, k] z[b, c, k, h, w] + bias[o]
Basis (the paper leaves it open, its only requirement is support on the disk): K piecewise-linear hat functions of
the geodesic distance r, psi_k(r) = max(0, 1 - |r / dr - k|), dr = theta_cutoff / K, k = 0 .. K-1, so that psi_k
vanishes at r = theta_cutoff (isotropic filters).
"""
import math

import numpy as np

from . import s2_oracle as O


def _heads(t, heads):
    B, C = t.shape[:2]
    return t.reshape((B * heads, C // heads) + t.shape[2:])


def _unheads(t, B):
    return t.reshape((B, -1) + t.shape[2:])


def mha_fwd(g, heads, x, pos, gamma, beta, Wq, bq, Wk, bk, Wv, bv, Wo, bo, eps=1e-5):
    """Returns y and the intermediates the backward needs (dict)."""
    x = np.asarray(x, np.float64)
    B, C = x.shape[:2]
    d = C // heads
    mean = x.mean(axis=(2, 3), keepdims=True)
    var = ((x - mean) ** 2).mean(axis=(2, 3), keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mean) * rstd
    xn = gamma[None, :, None, None] * xhat + beta[None, :, None, None] + pos[None]
    proj = lambda W, b, t: np.einsum("oc,bchw->bohw", W, t) + b[None, :, None, None]
    q, k, v = proj(Wq, bq, xn), proj(Wk, bk, xn), proj(Wv, bv, xn)
    scale = 1.0 / math.sqrt(d)
    a, lse = O.nattn_fwd(g, _heads(q, heads), _heads(k, heads), _heads(v, heads), scale)
    a = _unheads(a, B)
    y = x + proj(Wo, bo, a)
    return y, dict(xhat=xhat, rstd=rstd, xn=xn, q=q, k=k, v=v, a=a, scale=scale)


def mha_bwd(g, heads, x, pos, gamma, beta, Wq, bq, Wk, bk, Wv, bv, Wo, bo, dy, eps=1e-5):
    """Gradients of sum(dy * y) w.r.t. x, pos, gamma, beta and the four projections (dict)."""
    dy = np.asarray(dy, np.float64)
    y, s = mha_fwd(g, heads, x, pos, gamma, beta, Wq, bq, Wk, bk, Wv, bv, Wo, bo, eps)
    B = dy.shape[0]
    res = {}
    # y = x + Wo a + bo
    res["dWo"] = np.einsum("bohw,bchw->oc", dy, s["a"])
    res["dbo"] = dy.sum(axis=(0, 2, 3))
    da = np.einsum("oc,bohw->bchw", Wo, dy)
    # attention per head
    dq, dk, dv = O.nattn_bwd(g, _heads(s["q"], heads), _heads(s["k"], heads), _heads(s["v"], heads), _heads(da, heads),
                             s["scale"])
    dq, dk, dv = _unheads(dq, B), _unheads(dk, B), _unheads(dv, B)
    # projections
    dxn = np.zeros_like(dy)
    for name, W, dt in (("q", Wq, dq), ("k", Wk, dk), ("v", Wv, dv)):
        res["dW" + name] = np.einsum("bohw,bchw->oc", dt, s["xn"])
        res["db" + name] = dt.sum(axis=(0, 2, 3))
        dxn += np.einsum("oc,bohw->bchw", W, dt)
    # xn = gamma xhat + beta + pos
    res["dpos"] = dxn.sum(axis=0)
    res["dgamma"] = (dxn * s["xhat"]).sum(axis=(0, 2, 3))
    res["dbeta"] = dxn.sum(axis=(0, 2, 3))
    dxhat = dxn * gamma[None, :, None, None]
    # instance normalisation: xhat = (x - mean) rstd over the grid points of one (b, c)
    m1 = dxhat.mean(axis=(2, 3), keepdims=True)
    m2 = (dxhat * s["xhat"]).mean(axis=(2, 3), keepdims=True)
    res["dx"] = dy + s["rstd"] * (dxhat - m1 - s["xhat"] * m2)
    res["intermediates"] = dict(dq=dq, dk=dk, dv=dv, dxn=dxn, da=da, xn=s["xn"], xhat=s["xhat"], a=s["a"])
    return res


# ------------------------------------------------------------------------------------------------ DISCO convolution

def disco_psi(g, K):
    """psi[k, h, h', w'] (with the quadrature weight of the input point folded in) for the output point at longitude 0:
    zero outside the disk d <= theta_cutoff + 1e-9."""
    colat_i, wlat = O.grid(g["grid_type"], g["nlat_in"])
    colat_o, _ = O.grid(g["grid_type"], g["nlat_out"])
    omega = wlat * (2.0 * np.pi / g["nlon_in"])
    mask = O.indicator(g["grid_type"], g["nlat_in"], g["nlon_in"], g["nlat_out"], g["nlon_out"], g["theta"])
    psi = np.zeros((K, g["nlat_out"], g["nlat_in"], g["nlon_in"]))
    dr = g["theta"] / K
    for h in range(g["nlat_out"]):
        for hp in range(g["nlat_in"]):
            for wp in range(g["nlon_in"]):
                if not mask[h, hp, wp]:
                    continue
                r = O.geodesic(colat_o[h], 0.0, colat_i[hp], 2.0 * np.pi * wp / g["nlon_in"])
                for k in range(K):
                    psi[k, h, hp, wp] = max(0.0, 1.0 - abs(r / dr - k)) * omega[hp]
    return psi


def disco_fwd(g, K, x, weight, bias):
    """x [B, C, nlat_in, nlon_in], weight [O, C, K], bias [O] -> y [B, O, nlat_out, nlon_out], z [B, C, K, nlat_out, nlon_out]."""
    x = np.asarray(x, np.float64)
    psi = disco_psi(g, K)
    ps = g["nlon_in"] // g["nlon_out"]
    B, C = x.shape[:2]
    z = np.zeros((B, C, K, g["nlat_out"], g["nlon_out"]))
    for w in range(g["nlon_out"]):
        xs = np.roll(x, -w * ps, axis=3)                       # xs[..., w'] = x[..., (w' + w pscale) mod nlon_in]
        z[:, :, :, :, w] = np.einsum("khpw,bcpw->bckh", psi, xs)
    y = np.einsum("ock,bckhw->bohw", weight, z) + bias[None, :, None, None]
    return y, z


def disco_bwd(g, K, x, weight, bias, dy):
    """Gradients of sum(dy * y): dx, dweight, dbias."""
    dy = np.asarray(dy, np.float64)
    psi = disco_psi(g, K)
    ps = g["nlon_in"] // g["nlon_out"]
    _, z = disco_fwd(g, K, x, weight, bias)
    dweight = np.einsum("bohw,bckhw->ock", dy, z)
    dbias = dy.sum(axis=(0, 2, 3))
    dz = np.einsum("ock,bohw->bckhw", weight, dy)
    dx = np.zeros_like(np.asarray(x, np.float64))
    for w in range(g["nlon_out"]):
        # z[..., h, w] = sum psi[k, h, h', w'] x[h', w' + w ps]  =>  dx[h', w' + w ps] += psi[k, h, h', w'] dz[k, h, w]
        contrib = np.einsum("khpw,bckh->bcpw", psi, dz[:, :, :, :, w])
        dx += np.roll(contrib, w * ps, axis=3)
    return dx, dweight, dbias
