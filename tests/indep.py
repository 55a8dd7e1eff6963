"""Independent formulations used to pin the oracle (tests only).

Nothing here is shared with oracle/ or with the HIP library: quadrature
weights come from the exactness conditions solved as a linear system (or from
numpy's Gauss-Legendre routine), disk membership from the chord length of unit
vectors, and attention from a dense masked softmax in torch float64 whose
gradients come from autograd.
"""
import numpy as np
import torch

EQUIANGULAR = 0
LEGENDRE_GAUSS = 1
EQUIANGULAR_TRAPEZOID = 2
LEGENDRE_GAUSS_LOBATTO = 3
TIE_TOL = 1e-9


def colat_weights(grid_type, nlat):
    """Latitude nodes/weights for int f(t) sin(t) dt over [0, pi], NOT via the oracle's formulas."""
    if grid_type == LEGENDRE_GAUSS:
        x, w = np.polynomial.legendre.leggauss(nlat)
        order = np.argsort(-x)
        return np.arccos(x[order]), w[order]
    if grid_type == LEGENDRE_GAUSS_LOBATTO:
        # nodes: +-1 and the roots of the derivative of P_{n-1}, from numpy's polynomial class; weights from the
        # exactness conditions sum_i w_i P_k(x_i) = int_{-1}^{1} P_k dx = 2 [k = 0] for k = 0..n-1 (the Legendre
        # basis keeps the linear system well conditioned)
        m = nlat - 1
        inner = np.polynomial.legendre.Legendre.basis(m).deriv().roots().real if m > 1 else np.zeros(0)
        x = np.sort(np.concatenate([[-1.0], inner, [1.0]]))[::-1]
        A = np.polynomial.legendre.legvander(x, m).T
        rhs = np.zeros(nlat)
        rhs[0] = 2.0
        return np.arccos(np.clip(x, -1.0, 1.0)), np.linalg.solve(A, rhs)
    if grid_type == EQUIANGULAR_TRAPEZOID:
        # composite trapezoid rule for f(t) sin(t) on [0, pi] with nlat intervals; both end points carry sin = 0,
        # which is why the south pole can be left out of the grid
        t = np.linspace(0.0, np.pi, nlat + 1)
        w = np.full(nlat + 1, np.pi / nlat)
        w[[0, -1]] *= 0.5
        return t[:-1], (w * np.sin(t))[:-1]
    # Clenshaw-Curtis: the unique weights on t_h = pi h / n that integrate
    # cos(m t) sin(t) exactly for m = 0..n; moments: (1 + cos(m pi)) / (1 - m^2), 0 for m = 1.
    n = nlat - 1
    t = np.pi * np.arange(nlat) / n
    m = np.arange(nlat)
    A = np.cos(np.outer(m, t))
    rhs = np.where(m == 1, 0.0, (1.0 + np.cos(m * np.pi)) / (1.0 - np.where(m == 1, 0, m).astype(float) ** 2))
    return t, np.linalg.solve(A, rhs)


def unit_vectors(colat, nlon):
    lon = 2.0 * np.pi * np.arange(nlon) / nlon
    st, ct = np.sin(colat)[:, None], np.cos(colat)[:, None]
    return np.stack([st * np.cos(lon)[None, :], st * np.sin(lon)[None, :], np.broadcast_to(ct, (len(colat), nlon))], -1)


def dense_mask(g):
    """bool [N_out, N_in]: chord(x_i, x_j) <= 2 sin((theta + tol)/2), every pair evaluated directly."""
    ci, _ = colat_weights(g["grid_type"], g["nlat_in"])
    co, _ = colat_weights(g["grid_type"], g["nlat_out"])
    xi = unit_vectors(ci, g["nlon_in"]).reshape(-1, 3)
    xo = unit_vectors(co, g["nlon_out"]).reshape(-1, 3)
    out = np.empty((xo.shape[0], xi.shape[0]), bool)
    if g["theta"] + TIE_TOL >= np.pi:       # the disk is the whole sphere
        out[:] = True
        return out
    lim = (2.0 * np.sin((g["theta"] + TIE_TOL) / 2.0)) ** 2
    for s in range(0, xo.shape[0], 512):
        diff = xo[s:s + 512, None, :] - xi[None, :, :]
        out[s:s + 512] = (diff * diff).sum(-1) <= lim
    return out


def log_omega_tokens(g):
    """ln omega per input token j = h'*nlon_in + w'."""
    _, w = colat_weights(g["grid_type"], g["nlat_in"])
    with np.errstate(divide="ignore"):      # the trapezoid grid has a zero-weight pole row: ln 0 = -inf
        return np.repeat(np.log(w * 2.0 * np.pi / g["nlon_in"]), g["nlon_in"])


def dense_attention(g, q, k, v, scale, dout=None, mask=None):
    """Dense masked softmax in torch float64 on channels-first tensors.
    Returns out, lse (and dq, dk, dv from autograd if dout is given)."""
    nbh, d = q.shape[:2]
    e = v.shape[1]
    qt = torch.tensor(np.asarray(q, np.float64).reshape(nbh, d, -1).transpose(0, 2, 1).copy(), requires_grad=True)
    kt = torch.tensor(np.asarray(k, np.float64).reshape(nbh, d, -1).transpose(0, 2, 1).copy(), requires_grad=True)
    vt = torch.tensor(np.asarray(v, np.float64).reshape(nbh, e, -1).transpose(0, 2, 1).copy(), requires_grad=True)
    bias = torch.tensor(log_omega_tokens(g))[None, None, :]
    if mask is None:
        mask = dense_mask(g)
    neg = torch.where(torch.tensor(mask), 0.0, -np.inf).to(torch.float64)[None]
    logits = qt @ kt.transpose(1, 2) * scale + bias + neg
    lse = torch.logsumexp(logits, dim=-1)
    out = torch.softmax(logits, dim=-1) @ vt
    so = q.shape[2:]
    res = [out.detach().numpy().transpose(0, 2, 1).reshape((nbh, e) + so), lse.detach().numpy().reshape((nbh,) + so)]
    if dout is not None:
        gt = torch.tensor(np.asarray(dout, np.float64).reshape(nbh, e, -1).transpose(0, 2, 1).copy())
        (out * gt).sum().backward()
        res += [qt.grad.numpy().transpose(0, 2, 1).reshape(q.shape),
                kt.grad.numpy().transpose(0, 2, 1).reshape(k.shape),
                vt.grad.numpy().transpose(0, 2, 1).reshape(v.shape)]
    return res


def dense_cond(g, q, k, v, dout, scale, mask=None):
    """Rounding sensitivities of out, lse, dq, dk, dv (sums of the absolute values of the elementary products, each
    weighted by the number of perturbed factors it carries), evaluated with dense matrices in numpy float64:
    a = |scale| |q|.|k|, c_lse = 1 + sum p a, w = 1 + a + c_lse, c_out = sum p w |v|,
    t = |dout.v - D| w + |dout|.|v| + |dout|.c_out, c_dq = |scale| (p t) |k|, c_dk = |scale| (p t)^T |q|,
    c_dv = (p w)^T |dout|."""
    nbh, d = q.shape[:2]
    e = v.shape[1]
    tok = lambda x, c: np.asarray(x, np.float64).reshape(nbh, c, -1).transpose(0, 2, 1)
    Q, K, V, G = tok(q, d), tok(k, d), tok(v, e), tok(dout, e)
    if mask is None:
        mask = dense_mask(g)
    bias = log_omega_tokens(g)[None, None, :]
    with np.errstate(invalid="ignore"):
        S = np.where(mask[None], Q @ K.transpose(0, 2, 1) * scale + bias, -np.inf)
    m = S.max(-1, keepdims=True)
    P = np.exp(S - m)
    P /= P.sum(-1, keepdims=True)
    A = abs(scale) * (np.abs(Q) @ np.abs(K).transpose(0, 2, 1))
    A = np.where(P > 0, A, 0.0)
    c_lse = 1.0 + (P * A).sum(-1)
    W = 1.0 + A + c_lse[..., None]
    c_out = (P * W) @ np.abs(V)
    out = P @ V
    D = (G * out).sum(-1)
    Dabs = (np.abs(G) * c_out).sum(-1)
    T = np.abs(G @ V.transpose(0, 2, 1) - D[..., None]) * W + np.abs(G) @ np.abs(V).transpose(0, 2, 1) + Dabs[..., None]
    PT = P * T
    c_dq = abs(scale) * (PT @ np.abs(K))
    c_dk = abs(scale) * (PT.transpose(0, 2, 1) @ np.abs(Q))
    c_dv = (P * W).transpose(0, 2, 1) @ np.abs(G)
    so, si = q.shape[2:], k.shape[2:]
    back = lambda x, c, s: x.transpose(0, 2, 1).reshape((nbh, c) + tuple(s))
    return back(c_out, e, so), c_lse.reshape((nbh,) + tuple(so)), back(c_dq, d, so), back(c_dk, d, si), back(c_dv, e, si)
