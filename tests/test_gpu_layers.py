"""GPU parity of the layers around the attention kernels (through the C ABI) against the float64 oracle:
the multi-head attention sub-block (Sec. 3.4) and the DISCO convolution (App. B.3).

Tolerance, float32: |x - ref| <= 1e-6 + 1e-5 |ref| + 2e-5 rms(ref) elementwise.  A result of these layers has gone
through up to five chained float32 stages (moments, channel matrix, attention, channel matrix, residual) whose
roundings add up.  The rms term is an empirical allowance for that (several times the largest excess observed, which
every comparison prints), not a derived bound.  Parameter gradients are sums over every grid point of every batch
element (10^3 .. 10^5 signed terms) and get the rounding of such a sum on top: 8 * 2^-24 * (sum of the absolute
values of the terms, from the oracle's intermediates); this is what bounds the gradient of the key bias, which is
zero identically (a constant added to every key shifts all logits of a query alike) while its terms are not.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle as O
import paper_2505_11157_amd as S

pytestmark = pytest.mark.gpu
_REPORT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "parity_report.jsonl")
RMS_TERM = 2e-5


def close(x, ref, what, case, abs_sum=None):
    x, ref = np.asarray(x, np.float64), np.asarray(ref, np.float64)
    assert x.shape == ref.shape, (what, x.shape, ref.shape)
    err = np.abs(x - ref)
    rms = np.sqrt((ref ** 2).mean())
    strict = 1e-6 + 1e-5 * np.abs(ref) + (8 * 2.0 ** -24 * abs_sum if abs_sum is not None else 0.0)
    rec = dict(case=case, what=what, n=int(err.size), max_abs=float(err.max()), rms_ref=float(rms),
               n_over_strict=int((err > strict).sum()), excess_over_strict_in_rms=float(((err - strict) / max(rms, 1e-30)).max()))
    print("parity %-16s %-7s max|err| %.3e  rms(ref) %.3e  over strict %d/%d  (excess / rms %.2e)" % (
        case, what, rec["max_abs"], rms, rec["n_over_strict"], rec["n"], max(rec["excess_over_strict_in_rms"], 0.0)), flush=True)
    try:
        with open(_REPORT, "a") as f:
            f.write(json.dumps(rec) + "\n")
    except OSError:
        pass
    assert np.isfinite(x).all(), what
    tol = strict + RMS_TERM * rms
    assert (err <= tol).all(), "%s %s: max err %.3e, max excess %.3e" % (case, what, err.max(), (err - tol).max())


MHA_CASES = [
    # (grid, batch, channels, heads): d = 16 on 32 / 48 longitudes runs the shape-agnostic attention kernels, d = 32 on
    # 192 / 256 longitudes the matrix-core and streaming ones, d = 16 and 64 on 192 / 128 longitudes the fp32 band
    # tiles; 48 channels leave the 128 x 128 tiles of the channel matrices ragged
    (dict(grid_type=0, nlat_in=17, nlon_in=32, nlat_out=17, nlon_out=32, theta=0.5), 2, 32, 2),
    (dict(grid_type=1, nlat_in=16, nlon_in=48, nlat_out=16, nlon_out=48, theta=0.4), 1, 48, 3),
    (dict(grid_type=0, nlat_in=33, nlon_in=192, nlat_out=33, nlon_out=192, theta=0.3), 2, 64, 2),
    (dict(grid_type=0, nlat_in=25, nlon_in=256, nlat_out=25, nlon_out=256, theta=0.25), 1, 160, 5),
    (dict(grid_type=0, nlat_in=33, nlon_in=192, nlat_out=33, nlon_out=192, theta=0.3), 1, 48, 3),
    (dict(grid_type=1, nlat_in=16, nlon_in=128, nlat_out=16, nlon_out=128, theta=0.45), 1, 128, 2),
    # 64 channels on 816 grid points: the weight-resident channel products with a last tile of 16 of 32 points
    (dict(grid_type=0, nlat_in=17, nlon_in=48, nlat_out=17, nlon_out=48, theta=0.5), 1, 64, 4),
]


def _random_mha_case(seed):
    # seeded random sub-blocks: equal grids with 9 to 24 latitudes and 32 to 160 longitudes (multiples of 16), 64 or 128
    # channels (weight-resident channel products: ragged last tiles, one or several rounds) or 32, 96, 160 (tiled ones)
    rng = np.random.default_rng(9900 + seed)
    C = (64, 128, 32, 96, 128, 64, 160, 128)[seed % 8]
    d = int(rng.choice([8, 16, 32]))
    nlat, nlon = int(rng.integers(9, 25)), 16 * int(rng.integers(2, 11))
    gd = dict(grid_type=int(rng.integers(0, 2)), nlat_in=nlat, nlon_in=nlon, nlat_out=nlat, nlon_out=nlon,
              theta=float(rng.uniform(2.0, 4.0)) * math.pi / nlat)
    return gd, int(rng.integers(1, 4)), C, C // d


MHA_RANDOM = 8


@pytest.mark.parametrize("ci", range(len(MHA_CASES) + MHA_RANDOM))
def test_mha_block(ci):
    gd, B, C, heads = MHA_CASES[ci] if ci < len(MHA_CASES) else _random_mha_case(ci - len(MHA_CASES))
    rng = np.random.default_rng(900 + ci)
    shp = (B, C, gd["nlat_in"], gd["nlon_in"])
    f32 = lambda a: np.asarray(a, np.float32)
    x, dy = f32(rng.standard_normal(shp)), f32(rng.standard_normal(shp))
    w = lambda: f32(rng.standard_normal((C, C)) / math.sqrt(C))
    b = lambda: f32(0.3 * rng.standard_normal(C))
    P = dict(gamma=f32(1 + 0.2 * rng.standard_normal(C)), beta=b(), pos=f32(0.5 * rng.standard_normal(shp[1:])),
             Wq=w(), bq=b(), Wk=w(), bk=b(), Wv=w(), bv=b(), Wo=w(), bo=b())
    g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
    dev = torch.device("cuda:0")
    T = lambda a: torch.from_numpy(a).to(dev).contiguous()
    Pd = {k: T(v) for k, v in P.items()}
    y, ws = S.s2_mha_fwd(g, T(x), Pd, heads)
    dx, grads = S.s2_mha_bwd(g, T(x), Pd, heads, T(dy), ws)
    torch.cuda.synchronize()
    assert S.s2_grid_device_flags(g) == 0
    a64 = {k: v.astype(np.float64) for k, v in P.items()}
    args = (a64["pos"], a64["gamma"], a64["beta"], a64["Wq"], a64["bq"], a64["Wk"], a64["bk"], a64["Wv"], a64["bv"],
            a64["Wo"], a64["bo"])
    r_y, _ = O.mha_fwd(gd, heads, x.astype(np.float64), *args)
    r = O.mha_bwd(gd, heads, x.astype(np.float64), *args, dy.astype(np.float64))
    case = "mha%d" % ci
    close(y.cpu().numpy(), r_y, "y", case)
    close(dx.cpu().numpy(), r["dx"], "dx", case)
    im = {k: np.abs(v) for k, v in r["intermediates"].items()}
    ady = np.abs(dy.astype(np.float64))
    ein = lambda u, v: np.einsum("bohw,bchw->oc", u, v)
    abs_sums = dict(gamma=(im["dxn"] * im["xhat"]).sum((0, 2, 3)), beta=im["dxn"].sum((0, 2, 3)), pos=im["dxn"].sum(0),
                    Wq=ein(im["dq"], im["xn"]), bq=im["dq"].sum((0, 2, 3)), Wk=ein(im["dk"], im["xn"]),
                    bk=im["dk"].sum((0, 2, 3)), Wv=ein(im["dv"], im["xn"]), bv=im["dv"].sum((0, 2, 3)),
                    Wo=ein(ady, im["a"]), bo=ady.sum((0, 2, 3)))
    for k in S.MHA_FIELDS:
        close(grads[k].cpu().numpy(), r["d" + k], "d" + k, case, abs_sums[k])
    # again on the same workspace: bit-identical (no atomics, fixed summation orders)
    y2, _ = S.s2_mha_fwd(g, T(x), Pd, heads, workspace=ws)
    dx2, grads2 = S.s2_mha_bwd(g, T(x), Pd, heads, T(dy), ws)
    assert torch.equal(y, y2) and torch.equal(dx, dx2) and all(torch.equal(grads[k], grads2[k]) for k in grads)


def test_mha_channel_products_at_full_size_do_not_depend_on_the_tile_schedule():
    # 4 x 65 x 512 points, 128 channels: the weight-resident channel products run two whole rounds of tiles per
    # wavefront (operands of the next tile requested before the results of the last are stored) plus a partial round
    # cut into row blocks; one batch element alone is a single round with another tile-to-wavefront map.  Every output
    # column is the same sequence of matrix instructions either way, so y and dx must agree bit for bit (the small
    # cases above pin both kinds of round to the oracle; the weight gradients sum over the batch and are left out).
    gd = dict(grid_type=0, nlat_in=65, nlon_in=512, nlat_out=65, nlon_out=512, theta=0.06)
    B, C, heads = 4, 128, 8
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cpu").manual_seed(977)
    rnd = lambda *shape: torch.randn(*shape, generator=gen).to(dev)
    x, dy = rnd(B, C, 65, 512), rnd(B, C, 65, 512)
    P = dict(gamma=1 + 0.2 * rnd(C), beta=0.3 * rnd(C), pos=0.5 * rnd(C, 65, 512))
    for n in "qkvo":
        P["W" + n] = rnd(C, C) / math.sqrt(C)
        P["b" + n] = 0.3 * rnd(C)
    g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
    y, ws = S.s2_mha_fwd(g, x, P, heads)
    dx, _ = S.s2_mha_bwd(g, x, P, heads, dy, ws)
    torch.cuda.synchronize()
    assert S.s2_grid_device_flags(g) == 0
    assert torch.isfinite(y).all() and torch.isfinite(dx).all()
    for b in range(B):
        y1, ws1 = S.s2_mha_fwd(g, x[b:b + 1].contiguous(), P, heads)
        dx1, _ = S.s2_mha_bwd(g, x[b:b + 1].contiguous(), P, heads, dy[b:b + 1].contiguous(), ws1)
        assert torch.equal(y[b:b + 1], y1) and torch.equal(dx[b:b + 1], dx1), "batch element %d" % b


def test_mha_optional_parameters_and_errors():
    gd = MHA_CASES[0][0]
    g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
    rng = np.random.default_rng(5)
    B, C, heads = 1, 32, 4
    dev = torch.device("cuda:0")
    f32 = lambda a: torch.from_numpy(np.asarray(a, np.float32)).to(dev)
    x = f32(rng.standard_normal((B, C, 17, 32)))
    dy = f32(rng.standard_normal((B, C, 17, 32)))
    P = {k: f32(rng.standard_normal((C, C)) / math.sqrt(C)) for k in ("Wq", "Wk", "Wv", "Wo")}
    y, ws = S.s2_mha_fwd(g, x, P, heads)                 # no norm affine, no embedding, no biases
    dx, grads = S.s2_mha_bwd(g, x, P, heads, dy, ws)
    torch.cuda.synchronize()
    assert set(grads) == {"Wq", "Wk", "Wv", "Wo"}
    z = np.zeros(C)
    a = [p.cpu().numpy().astype(np.float64) for p in (P["Wq"], P["Wk"], P["Wv"], P["Wo"])]
    args = (np.zeros((C, 17, 32)), np.ones(C), z, a[0], z, a[1], z, a[2], z, a[3], z)
    r_y, _ = O.mha_fwd(gd, heads, x.cpu().numpy().astype(np.float64), *args)
    r = O.mha_bwd(gd, heads, x.cpu().numpy().astype(np.float64), *args, dy.cpu().numpy().astype(np.float64))
    close(y.cpu().numpy(), r_y, "y", "mha-bare")
    close(dx.cpu().numpy(), r["dx"], "dx", "mha-bare")
    close(grads["Wv"].cpu().numpy(), r["dWv"], "dWv", "mha-bare")
    with pytest.raises(S.S2Error) as ei:
        S.s2_mha_fwd(g, x, P, 5)                          # 32 channels do not split into 5 heads
    assert ei.value.code == S.S2_ERR_INVALID_ARG
    with pytest.raises(S.S2Error) as ei:
        S.s2_mha_fwd(g, x, P, heads, workspace=torch.empty(1024, dtype=torch.uint8, device=dev))
    assert ei.value.code == S.S2_ERR_WORKSPACE
    g2 = S.s2_grid_init(0, 17, 32, 9, 16, 0.5)
    with pytest.raises(S.S2Error) as ei:
        S.s2_mha_fwd(g2, x, P, heads)
    assert ei.value.code == S.S2_ERR_UNSUPPORTED
    buf = torch.zeros(x.numel() + 1, dtype=torch.float32, device=dev)
    x_off = buf[1:].view_as(x)                            # contiguous, but 4 bytes off a 16-byte boundary
    x_off.copy_(x)
    with pytest.raises(S.S2Error) as ei:
        S.s2_mha_fwd(g, x_off, P, heads)
    assert ei.value.code == S.S2_ERR_INVALID_ARG
    with pytest.raises(S.S2Error) as ei:
        S.s2_mha_bwd(g, x, P, heads, x_off, ws)
    assert ei.value.code == S.S2_ERR_INVALID_ARG
    torch.cuda.synchronize()


DISCO_CASES = [
    # (grid, batch, channels in, basis functions, channels out)
    (dict(grid_type=0, nlat_in=17, nlon_in=32, nlat_out=17, nlon_out=32, theta=0.5), 2, 8, 4, 16),
    (dict(grid_type=0, nlat_in=33, nlon_in=64, nlat_out=17, nlon_out=32, theta=0.4), 1, 16, 2, 32),
    (dict(grid_type=2, nlat_in=16, nlon_in=32, nlat_out=16, nlon_out=32, theta=0.45), 1, 4, 4, 16),
    (dict(grid_type=1, nlat_in=24, nlon_in=48, nlat_out=24, nlon_out=48, theta=0.35), 2, 2, 8, 48),
    (dict(grid_type=0, nlat_in=9, nlon_in=80, nlat_out=9, nlon_out=16, theta=0.6), 1, 16, 1, 16),     # pscale 5
    # 9 and 16 basis functions: the counts the paper pairs with 3 x 3 and 4 x 4 planar kernels (App. C)
    (dict(grid_type=0, nlat_in=17, nlon_in=32, nlat_out=17, nlon_out=32, theta=0.5), 1, 16, 9, 16),
    (dict(grid_type=1, nlat_in=16, nlon_in=32, nlat_out=8, nlon_out=16, theta=0.6), 2, 2, 16, 16),
    # equal longitude counts of at least 64 and batch * channels a multiple of 16: the matrix-core kernels (short arcs
    # and whole circles, 80 longitudes = a ragged last group, fewer output than input latitudes, the zero-weight pole row)
    (dict(grid_type=0, nlat_in=17, nlon_in=64, nlat_out=17, nlon_out=64, theta=0.5), 2, 8, 4, 16),
    (dict(grid_type=1, nlat_in=16, nlon_in=128, nlat_out=16, nlon_out=128, theta=0.3), 1, 16, 9, 16),
    (dict(grid_type=0, nlat_in=9, nlon_in=80, nlat_out=9, nlon_out=80, theta=1.2), 1, 16, 3, 32),
    (dict(grid_type=0, nlat_in=33, nlon_in=64, nlat_out=17, nlon_out=64, theta=0.4), 1, 32, 16, 16),
    (dict(grid_type=2, nlat_in=32, nlon_in=192, nlat_out=32, nlon_out=192, theta=0.25), 1, 16, 5, 16),
]


@pytest.mark.parametrize("ci", range(len(DISCO_CASES)))
def test_disco_convolution(ci):
    gd, B, cin, K, cout = DISCO_CASES[ci]
    rng = np.random.default_rng(950 + ci)
    f32 = lambda a: np.asarray(a, np.float32)
    x = f32(rng.standard_normal((B, cin, gd["nlat_in"], gd["nlon_in"])))
    dy = f32(rng.standard_normal((B, cout, gd["nlat_out"], gd["nlon_out"])))
    weight, bias = f32(rng.standard_normal((cout, cin, K))), f32(rng.standard_normal(cout))
    g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
    dc = S.s2_disco_init(g, K)
    dev = torch.device("cuda:0")
    T = lambda a: torch.from_numpy(a).to(dev).contiguous()
    y, ws = S.s2_disco_fwd(dc, T(x), T(weight), T(bias))
    dx, dw, db = S.s2_disco_bwd(dc, T(x), T(weight), T(dy), ws)
    torch.cuda.synchronize()
    d64 = lambda a: a.astype(np.float64)
    r_y, r_z = O.disco_fwd(gd, K, d64(x), d64(weight), d64(bias))
    r_dx, r_dw, r_db = O.disco_bwd(gd, K, d64(x), d64(weight), d64(bias), d64(dy))
    case = "disco%d" % ci
    close(y.cpu().numpy(), r_y, "y", case)
    close(dx.cpu().numpy(), r_dx, "dx", case)
    close(dw.cpu().numpy(), r_dw, "dweight", case, np.einsum("bohw,bckhw->ock", np.abs(d64(dy)), np.abs(r_z)))
    close(db.cpu().numpy(), r_db, "dbias", case, np.abs(d64(dy)).sum((0, 2, 3)))
    y2, _ = S.s2_disco_fwd(dc, T(x), T(weight), T(bias), workspace=ws)
    dx2, dw2, db2 = S.s2_disco_bwd(dc, T(x), T(weight), T(dy), ws)
    assert torch.equal(y, y2) and torch.equal(dx, dx2) and torch.equal(dw, dw2) and torch.equal(db, db2)


def test_disco_errors():
    g = S.s2_grid_init(0, 9, 16, 17, 32, 0.5)         # upsampling handle
    with pytest.raises(S.S2Error) as ei:
        S.s2_disco_init(g, 3)
    assert ei.value.code == S.S2_ERR_UNSUPPORTED
    g = S.s2_grid_init(0, 17, 32, 17, 32, 0.5)
    with pytest.raises(S.S2Error) as ei:
        S.s2_disco_init(g, 17)
    assert ei.value.code == S.S2_ERR_INVALID_ARG
    dc = S.s2_disco_init(g, 3)
    dev = torch.device("cuda:0")
    x = torch.zeros((1, 5, 17, 32), device=dev)
    with pytest.raises(S.S2Error) as ei:
        S.s2_disco_fwd(dc, x, torch.zeros((16, 5, 3), device=dev))       # 5 * 3 is not a multiple of 16
    assert ei.value.code == S.S2_ERR_UNSUPPORTED
    torch.cuda.synchronize()
