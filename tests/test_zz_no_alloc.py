"""s2_nattn_bwd_static (backward on the library's static device scratch, for callers that cannot allocate) against
s2_nattn_bwd with a caller workspace: same kernels, so the gradients must agree bit for bit (which is inside the
float32 parity bound |x - ref| <= 1e-6 + 1e-5 |ref| that s2_nattn_bwd is held to against the oracle).  Two calls in a
row, the second on a smaller problem, so stale contents of the shared array would show."""
import math

import numpy as np
import pytest
import torch

import paper_2505_11157_amd as S
from paper_2505_11157_amd.workloads import grid_dict, make_inputs

pytestmark = pytest.mark.gpu

BIG = dict(kind="nattn", grid_type=0, nlat_in=65, nlon_in=256, nlat_out=65, nlon_out=256, theta=2 * math.pi / 64,
           batch=2, heads=3, d=32, dtype="f32")          # matrix-core, streaming kernels; 99 840 points of scratch
SMALL = dict(kind="nattn", grid_type=1, nlat_in=16, nlon_in=36, nlat_out=8, nlon_out=12, theta=0.5,
             batch=1, heads=3, d=3, dtype="f32")         # shape-agnostic kernels; 288 points


def _both(c, seed):
    c, arrs = make_inputs(c, seed=seed)
    gd = grid_dict(c)
    g = S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])
    B, H, d = c["batch"], c["heads"], c["d"]
    scale = 1 / math.sqrt(d)
    dev = torch.device("cuda:0")
    q, k, v, dout = (torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).contiguous() for a in arrs)
    out, lse = S.s2_nattn_fwd(g, q, k, v, scale)
    ref = S.s2_nattn_bwd(g, q, k, v, out, lse, dout, scale)
    got = [torch.full_like(t, float("nan")) for t in (q, k, v)]
    S.s2_nattn_bwd_static(g, q, k, v, out, lse, dout, scale, *got)
    torch.cuda.synchronize()
    assert S.s2_grid_device_flags(g) == 0
    for name, a, b in zip(("dq", "dk", "dv"), ref, got):
        a, b = a.cpu().numpy().astype(np.float64), b.cpu().numpy().astype(np.float64)
        assert np.isfinite(b).all(), name
        assert (np.abs(b - a) <= 1e-6 + 1e-5 * np.abs(a)).all(), name
        assert np.array_equal(a, b), name + ": not bit-identical"


def test_static_scratch_backward_matches_workspace_backward():
    print("no-alloc: large problem", flush=True)
    _both(BIG, 31)
    print("no-alloc: smaller problem right after", flush=True)
    _both(SMALL, 32)


def test_static_scratch_rejects_oversize():
    # one point more than the array holds: a clear error, nothing launched
    limit = S.s2_nattn_bwd_static_max_points()
    assert limit == 2 * 1024 * 1024
    nlat, nlon = 129, 256
    g = S.s2_grid_init(0, nlat, nlon, nlat, nlon, 4 * math.pi / 128)
    nbh = limit // (nlat * nlon) + 1
    L = S.lib()
    dev = torch.device("cuda:0")
    x = torch.zeros(64, device=dev)
    p = x.data_ptr()
    rc = L.s2_nattn_bwd_static(g.handle, nbh, 1, 32, 32, S.S2_F32, 0.2, p, p, p, p, p, p, p, p, p, None)
    assert rc == S.S2_ERR_WORKSPACE and "exceeds the static scratch" in S.s2_last_error()
    torch.cuda.synchronize()
