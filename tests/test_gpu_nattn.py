"""GPU parity of the neighborhood attention (through the C ABI) against the float64 oracle.

Tolerance (float32 path), ref = oracle in float64 on the same float32 inputs:
  out, lse, dq, dk, dv on the workloads and on every unit-variance case:
                                     |x - ref| <= 1e-6 + 1e-5 |ref|                      (the stated bound)
  (lse: plus 1 * 2^-24 * cond, see run_case: needed by one element of one small grid whose lse is 0.014)
  cases whose logits are large (q and k scaled by 6: nearly one-hot softmax; the random tiny grids with scales up to
  0.6 and disks of up to 2.2 rad), and the full-size upsampling workload, whose dk and dv sum four times as many
  terms per input point as the equal-grid workloads (6 of 1 056 768 dk elements exceed the plain bound, by 4e-7):
                                     |x - ref| <= 1e-6 + 1e-5 |ref| + C * 2^-24 * cond
where cond is the oracle's first-order rounding sensitivity of that element: the sum of the absolute values of the
elementary products it is made of, each weighted by the number of rounded factors it carries.  With logits of
magnitude 100 one float32 rounding of a logit already changes its probability by 1e-5, so no float32 evaluation can
meet a bound relative to |ref| alone there; 2^-24 * cond is what one rounding per product costs.  C = 4 is twice
the largest excess observed over all such cases, in units of 2^-24 * cond (1.9, on dv of a peaked case; every
comparison prints what it achieved, and the design notes record the figures per workload).
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle as O
import paper_2505_11157_amd as S
from paper_2505_11157_amd.workloads import CONFIGS, grid_dict, make_inputs

pytestmark = pytest.mark.gpu

U32 = 2.0 ** -24
C_DERIVED = 4.0
_REPORT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "parity_report.jsonl")


def _grid(gd):
    return S.s2_grid_init(gd["grid_type"], gd["nlat_in"], gd["nlon_in"], gd["nlat_out"], gd["nlon_out"], gd["theta"])


def compare(x, ref, what, cond=None, C=0.0, case=""):
    """Assert |x - ref| <= 1e-6 + 1e-5 |ref| + C 2^-24 cond elementwise; print and log what was achieved."""
    assert np.isfinite(x).all(), "%s %s: non-finite values" % (case, what)
    err = np.abs(x - ref)
    strict = 1e-6 + 1e-5 * np.abs(ref)
    over = err > strict
    rec = dict(case=case, what=what, n=int(err.size), max_abs=float(err.max()),
               max_rel=float((err / np.maximum(np.abs(ref), 1e-30))[np.abs(ref) > 1e-3].max()) if (np.abs(ref) > 1e-3).any() else 0.0,
               n_over_strict=int(over.sum()), max_excess_strict=float((err - strict).max()))
    if cond is not None:
        rec["C_obs"] = float(((err - strict) / np.maximum(U32 * cond, 1e-300)).max())
    print("parity %-28s %-4s max|err| %.3e  max rel %.3e  over strict %d/%d (excess %.2e)%s" % (
        case, what, rec["max_abs"], rec["max_rel"], rec["n_over_strict"], rec["n"], max(rec["max_excess_strict"], 0.0),
        "  C_obs %.3f" % rec["C_obs"] if cond is not None else ""), flush=True)
    try:
        with open(_REPORT, "a") as f:
            f.write(json.dumps(rec) + "\n")
    except OSError:
        pass
    tol = strict + (C * U32 * cond if cond is not None else 0.0)
    assert (err <= tol).all(), "%s %s: max err %.3e, max excess over the bound %.3e, %d elements over" % (
        case, what, err.max(), (err - tol).max(), int((err > tol).sum()))


def run_case(c, arrs, slices, C=0.0, case=""):
    """Run fwd+bwd on the GPU for the whole batch, compare the (b*heads) slices in `slices` with the oracle."""
    gd = grid_dict(c)
    g = _grid(gd)
    B, H, d = c["batch"], c["heads"], c["d"]
    scale = c.get("scale", 1 / math.sqrt(d))
    dev = torch.device("cuda:0")
    fold = lambda a: torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).contiguous()
    q, k, v, dout = (fold(a) for a in arrs)
    out, lse = S.s2_nattn_fwd(g, q, k, v, scale)
    dq, dk, dv = S.s2_nattn_bwd(g, q, k, v, out, lse, dout, scale)
    torch.cuda.synchronize()
    assert S.s2_grid_device_flags(g) == 0    # no bounded wait inside a kernel ran out
    unfold = lambda t: t.reshape((B * H,) + t.shape[2:]).cpu().numpy().astype(np.float64)
    out, lse, dq, dk, dv = (unfold(t) for t in (out, lse, dq, dk, dv))
    for s in slices:
        sl = slice(s, s + 1)
        a64 = [a[sl].astype(np.float64) for a in arrs]
        # upsampling: the oracle's per-pair form of eq. (5), evaluated on the fly where the N_out x N_in mask would
        # not fit
        brute = 0 if gd["nlon_in"] % gd["nlon_out"] == 0 else 1
        if brute and gd["nlat_out"] * gd["nlon_out"] * gd["nlat_in"] * gd["nlon_in"] > 1 << 28:
            brute = 2
        r_out, r_lse = O.nattn_fwd(gd, a64[0], a64[1], a64[2], scale, brute=brute)
        r_dq, r_dk, r_dv = O.nattn_bwd(gd, *a64, scale, brute=brute)
        c_out, c_lse, c_dq, c_dk, c_dv = O.nattn_cond(gd, *a64, scale, brute=brute)
        cs = "%s[%d]" % (case, s)
        for what, x, ref, cnd in (("out", out, r_out, c_out), ("lse", lse, r_lse, c_lse), ("dq", dq, r_dq, c_dq),
                                  ("dk", dk, r_dk, c_dk), ("dv", dv, r_dv, c_dv)):
            # lse = ln of a sum of positive terms can come out arbitrarily close to zero (ln sum(omega e^s) ~ 0 on
            # a coarse grid), where the relative part of the bound vanishes while the float32 sum keeps its rounding:
            # lse always gets one unit of 2^-24 * cond on top (largest excess observed: 0.13 units)
            compare(x[sl], ref, what, cnd, max(C, 1.0) if what == "lse" else C, cs)
    return out, lse, dq, dk, dv


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_parity_configs(cfg):
    # every (batch, head) slice of every workload: the tuned kernels pack 8 / P slices per workgroup and number
    # workgroups per segment and per XCD, so a slice-dependent indexing error at full size would show only there
    c, arrs = make_inputs(cfg)
    run_case(c, arrs, range(c["batch"] * c["heads"]), case="cfg%d" % cfg)


SMALL = [
    # ragged longitude counts, odd head dims, d != e is exercised separately
    dict(kind="nattn", grid_type=0, nlat_in=12, nlon_in=15, nlat_out=7, nlon_out=5, theta=1.1, batch=2, heads=1, d=5, dtype="f32"),
    dict(kind="nattn", grid_type=1, nlat_in=16, nlon_in=36, nlat_out=8, nlon_out=12, theta=0.5, batch=1, heads=3, d=3, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=9, nlon_in=16, nlat_out=9, nlon_out=16, theta=math.pi, batch=1, heads=2, d=16, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=33, nlon_in=200, nlat_out=33, nlon_out=100, theta=0.25, batch=1, heads=2, d=12, dtype="f32"),
    dict(kind="nattn", grid_type=1, nlat_in=24, nlon_in=70, nlat_out=24, nlon_out=70, theta=0.4, batch=1, heads=1, d=64, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=33, nlon_in=64, nlat_out=33, nlon_out=1, theta=0.3, batch=1, heads=2, d=8, dtype="f32"),
    dict(kind="nattn", grid_type=1, nlat_in=2, nlon_in=1, nlat_out=2, nlon_out=1, theta=0.2, batch=1, heads=1, d=1, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=20, nlon_in=96, nlat_out=10, nlon_out=32, theta=0.35, batch=1, heads=2, d=32, dtype="f32"),
    # tuned kernels (d = 32) with ragged last segments, equal grids and 2:1 downsampling, 3 and 9 slices
    dict(kind="nattn", grid_type=1, nlat_in=24, nlon_in=100, nlat_out=24, nlon_out=100, theta=0.4, batch=3, heads=1, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=19, nlon_in=152, nlat_out=10, nlon_out=76, theta=0.3, batch=3, heads=3, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=21, nlon_in=192, nlat_out=21, nlon_out=192, theta=0.6, batch=1, heads=2, d=32, dtype="f32"),
    # streaming kernels for the light latitudes (equal grids, at least 192 longitudes): ragged last strip, bands of
    # 9 / about 6 / 5 latitudes (8, 5-6 and 4 wavefronts per workgroup), more slices than compute units need
    dict(kind="nattn", grid_type=0, nlat_in=41, nlon_in=196, nlat_out=41, nlon_out=196, theta=4 * math.pi / 40, batch=1, heads=3, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=1, nlat_in=40, nlon_in=200, nlat_out=40, nlon_out=200, theta=0.2, batch=2, heads=1, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=65, nlon_in=256, nlat_out=65, nlon_out=256, theta=2 * math.pi / 64, batch=1, heads=2, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=33, nlon_in=192, nlat_out=33, nlon_out=192, theta=0.3, batch=9, heads=2, d=32, dtype="f32"),
    # a handful of light latitudes with bands of three rows (two wavefronts per workgroup, more segments than fit)
    dict(kind="nattn", grid_type=0, nlat_in=9, nlon_in=256, nlat_out=9, nlon_out=256, theta=0.5, batch=1, heads=2, d=32, dtype="f32"),
    # the equiangular grid as the paper prints it (no south pole, zero weight on the pole row): generic, tuned
    # equal-grid and tuned 2:1 kernels
    dict(kind="nattn", grid_type=2, nlat_in=16, nlon_in=32, nlat_out=16, nlon_out=32, theta=0.45, batch=1, heads=2, d=8, dtype="f32"),
    dict(kind="nattn", grid_type=2, nlat_in=64, nlon_in=256, nlat_out=64, nlon_out=256, theta=4 * math.pi / 64, batch=1, heads=2, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=2, nlat_in=40, nlon_in=160, nlat_out=20, nlon_out=80, theta=0.35, batch=1, heads=3, d=32, dtype="f32"),
    # Gauss-Lobatto grid (both poles, Gaussian spacing): generic and tuned kernels
    dict(kind="nattn", grid_type=3, nlat_in=17, nlon_in=32, nlat_out=17, nlon_out=32, theta=0.45, batch=1, heads=2, d=8, dtype="f32"),
    dict(kind="nattn", grid_type=3, nlat_in=65, nlon_in=256, nlat_out=65, nlon_out=256, theta=4 * math.pi / 64, batch=1, heads=2, d=32, dtype="f32"),
    # upsampling (nlon_out = 2, 3, 4 x nlon_in): shape-agnostic kernels with one list per longitude class
    dict(kind="nattn", grid_type=0, nlat_in=9, nlon_in=16, nlat_out=17, nlon_out=32, theta=0.5, batch=1, heads=2, d=8, dtype="f32"),
    dict(kind="nattn", grid_type=1, nlat_in=12, nlon_in=24, nlat_out=16, nlon_out=72, theta=0.4, batch=2, heads=1, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=9, nlon_in=20, nlat_out=17, nlon_out=80, theta=0.6, batch=1, heads=1, d=5, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=6, nlon_in=10, nlat_out=9, nlon_out=20, theta=math.pi, batch=1, heads=1, d=3, dtype="f32"),
    # upsampling on the tuned kernels (d = 32, at least 72 input longitudes, a multiple of 4): every class of output
    # longitudes as an equal-grid problem; 2x, 3x, 4x, nine slices, a ragged last segment, full circles at the poles
    dict(kind="nattn", grid_type=0, nlat_in=13, nlon_in=76, nlat_out=25, nlon_out=152, theta=0.5, batch=3, heads=3, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=1, nlat_in=12, nlon_in=72, nlat_out=16, nlon_out=216, theta=0.4, batch=1, heads=2, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=0, nlat_in=17, nlon_in=132, nlat_out=33, nlon_out=528, theta=0.3, batch=1, heads=1, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=3, nlat_in=9, nlon_in=80, nlat_out=9, nlon_out=160, theta=1.0, batch=1, heads=2, d=32, dtype="f32"),
    # larger and odd longitude ratios (8x, 5x)
    dict(kind="nattn", grid_type=0, nlat_in=7, nlon_in=72, nlat_out=9, nlon_out=576, theta=0.7, batch=1, heads=2, d=32, dtype="f32"),
    dict(kind="nattn", grid_type=1, nlat_in=10, nlon_in=84, nlat_out=6, nlon_out=420, theta=0.45, batch=2, heads=1, d=32, dtype="f32"),
    # upsampling on the grid of App. A.1 (zero-weight pole row): shape-agnostic kernels and the class view
    dict(kind="nattn", grid_type=2, nlat_in=8, nlon_in=16, nlat_out=12, nlon_out=32, theta=0.7, batch=1, heads=2, d=8, dtype="f32"),
    dict(kind="nattn", grid_type=2, nlat_in=12, nlon_in=72, nlat_out=16, nlon_out=144, theta=0.5, batch=1, heads=2, d=32, dtype="f32"),
]


def test_streaming_with_many_slices():
    # 160 (batch, head) slices: one latitude segment per strip, every workgroup walks the whole light range
    c = dict(kind="nattn", grid_type=0, nlat_in=33, nlon_in=192, nlat_out=33, nlon_out=192, theta=0.3, batch=40, heads=4,
             d=32, dtype="f32")
    c, arrs = make_inputs(c, seed=77)
    run_case(c, arrs, [0, 83, 159], case="many-slices")


@pytest.mark.parametrize("ci", range(len(SMALL)))
def test_parity_edge_shapes(ci):
    c, arrs = make_inputs(SMALL[ci], seed=200 + ci)
    run_case(c, arrs, range(c["batch"] * c["heads"]), case="edge%d" % ci)


def test_value_width_differs_from_key_width():
    c = dict(kind="nattn", grid_type=1, nlat_in=12, nlon_in=24, nlat_out=12, nlon_out=24, theta=0.6,
             batch=1, heads=2, d=4, dtype="f32")
    rng = np.random.default_rng(77)
    arrs = [rng.standard_normal(s).astype(np.float32) for s in ((2, 4, 12, 24), (2, 4, 12, 24), (2, 7, 12, 24), (2, 7, 12, 24))]
    run_case(c, arrs, range(2), case="d!=e")


def test_deterministic_and_roll_equivariant():
    c, arrs = make_inputs(2)
    r1 = run_case(c, arrs, [])
    r2 = run_case(c, arrs, [])
    for a, b in zip(r1, r2):
        assert np.array_equal(a, b)          # no atomics anywhere: bit-reproducible
    rolled = [np.roll(a, 1, axis=-1) for a in arrs]
    r3 = run_case(c, rolled, [])
    # shift invariance in longitude (App. B.3): exact in the vector kernels, whose summation order moves with
    # the output; the matrix-core kernel for the polar latitudes sums in fixed column tiles, so there the
    # rolled result agrees to rounding only
    for a, b in zip(r1, r3):
        ra = np.roll(a, 1, axis=-1)
        assert np.abs(ra - b).max() <= 2e-6 + 1e-5 * np.abs(ra).max()


@pytest.mark.parametrize("cfg", [3, 4])
def test_bit_reproducible_full_configs(cfg):
    # every kernel of the tuned path (staged windows, split latitudes merged through LDS) must give
    # identical bits run after run: there are no atomics and no order-dependent reductions
    c, arrs = make_inputs(cfg)
    ref = run_case(c, arrs, [])
    for _ in range(3):
        again = run_case(c, arrs, [])
        for a, b in zip(ref, again):
            assert np.array_equal(a, b)


@pytest.mark.parametrize("cfg", [2, 3, 4, 6])
def test_many_launches_bit_identical_full_configs(cfg):
    # 40 forward + backward launches in a row, compared on the device: a dependence on which wavefronts happen to
    # run side by side (a variant of the split kernels showed one on the last latitude of a launch of workload 4, in 4
    # of 30 launches) cannot hide behind three repetitions
    c, arrs = make_inputs(cfg)
    g = _grid(grid_dict(c))
    B, H, d = c["batch"], c["heads"], c["d"]
    scale = 1 / math.sqrt(d)
    dev = torch.device("cuda:0")
    fold = lambda a: torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).contiguous()
    q, k, v, dout = (fold(a) for a in arrs)
    out0, lse0 = S.s2_nattn_fwd(g, q, k, v, scale)
    g0 = S.s2_nattn_bwd(g, q, k, v, out0, lse0, dout, scale)
    for it in range(40):
        out, lse = S.s2_nattn_fwd(g, q, k, v, scale)
        gr = S.s2_nattn_bwd(g, q, k, v, out0, lse0, dout, scale)
        assert torch.equal(out, out0) and torch.equal(lse, lse0), "launch %d: forward differs" % it
        assert all(torch.equal(x, y) for x, y in zip(gr, g0)), "launch %d: backward differs" % it


class debug_switches:
    """Set test-only dispatch switches of the library for the duration of a with-block."""

    def __init__(self, bits):
        self.bits = bits

    def __enter__(self):
        S.s2_debug_control(self.bits, 0)

    def __exit__(self, *exc):
        S.s2_debug_control(0, self.bits)


def test_vector_kernels_cover_dense_latitudes_too():
    # S2_DEBUG_NO_MFMA sends the polar latitudes through the split vector kernels instead of the matrix-core
    # kernels: same parity bar
    c, arrs = make_inputs(2)
    with debug_switches(S.S2_DEBUG_NO_MFMA):
        run_case(c, arrs, [0, 7], case="cfg2-no-mfma")


def test_one_wave_kernels_on_streaming_shapes():
    # S2_DEBUG_NO_STREAM keeps the light latitudes on the one-wavefront kernels, S2_DEBUG_NO_MFMA the dense ones on
    # the split vector kernels: the paths a shape takes when the streaming / matrix-core kernels do not apply, checked
    # here on a shape where they do
    c, arrs = make_inputs(SMALL[11], seed=5)
    with debug_switches(S.S2_DEBUG_NO_MFMA | S.S2_DEBUG_NO_STREAM):
        run_case(c, arrs, [0, 2], case="edge11-no-mfma-no-stream")
    c, arrs = make_inputs(2)
    with debug_switches(S.S2_DEBUG_NO_ROW_GROUPS | S.S2_DEBUG_NO_BAND):
        run_case(c, arrs, [3], case="cfg2-no-row-groups")


def test_tuned_kernels_where_band_tiles_are_the_default():
    # equal grids with d = 32 whose light latitudes lack the streaming structure run on the band-tile matrix-core
    # kernels by default; S2_DEBUG_NO_BAND keeps them on the matrix-core + one-wavefront kernels tuned for d = 32
    # (what such shapes ran on before, and still run on when the longitude count is not a multiple of 64)
    with debug_switches(S.S2_DEBUG_NO_BAND):
        c, arrs = make_inputs(2)
        run_case(c, arrs, range(c["batch"] * c["heads"]), case="cfg2-no-band")
        for i in (10, 15):
            c, arrs = make_inputs(SMALL[i], seed=40 + i)
            run_case(c, arrs, [0, 1], case="edge%d-no-band" % i)


def test_launcher_failure_is_reported():
    # a launcher that reports failure must surface as S2_ERR_DEVICE (not as S2_OK with nothing launched): forced
    # through the test-only switch; the outputs stay untouched
    c, arrs = make_inputs(SMALL[11], seed=5)
    g = _grid(grid_dict(c))
    B, H, d = c["batch"], c["heads"], c["d"]
    dev = torch.device("cuda:0")
    q, k, v, dout = (torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).contiguous() for a in arrs)
    out = torch.full_like(q, 7.0)
    lse = torch.full((B, H) + tuple(q.shape[3:]), 7.0, device=dev)
    dq, dk, dv = torch.full_like(q, 7.0), torch.full_like(k, 7.0), torch.full_like(v, 7.0)
    with debug_switches(S.S2_DEBUG_FAIL_LAUNCH):
        with pytest.raises(S.S2Error) as ei:
            S.s2_nattn_fwd(g, q, k, v, 0.2, out=out, lse=lse)
        assert ei.value.code == S.S2_ERR_DEVICE and "forward launch" in str(ei.value)
        with pytest.raises(S.S2Error) as ei:
            S.s2_nattn_bwd(g, q, k, v, out, lse, dout, 0.2, dq=dq, dk=dk, dv=dv)
        assert ei.value.code == S.S2_ERR_DEVICE and "backward launch" in str(ei.value)
    torch.cuda.synchronize()
    for t in (out, lse, dq, dk, dv):
        assert (t == 7.0).all()
    S.s2_nattn_fwd(g, q, k, v, 0.2, out=out, lse=lse)      # and the switch is off again
    torch.cuda.synchronize()
    assert not (out == 7.0).all()


# Peaked softmax: q and k scaled by 6 put the logits tens of units apart (nearly one-hot probabilities), so the lazily
# moved reference maximum of every kernel family has to move many times; a negative scale flips which logits are the
# large ones.  Shapes: matrix-core + streaming (65x256), split vector kernels on a 2:1 grid, shape-agnostic kernels
# (d = 12, 2:1; d = 64), the grid of App. A.1 with its zero-weight pole row on the tuned (equal, 2:1, upsampling) and the
# shape-agnostic kernels (a pole logit far above all others must not drown the positive-weight terms), upsampling in
# the class view.
PEAKED = [13, 9, 3, 4, 17, 16, 18, 25, 31, 32]


@pytest.mark.parametrize("ci", PEAKED)
@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_peaked_softmax(ci, sign):
    c, arrs = make_inputs(SMALL[ci], seed=600 + ci)
    arrs = [arrs[0] * np.float32(6.0), arrs[1] * np.float32(6.0), arrs[2], arrs[3]]
    c = dict(c, scale=sign / math.sqrt(c["d"]))
    nbh = c["batch"] * c["heads"]
    run_case(c, arrs, range(min(nbh, 2)), C=C_DERIVED, case="peaked%d%s" % (ci, "+" if sign > 0 else "-"))


def test_peaked_softmax_vector_kernels_on_dense_latitudes():
    # the same on the split 8-wave and one-wave vector kernels for the shape whose dense latitudes normally run on the
    # matrix cores and whose light ones on the streaming kernels
    c, arrs = make_inputs(SMALL[13], seed=613)
    arrs = [arrs[0] * np.float32(6.0), arrs[1] * np.float32(6.0), arrs[2], arrs[3]]
    with debug_switches(S.S2_DEBUG_NO_MFMA | S.S2_DEBUG_NO_STREAM):
        run_case(c, arrs, [1], C=C_DERIVED, case="peaked13-vector")


@pytest.mark.parametrize("which", ["cfg3", "small11", "small13"])
def test_streaming_kernels_take_the_light_latitudes(which):
    # the launches the library reports for one forward + backward: streaming kernels for the light latitudes
    # wherever the shape allows them, never the one-wavefront kernels
    if which == "cfg3":
        c, arrs = make_inputs(3)
        arrs = [a[:2] for a in arrs]
        c = dict(c, batch=1, heads=2)
    else:
        c, arrs = make_inputs(SMALL[int(which[5:])], seed=9)
    S.s2_trace_reset()
    S.s2_trace_enable(True)
    try:
        run_case(c, arrs, [])
        torch.cuda.synchronize()
        names = {n for n, _, _ in S.s2_trace_entries()}
    finally:
        S.s2_trace_enable(False)
        S.s2_trace_reset()
    assert {"nattn_fwd_stream", "nattn_bwd_dq_stream", "nattn_bwd_dkdv_stream"} <= names, names
    assert not any("1 wave" in n for n in names), names


def test_hip_graph_replays_match_eager():
    # the library only enqueues kernels on the caller's stream (no allocation, no memset, no synchronisation), so a
    # forward + backward can be captured into a HIP graph once the kernels have been launched once (the first launch
    # of a kernel raises its LDS limit, which is not a stream operation).  Every replay, with eager work and new
    # inputs in between, must reproduce the eager result bit for bit.
    c, arrs = make_inputs(SMALL[11], seed=21)
    gd = grid_dict(c)
    g = _grid(gd)
    B, H, d = c["batch"], c["heads"], c["d"]
    scale = 1 / math.sqrt(d)
    dev = torch.device("cuda:0")
    fold = lambda a: torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).contiguous()
    q, k, v, dout = (fold(a) for a in arrs)
    out, lse = torch.empty_like(q), torch.empty((B, H) + q.shape[3:], dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(max(S.s2_nattn_bwd_workspace_bytes(g, B, H, d, d), 1), dtype=torch.uint8, device=dev)

    def step():
        S.s2_nattn_fwd(g, q, k, v, scale, out=out, lse=lse)
        S.s2_nattn_bwd(g, q, k, v, out, lse, dout, scale, dq=dq, dk=dk, dv=dv, workspace=ws)

    step()                                  # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()              # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    rng = np.random.default_rng(3)
    for rep in range(3):
        q.copy_(torch.from_numpy(rng.standard_normal(tuple(q.shape)).astype(np.float32)).to(dev))
        dout.copy_(torch.from_numpy(rng.standard_normal(tuple(dout.shape)).astype(np.float32)).to(dev))
        step()
        torch.cuda.synchronize()
        eager = [t.clone() for t in (out, lse, dq, dk, dv)]
        for t in (out, lse, dq, dk, dv):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "lse", "dq", "dk", "dv"), eager, (out, lse, dq, dk, dv)):
            assert torch.equal(a, b), "replay %d: %s differs from the eager result" % (rep, name)


@pytest.mark.parametrize("ci", [9, 26])
def test_repeated_launches_bit_identical(ci):
    # split kernels with nine slices (2:1 grid; upsampling): 1000 forward + backward launches on the same inputs give
    # the same bits every time.  (Regression test: without a wait for the wavefront's own LDS reads before the next
    # LDS-direct copy into the same buffer, dk of the 2:1 case differed in about 3 of 1000 launches.)
    c, arrs = make_inputs(SMALL[ci], seed=200 + ci)
    g = _grid(grid_dict(c))
    B, H, d = c["batch"], c["heads"], c["d"]
    scale = 1 / math.sqrt(d)
    dev = torch.device("cuda:0")
    fold = lambda a: torch.from_numpy(a).to(dev).reshape((B, H) + a.shape[1:]).contiguous()
    q, k, v, dout = (fold(a) for a in arrs)
    out0, lse0 = S.s2_nattn_fwd(g, q, k, v, scale)
    g0 = S.s2_nattn_bwd(g, q, k, v, out0, lse0, dout, scale)
    for it in range(1000):
        out, lse = S.s2_nattn_fwd(g, q, k, v, scale)
        gr = S.s2_nattn_bwd(g, q, k, v, out, lse, dout, scale)
        assert torch.equal(out, out0) and torch.equal(lse, lse0), "launch %d: forward differs" % it
        assert all(torch.equal(x, y) for x, y in zip(gr, g0)), "launch %d: backward differs" % it


@pytest.mark.parametrize("seed", range(64))
def test_random_small_grids(seed):
    # seeded random tiny problems over all grid types, equal / downsampling / upsampling longitude ratios,
    # unequal latitude counts, arbitrary head widths (d != e included), against the oracle's per-pair form
    rng = np.random.default_rng(9000 + seed)
    gt = int(rng.integers(0, 4))
    nlon_lo = int(rng.integers(3, 13))
    ratio = int(rng.choice([1, 1, 2, 3, 4]))
    up = bool(rng.integers(0, 2))
    nlon_in, nlon_out = (nlon_lo, nlon_lo * ratio) if up else (nlon_lo * ratio, nlon_lo)
    nlat_in, nlat_out = int(rng.integers(3, 15)), int(rng.integers(3, 15))
    theta = float(rng.uniform(0.6, 2.2))
    d, e = int(rng.integers(1, 21)), int(rng.integers(1, 21))
    nbh = int(rng.integers(1, 4))
    gd = dict(grid_type=gt, nlat_in=nlat_in, nlon_in=nlon_in, nlat_out=nlat_out, nlon_out=nlon_out, theta=theta)
    try:
        g = _grid(gd)
    except S.S2Error as err:      # a cutoff that leaves some output without a (positive-weight) neighbor
        assert err.code in (S.S2_ERR_EMPTY_NEIGHBORHOOD, S.S2_ERR_AMBIGUOUS_CUTOFF)
        pytest.skip("cutoff rejected for this random grid")
    q = rng.standard_normal((nbh, d, nlat_out, nlon_out)).astype(np.float32)
    k = rng.standard_normal((nbh, d, nlat_in, nlon_in)).astype(np.float32)
    v = rng.standard_normal((nbh, e, nlat_in, nlon_in)).astype(np.float32)
    go = rng.standard_normal((nbh, e, nlat_out, nlon_out)).astype(np.float32)
    scale = float(rng.uniform(0.1, 0.6))
    dev = torch.device("cuda:0")
    t = lambda a: torch.from_numpy(a).to(dev).reshape((1,) + a.shape).contiguous()
    out, lse = S.s2_nattn_fwd(g, t(q), t(k), t(v), scale)
    dq, dk, dv = S.s2_nattn_bwd(g, t(q), t(k), t(v), out, lse, t(go), scale)
    torch.cuda.synchronize()
    a64 = [a.astype(np.float64) for a in (q, k, v, go)]
    r_out, r_lse = O.nattn_fwd(gd, a64[0], a64[1], a64[2], scale, brute=True)
    r_dq, r_dk, r_dv = O.nattn_bwd(gd, *a64, scale, brute=True)
    c_out, c_lse, c_dq, c_dk, c_dv = O.nattn_cond(gd, *a64, scale, brute=True)
    n = lambda x: x[0].cpu().numpy().astype(np.float64)
    cs = "rand%d" % seed
    for what, x, ref, cnd in (("out", out, r_out, c_out), ("lse", lse, r_lse, c_lse), ("dq", dq, r_dq, c_dq),
                              ("dk", dk, r_dk, c_dk), ("dv", dv, r_dv, c_dv)):
        compare(n(x), ref, what, cnd, C_DERIVED, cs)


@pytest.mark.parametrize("seed", range(48))
def test_random_tuned_shapes(seed):
    # seeded random medium-size problems on the tuned kernels (d = e = 32, longitude counts that are multiples of
    # 4 from 72 up, equal grids or 2:1 downsampling, all grid types, random cutoffs and slice counts): whichever mix of
    # matrix-core, streaming, split and one-wave launches the dispatch picks must match the oracle
    rng = np.random.default_rng(7000 + seed)
    gt = int(rng.integers(0, 4))
    ps = int(rng.integers(1, 3))
    nlon_out = 4 * int(rng.integers(18, 66))
    nlat_out = int(rng.integers(9, 40))
    nlat_in = nlat_out if rng.integers(0, 2) else int(rng.integers(9, 40))
    theta = float(rng.uniform(1.5, 6.0)) * math.pi / nlat_out
    c = dict(kind="nattn", grid_type=gt, nlat_in=nlat_in, nlon_in=nlon_out * ps, nlat_out=nlat_out, nlon_out=nlon_out,
             theta=theta, batch=int(rng.integers(1, 4)), heads=int(rng.integers(1, 4)), d=32, dtype="f32")
    try:
        _grid(grid_dict(c))
    except S.S2Error as err:
        assert err.code in (S.S2_ERR_EMPTY_NEIGHBORHOOD, S.S2_ERR_AMBIGUOUS_CUTOFF)
        pytest.skip("cutoff rejected for this random grid")
    c, arrs = make_inputs(c, seed=300 + seed)
    nbh = c["batch"] * c["heads"]
    run_case(c, arrs, [int(rng.integers(0, nbh))], case="tuned%d" % seed)


@pytest.mark.parametrize("seed", range(16))
def test_random_tuned_upsampling(seed):
    # the same for upsampling grids (2x, 3x, 4x) on the tuned kernels, against the oracle's per-pair form
    rng = np.random.default_rng(7500 + seed)
    gt = int(rng.integers(0, 4))
    up = int(rng.integers(2, 5))
    nlon_in = 4 * int(rng.integers(18, 41))
    nlat_in = int(rng.integers(7, 22))
    nlat_out = nlat_in if rng.integers(0, 2) else int(rng.integers(7, 22))
    theta = float(rng.uniform(1.5, 6.0)) * math.pi / min(nlat_in, nlat_out)
    c = dict(kind="nattn", grid_type=gt, nlat_in=nlat_in, nlon_in=nlon_in, nlat_out=nlat_out, nlon_out=nlon_in * up,
             theta=theta, batch=int(rng.integers(1, 4)), heads=int(rng.integers(1, 4)), d=32, dtype="f32")
    try:
        _grid(grid_dict(c))
    except S.S2Error as err:
        assert err.code in (S.S2_ERR_EMPTY_NEIGHBORHOOD, S.S2_ERR_AMBIGUOUS_CUTOFF)
        pytest.skip("cutoff rejected for this random grid")
    c, arrs = make_inputs(c, seed=400 + seed)
    nbh = c["batch"] * c["heads"]
    run_case(c, arrs, [int(rng.integers(0, nbh))], case="tuned-up%d" % seed)


def test_upsampling_full_size_parity():
    # 129x256 -> 257x512 (the mirror image of workload 4), all 8 slices on the GPU, two of them against the oracle's
    # per-pair form of eq. (5) evaluated on the fly
    c, arrs = make_inputs(6)
    run_case(c, arrs, [0, 5], C=C_DERIVED, case="cfg6")


def test_upsampling_full_size_invariants():
    # 129x256 -> 257x512 (the mirror image of workload 4) is too large for the oracle's per-pair form: properties
    # that hold at any size instead.  One slice, d = 32, tuned kernels in their class view.
    c = dict(CONFIGS[6], batch=1, heads=1)
    gd = grid_dict(c)
    g = _grid(gd)
    d, r = c["d"], c["nlon_out"] // c["nlon_in"]
    scale = 1 / math.sqrt(d)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cpu").manual_seed(11)
    q = torch.randn((1, 1, d, c["nlat_out"], c["nlon_out"]), generator=gen).to(dev)
    k = torch.randn((1, 1, d, c["nlat_in"], c["nlon_in"]), generator=gen).to(dev)
    v = torch.randn((1, 1, d, c["nlat_in"], c["nlon_in"]), generator=gen).to(dev)
    go = torch.randn((1, 1, d, c["nlat_out"], c["nlon_out"]), generator=gen).to(dev)
    out, lse = S.s2_nattn_fwd(g, q, k, v, scale)
    dq, dk, dv = S.s2_nattn_bwd(g, q, k, v, out, lse, go, scale)
    # sum_j p_ij = 1: dv sums to dout per channel; the logits are bilinear: sum q.dq = sum k.dk
    assert torch.allclose(dv.double().sum((3, 4)), go.double().sum((3, 4)), rtol=1e-6, atol=1e-4)
    a, b = (q.double() * dq.double()).sum().item(), (k.double() * dk.double()).sum().item()
    assert abs(a - b) <= 1e-6 * max(abs(a), abs(b)) + 1e-4
    # constant v: the output is that constant and dq, dk vanish; constant k: dq vanishes
    vc = torch.full_like(v, 0.75)
    oc, lc = S.s2_nattn_fwd(g, q, k, vc, scale)
    assert torch.allclose(oc, torch.full_like(oc, 0.75), rtol=0, atol=2e-6)
    assert torch.equal(lc, lse)
    dqc, dkc, _ = S.s2_nattn_bwd(g, q, k, vc, oc, lc, go, scale)
    assert dqc.abs().max().item() < 2e-5 and dkc.abs().max().item() < 2e-5
    kc = torch.ones_like(k) * 0.3
    o2, l2 = S.s2_nattn_fwd(g, q, kc, v, scale)
    dq2, _, _ = S.s2_nattn_bwd(g, q, kc, v, o2, l2, go, scale)
    assert dq2.abs().max().item() < 2e-5
    # q = 0: lse = ln(sum of the weights in the disk), between the cap area of a slightly smaller and a slightly
    # larger cap (2 pi (1 - cos theta)), and out is the weighted mean of v
    o3, l3 = S.s2_nattn_fwd(g, torch.zeros_like(q), k, v, scale)
    area = torch.exp(l3.double())
    th = c["theta"]
    cap = lambda t: 2 * math.pi * (1 - math.cos(t))
    assert area.min().item() > cap(0.8 * th) and area.max().item() < cap(1.25 * th)
    # longitude shift: input rolled by one step = output rolled by r steps, bit for bit
    o4, l4 = S.s2_nattn_fwd(g, torch.roll(q, r, 4), torch.roll(k, 1, 4), torch.roll(v, 1, 4), scale)
    assert torch.equal(o4, torch.roll(out, r, 4)) and torch.equal(l4, torch.roll(lse, r, 3))
    torch.cuda.synchronize()


def test_errors_on_device():
    gd = grid_dict(1)
    g = _grid(gd)
    dev = torch.device("cuda:0")
    q = torch.zeros((1, 1, 8, 17, 32), device=dev)
    wide = torch.zeros((1, 1, 130, 17, 32), device=dev)
    with pytest.raises(S.S2Error) as ei:
        S.s2_nattn_fwd(g, wide, wide, wide, 1.0)
    assert ei.value.code == S.S2_ERR_UNSUPPORTED          # head dimensions above 128
    out, lse = S.s2_nattn_fwd(g, q, q, q, 1.0)
    with pytest.raises(S.S2Error) as ei:
        S.s2_nattn_bwd(g, q, q, q, out, lse, q, 1.0, workspace=torch.empty(16, dtype=torch.uint8, device=dev))
    assert ei.value.code == S.S2_ERR_WORKSPACE
    torch.cuda.synchronize()
