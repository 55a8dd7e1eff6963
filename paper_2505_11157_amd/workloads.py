"""The five synthetic workloads and their seeded input generator.

This module holds no arithmetic of the method: only shapes, cutoffs and
N(0,1) draws.  Both the HIP path and the CPU oracle are fed from here (by the
tests and the benchmark) so that they see identical inputs.

Recipe: numpy Generator(PCG64(1000 + cfg)), standard_normal float32, drawn in
the order q, k, v, dout in the library's tensor layout.  The grids, cutoffs
and shapes stand in for the paper's experiment shapes (128x256-class
equiangular / Gaussian grids, cutoffs of about four grid spacings, heads x 32
channels).  The bf16 workloads (global attention, and workload 7) round the
draws to bf16 (round to nearest even) before either side sees them.
"""
import math

import numpy as np

EQUIANGULAR = 0
LEGENDRE_GAUSS = 1
EQUIANGULAR_TRAPEZOID = 2
LEGENDRE_GAUSS_LOBATTO = 3

CONFIGS = {
    1: dict(kind="nattn", grid_type=EQUIANGULAR, nlat_in=17, nlon_in=32, nlat_out=17, nlon_out=32,
            theta=math.pi / 8, batch=1, heads=1, d=8, dtype="f32"),
    2: dict(kind="nattn", grid_type=LEGENDRE_GAUSS, nlat_in=64, nlon_in=128, nlat_out=64, nlon_out=128,
            theta=7 * math.pi / 64, batch=2, heads=4, d=32, dtype="f32"),
    3: dict(kind="nattn", grid_type=EQUIANGULAR, nlat_in=129, nlon_in=256, nlat_out=129, nlon_out=256,
            theta=4 * math.pi / 128, batch=4, heads=8, d=32, dtype="f32"),
    4: dict(kind="nattn", grid_type=EQUIANGULAR, nlat_in=257, nlon_in=512, nlat_out=129, nlon_out=256,
            theta=2 * math.pi / 128, batch=2, heads=4, d=32, dtype="f32"),
    5: dict(kind="global", grid_type=EQUIANGULAR, nlat_in=65, nlon_in=128, nlat_out=65, nlon_out=128,
            theta=math.pi, batch=4, heads=8, d=64, dtype="bf16"),
    # not one of the five reference workloads: the mirror image of workload 4 (a decoder's upsampling layer,
    # queries on the fine grid, keys and values on the coarse one), used to measure the upsampling path
    6: dict(kind="nattn", grid_type=EQUIANGULAR, nlat_in=129, nlon_in=256, nlat_out=257, nlon_out=512,
            theta=2 * math.pi / 128, batch=2, heads=4, d=32, dtype="f32"),
    # workload 3 with bf16 tensors (float32 accumulation and logsumexp): the reduced-precision variant of the
    # neighborhood path, measured as a secondary workload
    7: dict(kind="nattn", grid_type=EQUIANGULAR, nlat_in=129, nlon_in=256, nlat_out=129, nlon_out=256,
            theta=4 * math.pi / 128, batch=4, heads=8, d=32, dtype="bf16"),
    # workload 3 with other head dimensions (the paper's models vary the head width, App. C): the fp32 band-tile
    # matrix-core kernels
    8: dict(kind="nattn", grid_type=EQUIANGULAR, nlat_in=129, nlon_in=256, nlat_out=129, nlon_out=256,
            theta=4 * math.pi / 128, batch=4, heads=8, d=16, dtype="f32"),
    9: dict(kind="nattn", grid_type=EQUIANGULAR, nlat_in=129, nlon_in=256, nlat_out=129, nlon_out=256,
            theta=4 * math.pi / 128, batch=4, heads=8, d=64, dtype="f32"),
}


def grid_dict(cfg):
    c = CONFIGS[cfg] if isinstance(cfg, int) else cfg
    return {k: c[k] for k in ("grid_type", "nlat_in", "nlon_in", "nlat_out", "nlon_out", "theta")}


def round_to_bf16(x):
    """float32 array -> float32 array holding the nearest-even bf16 values."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def shapes(c):
    """Tensor shapes (q, k, v, dout) with batch and heads folded into one leading axis."""
    nbh = c["batch"] * c["heads"]
    d = c["d"]
    if c["kind"] == "global":
        n = c["nlat_in"] * c["nlon_in"]
        return (nbh, n, d), (nbh, n, d), (nbh, n, d), (nbh, n, d)
    so = (c["nlat_out"], c["nlon_out"])
    si = (c["nlat_in"], c["nlon_in"])
    return (nbh, d) + so, (nbh, d) + si, (nbh, d) + si, (nbh, d) + so


def make_inputs(cfg, seed=None, override=None):
    """Seeded float32 q, k, v, dout for a config number (or a config dict via override)."""
    c = dict(CONFIGS[cfg]) if isinstance(cfg, int) else dict(cfg)
    if override:
        c.update(override)
    if seed is None:
        seed = 1000 + (cfg if isinstance(cfg, int) else 0)
    rng = np.random.Generator(np.random.PCG64(seed))
    arrs = [rng.standard_normal(s, dtype=np.float32) for s in shapes(c)]
    if c["dtype"] == "bf16":
        arrs = [round_to_bf16(a) for a in arrs]
    return c, arrs
