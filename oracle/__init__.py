"""CPU oracle (float64, plain C + OpenMP) for spherical attention.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of the benchmark.  The product package never imports this.
"""
from .s2_oracle import (  # noqa: F401
    EQUIANGULAR,
    EQUIANGULAR_TRAPEZOID,
    LEGENDRE_GAUSS,
    LEGENDRE_GAUSS_LOBATTO,
    build,
    geodesic,
    global_bwd,
    global_fwd,
    grid,
    indicator,
    indicator_point,
    nattn_bwd,
    nattn_cond,
    nattn_fwd,
    neighbor_csr,
    omega,
)
from .s2_layers import disco_bwd, disco_fwd, disco_psi, mha_bwd, mha_fwd  # noqa: F401,E402
