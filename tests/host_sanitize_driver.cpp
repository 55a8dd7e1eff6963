// Host precompute of the library (quadrature, geodesic-disk tables, introspection, error paths) exercised as a plain
// executable, built with AddressSanitizer and UndefinedBehaviorSanitizer on the host side (no kernel is compiled in:
// the per-device set-up hooks of the kernel files are stubbed).  Prints "sanitize driver ok" when every call
// returned what it should.
#include <cmath>
#include <cstdio>
#include <vector>

#include "s2_nattn_kernels.h"

int s2_nattn_tiled_configure() { return 0; }
int s2_nattn_bwd_tiled_configure() { return 0; }
int s2_nattn_stream_configure() { return 0; }
int s2_nattn_mfma_configure() { return 0; }
int s2_nattn_band_configure() { return 0; }
int s2_mha_configure() { return 0; }
int s2_static_scratch_setup(int) { return 0; }

static int check_grid(int type, int nlat_in, int nlon_in, int nlat_out, int nlon_out, double theta)
{
    s2_grid_t *g = nullptr;
    const int rc = s2_grid_init(type, nlat_in, nlon_in, nlat_out, nlon_out, theta, &g);
    if (rc != S2_OK) return rc;
    std::vector<double> colat(nlat_in), omega(nlat_in);
    if (s2_grid_get_weights(g, colat.data(), omega.data()) != S2_OK) return -100;
    double sum = 0.0;
    for (int h = 0; h < nlat_in; ++h) sum += omega[h] * nlon_in;
    if (type != S2_GRID_EQUIANGULAR_TRAPEZOID && std::fabs(sum - 4.0 * M_PI) > 1e-11) return -101;
    std::vector<int64_t> row_ptr(nlat_out + 1);
    std::vector<int32_t> col(size_t(s2_grid_num_neighbors(g)));
    if (s2_grid_get_neighbors(g, row_ptr.data(), col.data()) != S2_OK) return -102;
    if (row_ptr[nlat_out] != int64_t(col.size())) return -103;
    for (int h = 0; h < nlat_out; ++h)
        for (int w = 0; w < nlon_out; w += (nlon_out > 7 ? nlon_out / 7 : 1)) {
            int n = 0;
            if (s2_grid_get_neighbors_at(g, h, w, nullptr, &n) != S2_OK || n < 1) return -104;
            std::vector<int32_t> at(n);
            if (s2_grid_get_neighbors_at(g, h, w, at.data(), &n) != S2_OK) return -105;
            for (int i = 0; i < n; ++i)
                if (at[i] < 0 || at[i] >= nlat_in * nlon_in) return -106;
        }
    s2_grid_destroy(g);
    return S2_OK;
}

int main()
{
    struct Case { int type, nlat_in, nlon_in, nlat_out, nlon_out; double theta; int want; };
    const Case cases[] = {
        {S2_GRID_EQUIANGULAR, 17, 32, 17, 32, M_PI / 8, S2_OK},
        {S2_GRID_LEGENDRE_GAUSS, 64, 128, 64, 128, 7 * M_PI / 64, S2_OK},
        {S2_GRID_EQUIANGULAR, 129, 256, 129, 256, 4 * M_PI / 128, S2_OK},
        {S2_GRID_EQUIANGULAR, 65, 128, 33, 64, 0.2, S2_OK},
        {S2_GRID_EQUIANGULAR, 33, 64, 65, 128, 0.2, S2_OK},
        {S2_GRID_EQUIANGULAR, 9, 20, 17, 80, 0.6, S2_OK},
        {S2_GRID_EQUIANGULAR_TRAPEZOID, 16, 32, 16, 32, 0.45, S2_OK},
        {S2_GRID_EQUIANGULAR_TRAPEZOID, 12, 72, 16, 144, 0.5, S2_OK},
        {S2_GRID_LEGENDRE_GAUSS_LOBATTO, 17, 32, 17, 32, 0.45, S2_OK},
        {S2_GRID_EQUIANGULAR, 9, 16, 9, 16, M_PI, S2_OK},
        {S2_GRID_LEGENDRE_GAUSS, 2, 1, 2, 1, 0.2, S2_OK},
        {S2_GRID_EQUIANGULAR, 1, 16, 9, 16, 0.5, S2_ERR_INVALID_ARG},
        {S2_GRID_EQUIANGULAR, 9, 16, 9, 16, 0.0, S2_ERR_INVALID_ARG},
        {S2_GRID_EQUIANGULAR, 9, 15, 9, 10, 0.5, S2_ERR_UNSUPPORTED},
        {7, 9, 16, 9, 16, 0.5, S2_ERR_INVALID_ARG},
        {S2_GRID_EQUIANGULAR, 33, 64, 6, 64, 0.01, S2_ERR_EMPTY_NEIGHBORHOOD},
    };
    for (const Case &c : cases) {
        const int rc = check_grid(c.type, c.nlat_in, c.nlon_in, c.nlat_out, c.nlon_out, c.theta);
        if (rc != c.want) {
            std::printf("case %d %dx%d -> %dx%d theta %g: got %d (%s), want %d\n", c.type, c.nlat_in, c.nlon_in,
                        c.nlat_out, c.nlon_out, c.theta, rc, s2_last_error(), c.want);
            return 1;
        }
    }
    if (s2_grid_init(0, 9, 16, 9, 16, 0.5, nullptr) != S2_ERR_INVALID_ARG) return 2;
    if (s2_debug_control(S2_DEBUG_NO_MFMA, 0) != S2_DEBUG_NO_MFMA || s2_debug_control(0, ~0u) != 0) return 3;
    std::printf("sanitize driver ok\n");
    return 0;
}
