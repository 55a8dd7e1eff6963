// Host precompute for spherical attention: quadrature weights and the compact
// geodesic-disk tables, in float64, plus the one upload to the device.
//
// Follows App. A.1 (quadrature on a lat-lon grid), Sec. 3.3 (equiangular and
// Gaussian grids), Sec. 3.2 eq. (5) (disk of geodesic radius theta_cutoff) and
// App. B.3 (the indicator depends on the output latitude only; every output
// longitude reuses it by a shift).
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <mutex>
#include <cstring>
#include <numeric>

#include "s2_nattn_kernels.h"

namespace {

constexpr double kPi = 3.141592653589793238462643383279502884;
constexpr double kTieTol = 1e-9;      // points within this of the cutoff count as inside
constexpr double kAmbiguous = 1e-12;  // |d - (theta + kTieTol)| below this is rejected

thread_local std::string g_last_error;

// Clenshaw-Curtis weights for int_0^pi f(t) sin t dt on t_h = pi h / n, written
// as the cosine series  w_h = (c_h / n) * sum''_{k even} 2/(1-k^2) cos(k h pi / n),
// the double prime halving the k = 0 and k = n terms.
void clenshaw_curtis_nodes(int nlat, std::vector<double> &colat, std::vector<double> &w)
{
    const int n = nlat - 1;
    colat.resize(nlat);
    w.resize(nlat);
    for (int h = 0; h <= n; ++h) {
        colat[h] = kPi * h / n;
        double series = 0.0;
        for (int k = 0; k <= n; k += 2) {
            double term = 2.0 / (1.0 - double(k) * double(k)) * std::cos(kPi * double(k) * double(h) / double(n));
            if (k == 0 || k == n) term *= 0.5;
            series += term;
        }
        w[h] = ((h == 0 || h == n) ? 1.0 : 2.0) / n * series;
    }
}

// Gauss-Legendre nodes by Newton iteration from Tricomi's estimate; weights
// from  w = 2 (1 - x^2) / (n P_{n-1}(x))^2.
void gauss_legendre_nodes(int n, std::vector<double> &colat, std::vector<double> &w)
{
    colat.resize(n);
    w.resize(n);
    for (int h = 0; h < n; ++h) {
        double x = (1.0 - (n - 1.0) / (8.0 * double(n) * n * n)) * std::cos(kPi * (4.0 * h + 3.0) / (4.0 * n + 2.0));
        double pm1 = 1.0;
        for (int it = 0; it < 64; ++it) {
            double p_prev = 1.0, p = x;
            for (int m = 1; m < n; ++m) {
                double p_next = ((2.0 * m + 1.0) * x * p - m * p_prev) / (m + 1.0);
                p_prev = p;
                p = p_next;
            }
            pm1 = p_prev;
            double deriv = n * (pm1 - x * p) / (1.0 - x * x);
            double step = p / deriv;
            x -= step;
            if (std::fabs(step) < 4e-16) break;
        }
        {   // P_{n-1} at the converged node
            double p_prev = 1.0, p = x;
            for (int m = 1; m < n; ++m) {
                double p_next = ((2.0 * m + 1.0) * x * p - m * p_prev) / (m + 1.0);
                p_prev = p;
                p = p_next;
            }
            pm1 = p_prev;
        }
        colat[h] = std::acos(x);
        w[h] = 2.0 * (1.0 - x * x) / (double(n) * n * pm1 * pm1);
    }
}

// Great-circle distance in haversine form, with hav and 1-hav both written as
// sums of non-negative terms so the result is accurate from 0 to pi:
//   hav   = sin^2(dt/2) cos^2(dp/2) + sin^2(st/2) sin^2(dp/2)
//   1-hav = cos^2(dt/2) cos^2(dp/2) + cos^2(st/2) sin^2(dp/2),  dt = t1-t2, st = t1+t2.
double great_circle(double t1, double t2, double dphi)
{
    const double sd = std::sin(0.5 * (t1 - t2)), cd = std::cos(0.5 * (t1 - t2));
    const double ss = std::sin(0.5 * (t1 + t2)), cs = std::cos(0.5 * (t1 + t2));
    const double sp = std::sin(0.5 * dphi), cp = std::cos(0.5 * dphi);
    const double hav = sd * sd * cp * cp + ss * ss * sp * sp;
    const double cohav = cd * cd * cp * cp + cs * cs * sp * sp;
    return 2.0 * std::atan2(std::sqrt(hav), std::sqrt(cohav));
}

// App. A.1 as printed: nlat equally spaced colatitudes starting at the north pole, the south pole left out,
// trapezoidal rule in colatitude: latitude weight = spacing * sin(colat).
void trapezoid_nodes(int nlat, std::vector<double> &colat, std::vector<double> &w)
{
    colat.resize(nlat);
    w.resize(nlat);
    const double spacing = kPi / nlat;
    for (int h = 0; h < nlat; ++h) {
        colat[h] = spacing * h;
        w[h] = h == 0 ? 0.0 : spacing * std::sin(colat[h]);
    }
}

// Gauss-Lobatto rule with n points: x = +-1 and the n-2 zeros of P'_{n-1}, which interlace the zeros of P_{n-1}:
// each one is bracketed by two neighbouring Gauss-Legendre nodes of order n-1 and found there by bisection on the
// sign of P'_{n-1} (derivative from the recurrence (1-x^2) P'_m = m (P_{m-1} - x P_m)), then bisected down to the last bit.  Weights 2 / (n (n-1) P_{n-1}(x)^2).
void gauss_lobatto_nodes(int n, std::vector<double> &colat, std::vector<double> &w)
{
    const int m = n - 1;
    auto eval = [m](double x, double &pm, double &dpm) {
        double p_prev = 1.0, p = m == 0 ? 1.0 : x;
        for (int k = 1; k < m; ++k) {
            const double p_next = ((2.0 * k + 1.0) * x * p - k * p_prev) / (k + 1.0);
            p_prev = p;
            p = p_next;
        }
        pm = p;
        dpm = m * (p_prev - x * p) / (1.0 - x * x);
    };
    std::vector<double> x(n);
    x[0] = 1.0;
    x[m] = -1.0;
    if (n > 2) {
        std::vector<double> gc, gw;
        gauss_legendre_nodes(m, gc, gw);              // zeros of P_m, north first (x decreasing)
        for (int i = 1; i < m; ++i) {
            double hi = std::cos(gc[i - 1]), lo = std::cos(gc[i]);      // P_m has one extremum in (lo, hi)
            double pm, dhi, dlo;
            eval(hi, pm, dhi);
            eval(lo, pm, dlo);
            for (int it = 0; it < 200 && hi - lo > 4e-16 * std::max(1.0, std::fabs(hi)); ++it) {
                const double mid = 0.5 * (lo + hi);
                double dmid;
                eval(mid, pm, dmid);
                if ((dmid > 0.0) == (dhi > 0.0)) { hi = mid; dhi = dmid; } else { lo = mid; dlo = dmid; }
                if (mid == lo && mid == hi) break;
            }
            x[i] = 0.5 * (lo + hi);
        }
    }
    colat.resize(n);
    w.resize(n);
    for (int i = 0; i < n; ++i) {
        double pm, dpm;
        if (i == 0) pm = 1.0;
        else if (i == m) pm = (m % 2) ? -1.0 : 1.0;
        else eval(x[i], pm, dpm);
        colat[i] = std::acos(x[i]);
        w[i] = 2.0 / (double(n) * m * pm * pm);
    }
}

int nodes(int grid_type, int nlat, std::vector<double> &colat, std::vector<double> &w)
{
    if (grid_type == S2_GRID_EQUIANGULAR) clenshaw_curtis_nodes(nlat, colat, w);
    else if (grid_type == S2_GRID_LEGENDRE_GAUSS) gauss_legendre_nodes(nlat, colat, w);
    else if (grid_type == S2_GRID_EQUIANGULAR_TRAPEZOID) trapezoid_nodes(nlat, colat, w);
    else if (grid_type == S2_GRID_LEGENDRE_GAUSS_LOBATTO) gauss_lobatto_nodes(nlat, colat, w);
    else return -1;
    return 0;
}

}  // namespace

void s2_set_error(const std::string &msg) { g_last_error = msg; }
int s2_fail(int code, const std::string &msg)
{
    g_last_error = msg;
    return code;
}

extern "C" const char *s2_last_error(void) { return g_last_error.c_str(); }

static int upload_tables(s2_grid *g)
{
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        g->on_device = false;
        return S2_OK;
    }
    S2_HIP_CHECK(hipGetDevice(&g->device));
    {
        // once per device: LDS limits of the kernels (not a stream operation, so it must not happen inside an
        // attention call that a caller may be capturing into a graph)
        static std::mutex mu;
        static std::vector<char> done;
        std::lock_guard<std::mutex> lock(mu);
        if (int(done.size()) < ndev) done.resize(ndev, 0);
        if (!done[g->device]) {
            if (s2_nattn_tiled_configure() || s2_nattn_bwd_tiled_configure() || s2_nattn_stream_configure() ||
                s2_nattn_mfma_configure() || s2_nattn_band_configure() || s2_mha_configure()) {
                (void)hipGetLastError();
                return s2_fail(S2_ERR_DEVICE, "raising the LDS limit of a kernel failed");
            }
            (void)s2_static_scratch_setup(g->device);   // on failure s2_nattn_bwd_static reports it
            done[g->device] = 1;
        }
    }
    std::vector<float> l2w(g->nlat_in);
    const double omega_ref = *std::max_element(g->omega_in.begin(), g->omega_in.end());
    for (int h = 0; h < g->nlat_in; ++h) l2w[h] = float(g->omega_in[h] / omega_ref);
    const int ntok = g->nlat_in * g->nlon_in;
    g->npad_tok = (ntok + 63) / 64 * 64;
    std::vector<float> wtok(g->npad_tok, 0.f);
    for (int j = 0; j < ntok; ++j) wtok[j] = l2w[j / g->nlon_in];
    const unsigned zero_word = 0u;
    // one blob: floats first, then the int tables, each 256-byte aligned
    struct Part { const void *src; size_t bytes; size_t off; };
    std::vector<Part> parts = {
        {l2w.data(), l2w.size() * sizeof(float), 0},
        {g->band_lo.data(), g->band_lo.size() * sizeof(int), 0},
        {g->band_n.data(), g->band_n.size() * sizeof(int), 0},
        {g->cnt.data(), g->cnt.size() * sizeof(int), 0},
        {g->tband_lo.data(), g->tband_lo.size() * sizeof(int), 0},
        {g->tband_n.data(), g->tband_n.size() * sizeof(int), 0},
        {g->tcnt.data(), g->tcnt.size() * sizeof(int), 0},
        {g->row_order.data(), g->row_order.size() * sizeof(int), 0},
        {g->trow_order.data(), g->trow_order.size() * sizeof(int), 0},
        {wtok.data(), wtok.size() * sizeof(float), 0},
        {g->st_cum.data(), g->st_cum.size() * sizeof(int), 0},
        {g->tst_cum.data(), g->tst_cum.size() * sizeof(int), 0},
        {&zero_word, sizeof(unsigned), 0},
        {g->ucnt.data(), g->ucnt.size() * sizeof(int), 0},
        {g->ulo.data(), g->ulo.size() * sizeof(int), 0},
    };
    size_t total = 0;
    for (auto &p : parts) {
        p.off = total;
        total += (p.bytes + 255) / 256 * 256;
    }
    std::vector<char> host(total, 0);
    for (auto &p : parts) std::memcpy(host.data() + p.off, p.src, p.bytes);
    if (hipMalloc(&g->dev_blob, total) != hipSuccess) {
        (void)hipGetLastError();
        return s2_fail(S2_ERR_ALLOC, "hipMalloc of the grid tables failed");
    }
    S2_HIP_CHECK(hipMemcpy(g->dev_blob, host.data(), total, hipMemcpyHostToDevice));
    char *base = static_cast<char *>(g->dev_blob);
    S2DeviceTables &t = g->dt;
    t.omega_rel = reinterpret_cast<const float *>(base + parts[0].off);
    t.ln_omega_ref = float(std::log(omega_ref));
    t.omega_ref = float(omega_ref);
    t.band_lo = reinterpret_cast<const int *>(base + parts[1].off);
    t.band_n = reinterpret_cast<const int *>(base + parts[2].off);
    t.cnt = reinterpret_cast<const int *>(base + parts[3].off);
    t.tband_lo = reinterpret_cast<const int *>(base + parts[4].off);
    t.tband_n = reinterpret_cast<const int *>(base + parts[5].off);
    t.tcnt = reinterpret_cast<const int *>(base + parts[6].off);
    t.row_order = reinterpret_cast<const int *>(base + parts[7].off);
    t.trow_order = reinterpret_cast<const int *>(base + parts[8].off);
    g->dev_w_tok = reinterpret_cast<const float *>(base + parts[9].off);
    t.st_cum = reinterpret_cast<const int *>(base + parts[10].off);
    t.tst_cum = reinterpret_cast<const int *>(base + parts[11].off);
    t.dev_flags = reinterpret_cast<unsigned *>(base + parts[12].off);
    t.upscale = g->upscale;
    t.ucnt = reinterpret_cast<const int *>(base + parts[13].off);
    t.ulo = reinterpret_cast<const int *>(base + parts[14].off);
    t.band_max = g->band_max;
    t.tband_max = g->tband_max;
    t.nlat_in = g->nlat_in; t.nlon_in = g->nlon_in;
    t.nlat_out = g->nlat_out; t.nlon_out = g->nlon_out;
    t.pscale = g->pscale;
    g->on_device = true;
    return S2_OK;
}

extern "C" int s2_grid_init(int grid_type, int nlat_in, int nlon_in, int nlat_out, int nlon_out,
                            double theta_cutoff, s2_grid_t **out_grid)
{
    if (!out_grid) return s2_fail(S2_ERR_INVALID_ARG, "out_grid is NULL");
    *out_grid = nullptr;
    if (grid_type != S2_GRID_EQUIANGULAR && grid_type != S2_GRID_LEGENDRE_GAUSS &&
        grid_type != S2_GRID_EQUIANGULAR_TRAPEZOID && grid_type != S2_GRID_LEGENDRE_GAUSS_LOBATTO)
        return s2_fail(S2_ERR_INVALID_ARG, "unknown grid_type");
    if (nlat_in < 2 || nlat_out < 2 || nlon_in < 1 || nlon_out < 1)
        return s2_fail(S2_ERR_INVALID_ARG, "need nlat >= 2 and nlon >= 1 on both grids");
    if (nlat_in > 32768 || nlon_in > 65536 || nlat_out > 32768 || nlon_out > 65536)
        return s2_fail(S2_ERR_INVALID_ARG, "grid too large");
    if (!(theta_cutoff > 0.0) || theta_cutoff > kPi + 1e-12)
        return s2_fail(S2_ERR_INVALID_ARG, "theta_cutoff must lie in (0, pi]");
    if (nlon_in % nlon_out != 0 && nlon_out % nlon_in != 0)
        return s2_fail(S2_ERR_UNSUPPORTED,
                       "nlon_in must be a multiple of nlon_out or the other way round (longitude shift invariance)");

    s2_grid *g = new (std::nothrow) s2_grid();
    if (!g) return s2_fail(S2_ERR_ALLOC, "out of host memory");
    g->grid_type = grid_type;
    g->nlat_in = nlat_in; g->nlon_in = nlon_in; g->nlat_out = nlat_out; g->nlon_out = nlon_out;
    g->upscale = nlon_out > nlon_in ? nlon_out / nlon_in : 1;
    g->pscale = g->upscale > 1 ? 1 : nlon_in / nlon_out;
    g->theta = theta_cutoff;
    std::vector<double> wlat_in, wlat_out;
    nodes(grid_type, nlat_in, g->colat_in, wlat_in);
    nodes(grid_type, nlat_out, g->colat_out, wlat_out);
    g->omega_in.resize(nlat_in);
    for (int h = 0; h < nlat_in; ++h) g->omega_in[h] = wlat_in[h] * (2.0 * kPi / nlon_in);

    // cnt_full[h][h'] = number of member longitudes of input latitude h'
    const double limit = theta_cutoff + kTieTol;
    std::vector<int> cnt_full(size_t(nlat_out) * nlat_in, 0);
    std::vector<char> member(nlon_in);
    for (int h = 0; h < nlat_out; ++h) {
        for (int hp = 0; hp < nlat_in; ++hp) {
            // the closest point of latitude circle h' lies on the output meridian
            if (std::fabs(g->colat_out[h] - g->colat_in[hp]) > limit + 1e-6) continue;
            int c = 0;
            for (int wp = 0; wp < nlon_in; ++wp) {
                const double dist = great_circle(g->colat_out[h], g->colat_in[hp], 2.0 * kPi * wp / nlon_in);
                if (std::fabs(dist - limit) < kAmbiguous && limit < kPi) {
                    delete g;
                    return s2_fail(S2_ERR_AMBIGUOUS_CUTOFF,
                                   "a grid point lies within 1e-12 rad of the inclusion threshold; perturb theta_cutoff");
                }
                member[wp] = dist <= limit;
                c += member[wp];
            }
            // the disk cuts a latitude circle in one arc centred on the output meridian
            const int hw = (c - 1) / 2;
            for (int wp = 0; wp < nlon_in && c > 0 && c < nlon_in; ++wp) {
                const bool want = std::min(wp, nlon_in - wp) <= hw;
                if (want != bool(member[wp]) || c % 2 == 0) {
                    delete g;
                    return s2_fail(S2_ERR_UNSUPPORTED, "internal: neighborhood is not a centred arc");
                }
            }
            cnt_full[size_t(h) * nlat_in + hp] = c;
        }
    }

    auto build_bands = [&](int n_rows, int n_cols, auto at, std::vector<int> &lo, std::vector<int> &n,
                           std::vector<int> &tab, int &bmax) -> bool {
        lo.assign(n_rows, 0);
        n.assign(n_rows, 0);
        bmax = 0;
        for (int r = 0; r < n_rows; ++r) {
            int first = -1, last = -1;
            for (int c = 0; c < n_cols; ++c)
                if (at(r, c) > 0) { if (first < 0) first = c; last = c; }
            if (first < 0) continue;
            for (int c = first; c <= last; ++c)
                if (at(r, c) <= 0) return false;   // band must be contiguous
            lo[r] = first;
            n[r] = last - first + 1;
            bmax = std::max(bmax, n[r]);
        }
        tab.assign(size_t(n_rows) * std::max(bmax, 1), 0);
        for (int r = 0; r < n_rows; ++r)
            for (int b = 0; b < n[r]; ++b) tab[size_t(r) * bmax + b] = at(r, lo[r] + b);
        return true;
    };
    bool ok = build_bands(nlat_out, nlat_in, [&](int h, int hp) { return cnt_full[size_t(h) * nlat_in + hp]; },
                          g->band_lo, g->band_n, g->cnt, g->band_max);
    ok = ok && build_bands(nlat_in, nlat_out, [&](int hp, int h) { return cnt_full[size_t(h) * nlat_in + hp]; },
                           g->tband_lo, g->tband_n, g->tcnt, g->tband_max);
    if (!ok) { delete g; return s2_fail(S2_ERR_UNSUPPORTED, "internal: latitude band is not contiguous"); }
    for (int h = 0; h < nlat_out; ++h) {
        // a neighborhood must hold at least one point of positive weight (the trapezoid grid has a zero-weight pole row)
        bool positive = false;
        for (int b = 0; b < g->band_n[h]; ++b) positive = positive || g->omega_in[g->band_lo[h] + b] > 0.0;
        if (!positive) {
            delete g;
            return s2_fail(S2_ERR_EMPTY_NEIGHBORHOOD,
                           "an output point has no input point of positive weight within theta_cutoff");
        }
    }

    // upsampling: arcs for the output longitudes between two input meridians (classes s = 1 .. upscale-1; s = 0 is
    // the centred arc above).  An output point off the input meridians is farther from every input latitude circle
    // than the one on the meridian, so the band of class 0 covers all classes (arcs may be empty).
    if (g->upscale > 1) {
        const int r = g->upscale;
        g->ucnt.assign(size_t(nlat_out) * r * g->band_max, 0);
        g->ulo.assign(size_t(nlat_out) * r * g->band_max, 0);
        for (int h = 0; h < nlat_out; ++h)
            for (int sc = 0; sc < r; ++sc)
                for (int b = 0; b < g->band_n[h]; ++b) {
                    const int hp = g->band_lo[h] + b;
                    int c = 0;
                    for (int wp = 0; wp < nlon_in; ++wp) {
                        const double dphi = 2.0 * kPi * (double(wp) / nlon_in - double(sc) / nlon_out);
                        const double dist = great_circle(g->colat_out[h], g->colat_in[hp], dphi);
                        if (std::fabs(dist - limit) < kAmbiguous && limit < kPi) {
                            delete g;
                            return s2_fail(S2_ERR_AMBIGUOUS_CUTOFF,
                                           "a grid point lies within 1e-12 rad of the inclusion threshold; perturb theta_cutoff");
                        }
                        member[wp] = dist <= limit;
                        c += member[wp];
                    }
                    int start = 0;
                    if (c > 0 && c < nlon_in) {
                        // the arc is one circular interval: it starts where a member follows a non-member
                        int nstart = 0;
                        for (int wp = 0; wp < nlon_in; ++wp)
                            if (member[wp] && !member[(wp + nlon_in - 1) % nlon_in]) { start = wp; ++nstart; }
                        if (nstart != 1) {
                            delete g;
                            return s2_fail(S2_ERR_UNSUPPORTED, "internal: neighborhood is not one arc");
                        }
                        if (start > nlon_in / 2) start -= nlon_in;      // signed offset from the meridian at or below
                    }
                    const size_t at = (size_t(h) * r + sc) * g->band_max + b;
                    g->ucnt[at] = c;
                    g->ulo[at] = start;
                }
        // an output between two input meridians is farther from every input point than the one on the meridian:
        // it can be left without a (positive-weight) neighbor although class 0 has one
        for (int h = 0; h < nlat_out; ++h)
            for (int sc = 0; sc < r; ++sc) {
                bool positive = false;
                for (int b = 0; b < g->band_n[h]; ++b)
                    positive = positive || (g->ucnt[(size_t(h) * r + sc) * g->band_max + b] > 0 &&
                                            g->omega_in[g->band_lo[h] + b] > 0.0);
                if (!positive) {
                    delete g;
                    return s2_fail(S2_ERR_EMPTY_NEIGHBORHOOD,
                                   "an output point has no input point of positive weight within theta_cutoff");
                }
            }
    }

    // canonical CSR: ascending h'*nlon_in + w', w' in [0, nlon_in)
    g->row_ptr.assign(nlat_out + 1, 0);
    for (int h = 0; h < nlat_out; ++h) {
        for (int b = 0; b < g->band_n[h]; ++b) {
            const int hp = g->band_lo[h] + b, c = g->cnt[size_t(h) * g->band_max + b];
            if (c == nlon_in) {
                for (int wp = 0; wp < nlon_in; ++wp) g->col.push_back(hp * nlon_in + wp);
            } else {
                const int hw = (c - 1) / 2;
                for (int wp = 0; wp <= hw; ++wp) g->col.push_back(hp * nlon_in + wp);
                for (int wp = nlon_in - hw; wp < nlon_in; ++wp) g->col.push_back(hp * nlon_in + wp);
            }
        }
        g->row_ptr[h + 1] = int64_t(g->col.size());
    }

    // The introspection calls keep the lists as eq. (5) defines them.  The kernels never meet an input latitude of
    // weight zero (the pole row of the grid of App. A.1): its points contribute nothing to any sum, but their
    // logits would enter the running maximum of the softmax, and a pole logit far above all others would let every
    // positive-weight term underflow.  Equal grids and downsampling: such rows are cut off the ends of the bands;
    // upsampling (whose dk/dv walk indexes the class tables by input latitude): their arcs are emptied.
    g->c_band_lo = g->band_lo; g->c_band_n = g->band_n; g->c_cnt = g->cnt; g->c_ucnt = g->ucnt; g->c_ulo = g->ulo;
    g->c_band_max = g->band_max;
    for (int hp = 0; hp < nlat_in; ++hp)
        if (!(g->omega_in[hp] > 0.0)) g->zero_lat.push_back(hp);
    if (!g->zero_lat.empty()) {
        if (g->upscale > 1) {
            for (int h = 0; h < nlat_out; ++h)
                for (int sc = 0; sc < g->upscale; ++sc)
                    for (int b = 0; b < g->band_n[h]; ++b)
                        if (!(g->omega_in[g->band_lo[h] + b] > 0.0)) g->ucnt[(size_t(h) * g->upscale + sc) * g->band_max + b] = 0;
        } else {
            for (int h = 0; h < nlat_out; ++h) {
                int lo = g->band_lo[h], n = g->band_n[h], skip = 0;
                while (n > 0 && !(g->omega_in[lo + n - 1] > 0.0)) --n;
                while (n > 0 && !(g->omega_in[lo + skip] > 0.0)) { ++skip; --n; }
                for (int b = 0; b < g->band_max; ++b)
                    g->cnt[size_t(h) * g->band_max + b] = b < n ? g->c_cnt[size_t(h) * g->band_max + b + skip] : 0;
                g->band_lo[h] = lo + skip;
                g->band_n[h] = n;            // > 0: every neighborhood holds a point of positive weight
            }
        }
    }

    // work of a latitude: offsets per output point (summed over its band), resp. per input latitude over its
    // transposed band, with the number of (output, input) pairs it stands for.  Upsampling: mean over the longitude classes
    // (forward) and the sum over output latitudes and classes of the arcs that hold an input point (backward).
    std::vector<long> work_out(nlat_out, 0), work_in(nlat_in, 0);
    std::vector<double> pairs_out(nlat_out, 0.0), pairs_in(nlat_in, 0.0);
    if (g->upscale > 1) {
        const int r = g->upscale;
        for (int h = 0; h < nlat_out; ++h)
            for (int sc = 0; sc < r; ++sc)
                for (int b = 0; b < g->band_n[h]; ++b) {
                    const int c = g->ucnt[(size_t(h) * r + sc) * g->band_max + b];
                    work_out[h] += c;
                    work_in[g->band_lo[h] + b] += c;
                }
        for (int h = 0; h < nlat_out; ++h) {
            pairs_out[h] = double(work_out[h]) * nlon_in;
            work_out[h] = (work_out[h] + r - 1) / r;
        }
        for (int hp = 0; hp < nlat_in; ++hp) pairs_in[hp] = double(work_in[hp]) * nlon_in;
    } else {
        for (int h = 0; h < nlat_out; ++h)
            for (int b = 0; b < g->band_n[h]; ++b) work_out[h] += g->cnt[size_t(h) * g->band_max + b];
        for (int hp = 0; hp < nlat_in; ++hp)
            for (int b = 0; b < g->tband_n[hp]; ++b) work_in[hp] += g->tcnt[size_t(hp) * g->tband_max + b];
        for (int h = 0; h < nlat_out; ++h) pairs_out[h] = double(work_out[h]) * nlon_out;
        for (int hp = 0; hp < nlat_in; ++hp) pairs_in[hp] = double(work_in[hp]) * nlon_out;
    }
    // latitudes sorted by work, heaviest first: launch order for load balance
    auto order_by_work = [](const std::vector<long> &work, std::vector<int> &order) {
        order.resize(work.size());
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return work[a] > work[b]; });
    };
    order_by_work(work_out, g->row_order);
    order_by_work(work_in, g->trow_order);
    // split classes: a latitude whose disk holds more than 260 * P / 2 offsets per point is split P ways
    constexpr long T = 260;
    auto classify = [](const std::vector<long> &work, const std::vector<double> &row_pairs, long thr, int (&cls)[4],
                       double (&pairs)[4]) {
        cls[0] = cls[1] = cls[2] = cls[3] = 0;
        pairs[0] = pairs[1] = pairs[2] = pairs[3] = 0.0;
        for (size_t r = 0; r < work.size(); ++r) {
            const long w = work[r];
            const int c = w > 4 * thr ? 0 : w > 2 * thr ? 1 : w > thr ? 2 : 3;
            ++cls[c];
            pairs[c] += row_pairs[r];
        }
    };
    classify(work_out, pairs_out, T, g->dt.fwd_cls, g->dt.fwd_pairs);
    classify(work_in, pairs_in, T, g->dt.bwd_cls, g->dt.bwd_pairs);
    classify(work_out, pairs_out, T / 4, g->dt.fwd_cls_fine, g->dt.fwd_pairs_fine);
    classify(work_in, pairs_in, T / 4, g->dt.bwd_cls_fine, g->dt.bwd_pairs_fine);

    // streaming plan for the light latitudes (work <= T): they must form one contiguous range whose bands
    // move monotonically, with short odd arcs (at most 65 offsets) on every row of the band
    auto stream_plan = [](int n_rows, const std::vector<int> &lo, const std::vector<int> &n, const std::vector<int> &tab,
                          int bmax, int &p_lo, int &p_hi, int &p_nw, std::vector<int> &cum) {
        p_lo = p_hi = p_nw = 0;
        cum.assign(1, 0);
        int first = -1, last = -1, count = 0;
        for (int r = 0; r < n_rows; ++r) {
            long work = 0;
            for (int b = 0; b < n[r]; ++b) work += tab[size_t(r) * bmax + b];
            if (work > T) continue;
            if (first < 0) first = r;
            last = r;
            ++count;
        }
        if (count == 0 || last - first + 1 != count) return;
        for (int r = first; r <= last; ++r) {
            if (n[r] < 1) return;
            for (int b = 0; b < n[r]; ++b) {
                const int c = tab[size_t(r) * bmax + b];
                if (c < 1 || c > 65 || c % 2 == 0) return;
            }
            if (r > first && (lo[r] < lo[r - 1] || lo[r] + n[r] < lo[r - 1] + n[r - 1])) return;
        }
        for (int w = 1; w <= 8; ++w) {
            bool ok = true;
            for (int r = first; r + w <= last && ok; ++r) ok = lo[r + w] >= lo[r] + n[r] - 1;
            if (!ok) continue;
            p_lo = first; p_hi = last + 1; p_nw = w;
            // cost of a latitude: offsets plus a fixed charge per band row (run set-up, softmax bookkeeping)
            for (int r = first; r <= last; ++r) {
                int c = 0;
                for (int b = 0; b < n[r]; ++b) c += tab[size_t(r) * bmax + b] + 2;
                cum.push_back(cum.back() + c);
            }
            return;
        }
    };
    stream_plan(nlat_out, g->band_lo, g->band_n, g->cnt, g->band_max, g->dt.st_lo, g->dt.st_hi, g->dt.st_nw,
                g->st_cum);
    stream_plan(nlat_in, g->tband_lo, g->tband_n, g->tcnt, g->tband_max, g->dt.tst_lo, g->dt.tst_hi, g->dt.tst_nw,
                g->tst_cum);

    // light range for the bf16 band-tile kernels: the latitudes of the last class must be one contiguous range with
    // odd arcs of at most 57 offsets (a 128-column stage then holds the window of 64 owners on every band row), and
    // the bands of four consecutive latitudes together span at most 64 rows (a workgroup keeps one row per lane)
    auto light_range = [](int n_rows, const std::vector<int> &blo, const std::vector<int> &n, const std::vector<int> &tab,
                          int bmax, int &lo, int &hi) {
        lo = hi = 0;
        int first = -1, last = -1, count = 0;
        for (int r = 0; r < n_rows; ++r) {
            long work = 0;
            for (int b = 0; b < n[r]; ++b) work += tab[size_t(r) * bmax + b];
            if (work > T) continue;
            if (first < 0) first = r;
            last = r;
            ++count;
        }
        if (count == 0 || last - first + 1 != count) return;
        for (int r = first; r <= last; ++r) {
            if (n[r] < 1) return;
            for (int b = 0; b < n[r]; ++b) {
                const int c = tab[size_t(r) * bmax + b];
                if (c < 1 || c > 57 || c % 2 == 0) return;
            }
        }
        for (int f = first; f <= last; f += 4) {
            int rmin = 1 << 30, rmax = -1;
            for (int r = f; r <= std::min(f + 3, last); ++r) {
                rmin = std::min(rmin, blo[r]);
                rmax = std::max(rmax, blo[r] + n[r] - 1);
            }
            if (rmax - rmin + 1 > 64) return;
        }
        lo = first;
        hi = last + 1;
    };
    auto rows_ok = [](int n_rows, const std::vector<int> &blo, const std::vector<int> &n) {
        for (int f = 0; f < n_rows; f += 4) {
            int rmin = 1 << 30, rmax = -1;
            for (int r = f; r < std::min(f + 4, n_rows); ++r)
                if (n[r] > 0) {
                    rmin = std::min(rmin, blo[r]);
                    rmax = std::max(rmax, blo[r] + n[r] - 1);
                }
            if (rmax - rmin + 1 > 64) return false;
        }
        return true;
    };
    g->dt.band_rows_ok = rows_ok(nlat_out, g->band_lo, g->band_n) && rows_ok(nlat_in, g->tband_lo, g->tband_n);
    light_range(nlat_out, g->band_lo, g->band_n, g->cnt, g->band_max, g->dt.bl_lo, g->dt.bl_hi);
    light_range(nlat_in, g->tband_lo, g->tband_n, g->tcnt, g->tband_max, g->dt.tbl_lo, g->dt.tbl_hi);

    int rc = upload_tables(g);
    if (rc != S2_OK) { delete g; return rc; }
    *out_grid = g;
    return S2_OK;
}

double s2_great_circle(double colat_a, double colat_b, double dphi) { return great_circle(colat_a, colat_b, dphi); }

extern "C" void s2_grid_destroy(s2_grid_t *g)
{
    if (!g) return;
    if (g->dev_blob) (void)hipFree(g->dev_blob);
    delete g;
}

extern "C" int s2_grid_device_flags(const s2_grid_t *g, unsigned *flags)
{
    if (!g || !flags) return s2_fail(S2_ERR_INVALID_ARG, "grid or flags is NULL");
    if (!g->on_device) return s2_fail(S2_ERR_DEVICE, "the grid handle has no device tables");
    S2_HIP_CHECK(hipDeviceSynchronize());
    S2_HIP_CHECK(hipMemcpy(flags, g->dt.dev_flags, sizeof(unsigned), hipMemcpyDeviceToHost));
    if (*flags) S2_HIP_CHECK(hipMemset(g->dt.dev_flags, 0, sizeof(unsigned)));
    return S2_OK;
}

extern "C" int s2_grid_get_weights(const s2_grid_t *g, double *colat_in, double *omega_in)
{
    if (!g) return s2_fail(S2_ERR_INVALID_ARG, "grid is NULL");
    if (colat_in) std::memcpy(colat_in, g->colat_in.data(), sizeof(double) * g->nlat_in);
    if (omega_in) std::memcpy(omega_in, g->omega_in.data(), sizeof(double) * g->nlat_in);
    return S2_OK;
}

extern "C" int64_t s2_grid_num_neighbors(const s2_grid_t *g) { return g ? int64_t(g->col.size()) : 0; }

extern "C" int s2_grid_get_neighbors_at(const s2_grid_t *g, int h, int w, int32_t *col, int *count)
{
    if (!g || !count) return s2_fail(S2_ERR_INVALID_ARG, "grid or count is NULL");
    if (h < 0 || h >= g->nlat_out || w < 0 || w >= g->nlon_out) return s2_fail(S2_ERR_INVALID_ARG, "no such output point");
    const int r = g->upscale, sc = w % r, m = r > 1 ? w / r : w * g->pscale;
    std::vector<int32_t> list;
    for (int b = 0; b < g->c_band_n[h]; ++b) {
        const int hp = g->c_band_lo[h] + b;
        int c, lo;
        if (r > 1) {
            const size_t at = (size_t(h) * r + sc) * g->c_band_max + b;
            c = g->c_ucnt[at];
            lo = g->c_ulo[at];
        } else {
            c = g->c_cnt[size_t(h) * g->c_band_max + b];
            lo = c == g->nlon_in ? 0 : -((c - 1) / 2);
        }
        std::vector<int32_t> row;
        for (int tt = 0; tt < c; ++tt) row.push_back(hp * g->nlon_in + ((m + lo + tt) % g->nlon_in + g->nlon_in) % g->nlon_in);
        std::sort(row.begin(), row.end());
        list.insert(list.end(), row.begin(), row.end());
    }
    if (col) std::memcpy(col, list.data(), sizeof(int32_t) * list.size());
    *count = int(list.size());
    return S2_OK;
}

extern "C" int s2_grid_get_neighbors(const s2_grid_t *g, int64_t *row_ptr, int32_t *col)
{
    if (!g) return s2_fail(S2_ERR_INVALID_ARG, "grid is NULL");
    if (row_ptr) std::memcpy(row_ptr, g->row_ptr.data(), sizeof(int64_t) * g->row_ptr.size());
    if (col) std::memcpy(col, g->col.data(), sizeof(int32_t) * g->col.size());
    return S2_OK;
}
