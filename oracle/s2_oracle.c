/*
 * s2_oracle.c -- CPU oracle for quadrature-weighted attention on the sphere.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, float64 statement
 * of what the method computes.  It is linked by nothing in the product path:
 * only the test-suite, the smoke check and the cpu_baseline leg of the
 * benchmark may load it.  It shares no source, header, table or helper with
 * the HIP library.
 *
 * What each function follows (paper: "Attention on the Sphere"):
 *   grids / quadrature .......... App. A.1 (quadrature rule on a lat-lon grid),
 *                                 Sec. 3.3 (equiangular and Gaussian grids)
 *   geodesic disk D(x) .......... Sec. 3.2, eq. (5): d(x,x') <= theta_cutoff
 *   indicator 1[h,h',w'] ........ App. B.3 (shift invariance in longitude)
 *   neighborhood attention ...... App. B.1 second equation, and its index
 *                                 form in App. B.3
 *   global attention ............ App. B.1 first equation; App. B.2 (log w bias)
 *   gradients ................... App. B.4, re-derived from the forward
 *                                 definition (the printed expressions carry
 *                                 typos; finite differences arbitrate)
 *
 * Readings taken where the paper is silent:
 *   - equiangular grid = both poles, colat_h = pi*h/(nlat-1), Clenshaw-Curtis
 *     latitude weights (strictly positive, exact sum); the grid of App. A.1 as
 *     printed (no south pole, trapezoidal weights, zero at the pole) is a third type;
 *   - Gaussian grid = Legendre-Gauss nodes in cos(colat), north first;
 *   - omega[h'] = latitude weight * 2*pi/nlon_in (input grid);
 *   - a point belongs to the disk iff d <= theta_cutoff + 1e-9 rad (cutoffs
 *     that are multiples of the grid spacing put many points exactly on the
 *     boundary; the guard makes membership independent of the distance formula);
 *   - pole rows are nlon distinct samples, each with the pole weight;
 *   - logits are q.k*scale + ln(omega), scale passed in (1/sqrt(d) in the tests);
 *   - logsumexp is natural log and includes omega.
 *
 * Tensor layouts: neighborhood functions use channels-first
 *   q   [nbh][d][nlat_out][nlon_out]     k [nbh][d][nlat_in][nlon_in]
 *   v   [nbh][e][nlat_in][nlon_in]       out like q with e channels
 *   lse [nbh][nlat_out][nlon_out]
 * global functions use token-major  q,k [nbh][N][d], v,out [nbh][N][e],
 * lse [nbh][N], token j = h*nlon + w.
 *
 * Parity pins (tests/test_oracle_*.py): closed-form quadrature values and
 * polynomial exactness, analytic disk membership, brute force vs shift form,
 * dense masked-softmax through a library routine incl. autograd, theta=pi ==
 * global, finite differences, symmetry/equivariance invariants.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define S2O_EQUIANGULAR 0
#define S2O_LEGENDRE_GAUSS 1
#define S2O_EQUIANGULAR_TRAPEZOID 2
#define S2O_LEGENDRE_GAUSS_LOBATTO 3
#define S2O_TIE_TOL 1e-9

static const double S2O_PI = 3.14159265358979323846264338327950288;

/* ---------------------------------------------------------------- grids -- */

/* Clenshaw-Curtis weights on colat_h = pi*h/n, h = 0..n (n = nlat-1), for
 * the integral of f(colat) sin(colat) over [0,pi]; they sum to 2. */
static void clenshaw_curtis(int nlat, double *colat, double *w)
{
    int n = nlat - 1;
    for (int h = 0; h <= n; ++h) {
        colat[h] = S2O_PI * (double)h / (double)n;
        double acc = 0.0;
        for (int j = 1; j <= n / 2; ++j) {
            double bj = (2 * j == n) ? 1.0 : 2.0;
            acc += bj / (4.0 * j * j - 1.0) * cos(2.0 * j * h * S2O_PI / (double)n);
        }
        double ch = (h == 0 || h == n) ? 1.0 : 2.0;
        w[h] = ch / (double)n * (1.0 - acc);
    }
}

/* Legendre polynomial P_n(x) and its derivative by the three-term recurrence. */
static void legendre_pn(int n, double x, double *pn, double *dpn)
{
    double p0 = 1.0, p1 = x;
    if (n == 0) { *pn = 1.0; *dpn = 0.0; return; }
    for (int m = 2; m <= n; ++m) {
        double p2 = ((2.0 * m - 1.0) * x * p1 - (m - 1.0) * p0) / (double)m;
        p0 = p1; p1 = p2;
    }
    *pn = p1;
    *dpn = (double)n * (x * p1 - p0) / (x * x - 1.0);
}

/* Legendre-Gauss nodes x_h (decreasing: north pole side first) and weights. */
static void legendre_gauss(int nlat, double *colat, double *w)
{
    for (int h = 0; h < nlat; ++h) {
        double x = cos(S2O_PI * (h + 0.75) / (nlat + 0.5));
        for (int it = 0; it < 100; ++it) {
            double p, dp;
            legendre_pn(nlat, x, &p, &dp);
            double dx = p / dp;
            x -= dx;
            if (fabs(dx) < 1e-15) break;
        }
        double p, dp;
        legendre_pn(nlat, x, &p, &dp);
        colat[h] = acos(x);
        w[h] = 2.0 / ((1.0 - x * x) * dp * dp);
    }
}

/* The equiangular grid the paper itself writes down (App. A.1): colat_i = pi*i/nlat for
 * i = 0..nlat-1 (north pole included, south pole not) with the trapezoidal weights
 * q_ij = 2 pi^2 / (nlat nlon) sin(colat_i), i.e. latitude weight (pi/nlat) sin(colat_i) times
 * 2 pi / nlon.  The pole row has weight zero: its points never contribute (ln 0 = -inf in the
 * logits); the weights sum to 4 pi only approximately. */
static void equiangular_trapezoid(int nlat, double *colat, double *w)
{
    for (int i = 0; i < nlat; ++i) {
        colat[i] = S2O_PI * (double)i / (double)nlat;
        w[i] = S2O_PI / (double)nlat * sin(colat[i]);
    }
}

/* Legendre-Gauss-Lobatto rule with n = nlat points in x = cos(colat): both poles (x = +-1) are
 * nodes, the interior nodes are the zeros of P'_{n-1}, and w_i = 2 / (n (n-1) P_{n-1}(x_i)^2).
 * A Gaussian-type grid that, unlike the Legendre-Gauss one, has points at the poles.
 * Newton on P'_m (m = n-1) from the Chebyshev-Lobatto points; P''_m comes from Legendre's
 * equation (1-x^2) P'' = 2x P' - m(m+1) P. */
static void legendre_gauss_lobatto(int nlat, double *colat, double *w)
{
    int m = nlat - 1;
    for (int i = 0; i < nlat; ++i) {
        double x;
        if (i == 0) x = 1.0;
        else if (i == m) x = -1.0;
        else {
            x = cos(S2O_PI * (double)i / (double)m);
            for (int it = 0; it < 100; ++it) {
                double p, dp;
                legendre_pn(m, x, &p, &dp);
                double d2p = (2.0 * x * dp - (double)m * (m + 1.0) * p) / (1.0 - x * x);
                double dx = dp / d2p;
                x -= dx;
                if (fabs(dx) < 1e-15) break;
            }
        }
        double p, dp;
        if (i == 0) p = 1.0;
        else if (i == m) p = (m % 2) ? -1.0 : 1.0;
        else legendre_pn(m, x, &p, &dp);
        colat[i] = acos(x);
        w[i] = 2.0 / ((double)nlat * (double)m * p * p);
    }
}

/* colat[nlat], wlat[nlat] (wlat sums to 2, approximately for the trapezoid grid).
 * Returns 0, or -1 on bad input. */
int s2o_grid(int grid_type, int nlat, double *colat, double *wlat)
{
    if (nlat < 2) return -1;
    if (grid_type == S2O_EQUIANGULAR) clenshaw_curtis(nlat, colat, wlat);
    else if (grid_type == S2O_LEGENDRE_GAUSS) legendre_gauss(nlat, colat, wlat);
    else if (grid_type == S2O_EQUIANGULAR_TRAPEZOID) equiangular_trapezoid(nlat, colat, wlat);
    else if (grid_type == S2O_LEGENDRE_GAUSS_LOBATTO) legendre_gauss_lobatto(nlat, colat, wlat);
    else return -1;
    return 0;
}

/* ------------------------------------------------------------- distance -- */

/* Great-circle distance between two points given as (colatitude, longitude):
 * angle between unit vectors, atan2(|a x b|, a.b). */
double s2o_geodesic(double colat1, double lon1, double colat2, double lon2)
{
    double a[3] = { sin(colat1) * cos(lon1), sin(colat1) * sin(lon1), cos(colat1) };
    double b[3] = { sin(colat2) * cos(lon2), sin(colat2) * sin(lon2), cos(colat2) };
    double c[3] = { a[1] * b[2] - a[2] * b[1], a[2] * b[0] - a[0] * b[2], a[0] * b[1] - a[1] * b[0] };
    double dot = a[0] * b[0] + a[1] * b[1] + a[2] * b[2];
    return atan2(sqrt(c[0] * c[0] + c[1] * c[1] + c[2] * c[2]), dot);
}

/* Indicator in the shift-invariant form of App. B.3: mask[h][h'][w'] = 1 iff
 * input point (h', lon index w') lies in the disk around the output point
 * (h, longitude 0).  mask has nlat_out*nlat_in*nlon_in bytes. */
int s2o_indicator(int grid_type, int nlat_in, int nlon_in, int nlat_out, int nlon_out,
                  double theta, uint8_t *mask)
{
    (void)nlon_out;
    double *ci = malloc(sizeof(double) * nlat_in), *wi = malloc(sizeof(double) * nlat_in);
    double *co = malloc(sizeof(double) * nlat_out), *wo = malloc(sizeof(double) * nlat_out);
    int rc = s2o_grid(grid_type, nlat_in, ci, wi) | s2o_grid(grid_type, nlat_out, co, wo);
    if (rc == 0) {
#pragma omp parallel for schedule(static)
        for (int h = 0; h < nlat_out; ++h)
            for (int hp = 0; hp < nlat_in; ++hp)
                for (int wp = 0; wp < nlon_in; ++wp) {
                    double dist = s2o_geodesic(co[h], 0.0, ci[hp], 2.0 * S2O_PI * wp / (double)nlon_in);
                    mask[((size_t)h * nlat_in + hp) * nlon_in + wp] = (dist <= theta + S2O_TIE_TOL);
                }
    }
    free(ci); free(wi); free(co); free(wo);
    return rc;
}

/* Brute-force membership of eq. (5) for ONE output point (h, w): row[j] = 1
 * iff input point j = h'*nlon_in + w_in (absolute longitude index) lies in the
 * disk.  No use of shift invariance; any nlon_in, nlon_out. */
int s2o_indicator_point(int grid_type, int nlat_in, int nlon_in, int nlat_out, int nlon_out,
                        double theta, int h, int w, uint8_t *row)
{
    double *ci = malloc(sizeof(double) * nlat_in), *wi = malloc(sizeof(double) * nlat_in);
    double *co = malloc(sizeof(double) * nlat_out), *wo = malloc(sizeof(double) * nlat_out);
    int rc = s2o_grid(grid_type, nlat_in, ci, wi) | s2o_grid(grid_type, nlat_out, co, wo);
    if (rc == 0) {
        double lon_o = 2.0 * S2O_PI * w / (double)nlon_out;
        for (int hp = 0; hp < nlat_in; ++hp)
            for (int win = 0; win < nlon_in; ++win) {
                double dist = s2o_geodesic(co[h], lon_o, ci[hp], 2.0 * S2O_PI * win / (double)nlon_in);
                row[(size_t)hp * nlon_in + win] = (dist <= theta + S2O_TIE_TOL);
            }
    }
    free(ci); free(wi); free(co); free(wo);
    return rc;
}

/* ------------------------------------------------ neighborhood attention -- */

typedef struct {
    int brute;              /* 1: dense [N_out][N_in] mask from per-pair distances; 2: per-pair distances evaluated
                               on the fly, nothing stored (any grid size) */
    int nlat_in, nlon_in, nlat_out, nlon_out, pscale;
    uint8_t *m;
    double *logw;           /* ln omega per input latitude */
    double *ci, *co;        /* colatitudes of the input and output grids (brute == 2) */
    double theta;
} s2o_ctx;

static int ctx_init(s2o_ctx *C, int grid_type, int nlat_in, int nlon_in, int nlat_out, int nlon_out,
                    double theta, int brute)
{
    memset(C, 0, sizeof(*C));
    C->brute = brute;
    C->nlat_in = nlat_in; C->nlon_in = nlon_in; C->nlat_out = nlat_out; C->nlon_out = nlon_out;
    if (nlat_in < 2 || nlat_out < 2 || nlon_in < 1 || nlon_out < 1) return -1;
    if (!brute && nlon_in % nlon_out != 0) return -2;   /* shift form needs an integer ratio */
    C->pscale = brute ? 0 : nlon_in / nlon_out;
    size_t n_in = (size_t)nlat_in * nlon_in, n_out = (size_t)nlat_out * nlon_out;
    double *ci = malloc(sizeof(double) * nlat_in), *wi = malloc(sizeof(double) * nlat_in);
    if (s2o_grid(grid_type, nlat_in, ci, wi)) { free(ci); free(wi); return -1; }
    C->logw = malloc(sizeof(double) * nlat_in);
    for (int hp = 0; hp < nlat_in; ++hp) C->logw[hp] = log(wi[hp] * 2.0 * S2O_PI / (double)nlon_in);
    C->theta = theta;
    if (brute == 2) {
        /* eq. (5) per pair at the moment it is asked for: keeps the colatitudes, stores no mask */
        double *wo = malloc(sizeof(double) * nlat_out);
        C->ci = ci;
        C->co = malloc(sizeof(double) * nlat_out);
        int rc2 = s2o_grid(grid_type, nlat_out, C->co, wo);
        free(wi); free(wo);
        return rc2;
    }
    free(ci); free(wi);
    int rc = 0;
    if (brute) {
        C->m = malloc(n_out * n_in);
        for (int h = 0; h < nlat_out && !rc; ++h)
            for (int w = 0; w < nlon_out && !rc; ++w)
                rc = s2o_indicator_point(grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta, h, w,
                                         C->m + ((size_t)h * nlon_out + w) * n_in);
    } else {
        C->m = malloc((size_t)nlat_out * n_in);
        rc = s2o_indicator(grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta, C->m);
    }
    return rc;
}

static void ctx_free(s2o_ctx *C) { free(C->m); free(C->logw); free(C->ci); free(C->co); }

/* Is input point (hp, win) [absolute longitude index] in the disk of output (h, w)? */
static inline int member(const s2o_ctx *C, int h, int w, int hp, int win)
{
    if (C->brute == 2) {
        /* the distance is at least the difference of the colatitudes (the two meridian arcs to the pole and the
         * geodesic form a spherical triangle), so most pairs are decided without the trigonometry */
        if (fabs(C->co[h] - C->ci[hp]) > C->theta + 1e-6) return 0;
        double dist = s2o_geodesic(C->co[h], 2.0 * S2O_PI * w / (double)C->nlon_out,
                                   C->ci[hp], 2.0 * S2O_PI * win / (double)C->nlon_in);
        return dist <= C->theta + S2O_TIE_TOL;
    }
    if (C->brute)
        return C->m[((size_t)h * C->nlon_out + w) * ((size_t)C->nlat_in * C->nlon_in) + (size_t)hp * C->nlon_in + win];
    int wp = (win - w * C->pscale) % C->nlon_in;
    if (wp < 0) wp += C->nlon_in;
    return C->m[((size_t)h * C->nlat_in + hp) * C->nlon_in + wp];
}

/* logits s_ij (incl. ln omega) of one output point against every member input
 * point; non-members get -inf.  Returns the maximum. */
static double point_logits(const s2o_ctx *C, int d, double scale, const double *qb, const double *kb,
                           int h, int w, double *s)
{
    size_t so = (size_t)C->nlat_out * C->nlon_out, si = (size_t)C->nlat_in * C->nlon_in;
    double m = -INFINITY;
    for (int hp = 0; hp < C->nlat_in; ++hp)
        for (int win = 0; win < C->nlon_in; ++win) {
            size_t j = (size_t)hp * C->nlon_in + win;
            if (!member(C, h, w, hp, win)) { s[j] = -INFINITY; continue; }
            double dot = 0.0;
            for (int l = 0; l < d; ++l)
                dot += qb[l * so + (size_t)h * C->nlon_out + w] * kb[l * si + j];
            s[j] = dot * scale + C->logw[hp];
            if (s[j] > m) m = s[j];
        }
    return m;
}

/* Forward.  out [nbh][e][nlat_out][nlon_out], lse [nbh][nlat_out][nlon_out].
 * brute = 1 evaluates the disk per (output, input) pair from eq. (5) without
 * shift invariance (tiny grids only: N_out*N_in bytes).  Returns 0 or <0. */
int s2o_nattn_fwd(int grid_type, int nlat_in, int nlon_in, int nlat_out, int nlon_out, double theta,
                  int brute, int nbh, int d, int e, double scale,
                  const double *q, const double *k, const double *v, double *out, double *lse)
{
    s2o_ctx C;
    int rc = ctx_init(&C, grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta, brute);
    if (rc) { ctx_free(&C); return rc; }
    size_t so = (size_t)nlat_out * nlon_out, si = (size_t)nlat_in * nlon_in;
    long total = (long)nbh * (long)so;
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * si);
        double *oi = malloc(sizeof(double) * e);
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < total; ++t) {
            int b = (int)(t / (long)so);
            int i = (int)(t % (long)so);
            int h = i / nlon_out, w = i % nlon_out;
            const double *qb = q + (size_t)b * d * so, *kb = k + (size_t)b * d * si, *vb = v + (size_t)b * e * si;
            double m = point_logits(&C, d, scale, qb, kb, h, w, s);
            double Z = 0.0;
            for (size_t j = 0; j < si; ++j)
                if (s[j] != -INFINITY) Z += exp(s[j] - m);
            double L = m + log(Z);
            lse[(size_t)b * so + i] = L;
            for (int c = 0; c < e; ++c) oi[c] = 0.0;
            for (size_t j = 0; j < si; ++j) {
                if (s[j] == -INFINITY) continue;
                double p = exp(s[j] - L);
                for (int c = 0; c < e; ++c) oi[c] += p * vb[c * si + j];
            }
            for (int c = 0; c < e; ++c) out[((size_t)b * e + c) * so + i] = oi[c];
        }
        free(s); free(oi);
    }
    ctx_free(&C);
    return 0;
}

/* Backward of L = sum(dout*out) w.r.t. q, k, v (omega carries no gradient).
 *   p_ij = exp(s_ij - lse_i),  D_i = dout_i . out_i,  dS_ij = p_ij (dout_i . v_j - D_i)
 *   dq_i = scale sum_j dS_ij k_j ;  dk_j = scale sum_i dS_ij q_i ;  dv_j = sum_i p_ij dout_i
 * dk, dv are evaluated as written: a sum over every output point i whose
 * disk contains j. */
int s2o_nattn_bwd(int grid_type, int nlat_in, int nlon_in, int nlat_out, int nlon_out, double theta,
                  int brute, int nbh, int d, int e, double scale,
                  const double *q, const double *k, const double *v, const double *dout,
                  double *dq, double *dk, double *dv)
{
    s2o_ctx C;
    int rc = ctx_init(&C, grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta, brute);
    if (rc) { ctx_free(&C); return rc; }
    size_t so = (size_t)nlat_out * nlon_out, si = (size_t)nlat_in * nlon_in;
    long total_o = (long)nbh * (long)so, total_i = (long)nbh * (long)si;
    double *lse = malloc(sizeof(double) * (size_t)total_o);
    double *D = malloc(sizeof(double) * (size_t)total_o);
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * si);
        double *oi = malloc(sizeof(double) * e);
        /* phase 1: per output point: lse_i, out_i, D_i, dq_i */
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < total_o; ++t) {
            int b = (int)(t / (long)so);
            int i = (int)(t % (long)so);
            int h = i / nlon_out, w = i % nlon_out;
            const double *qb = q + (size_t)b * d * so, *kb = k + (size_t)b * d * si, *vb = v + (size_t)b * e * si;
            const double *gb = dout + (size_t)b * e * so;
            double m = point_logits(&C, d, scale, qb, kb, h, w, s);
            double Z = 0.0;
            for (size_t j = 0; j < si; ++j)
                if (s[j] != -INFINITY) Z += exp(s[j] - m);
            double L = m + log(Z);
            for (int c = 0; c < e; ++c) oi[c] = 0.0;
            for (size_t j = 0; j < si; ++j) {
                if (s[j] == -INFINITY) continue;
                double p = exp(s[j] - L);
                for (int c = 0; c < e; ++c) oi[c] += p * vb[c * si + j];
            }
            double Di = 0.0;
            for (int c = 0; c < e; ++c) Di += gb[c * so + i] * oi[c];
            lse[t] = L; D[t] = Di;
            for (int l = 0; l < d; ++l) dq[((size_t)b * d + l) * so + i] = 0.0;
            for (size_t j = 0; j < si; ++j) {
                if (s[j] == -INFINITY) continue;
                double p = exp(s[j] - L), gv = 0.0;
                for (int c = 0; c < e; ++c) gv += gb[c * so + i] * vb[c * si + j];
                double dS = p * (gv - Di);
                for (int l = 0; l < d; ++l) dq[((size_t)b * d + l) * so + i] += scale * dS * kb[l * si + j];
            }
        }
        /* phase 2: per input point: dk_j, dv_j gathered over all outputs containing j */
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < total_i; ++t) {
            int b = (int)(t / (long)si);
            size_t j = (size_t)(t % (long)si);
            int hp = (int)(j / nlon_in), win = (int)(j % nlon_in);
            const double *qb = q + (size_t)b * d * so, *kb = k + (size_t)b * d * si, *vb = v + (size_t)b * e * si;
            const double *gb = dout + (size_t)b * e * so;
            for (int l = 0; l < d; ++l) dk[((size_t)b * d + l) * si + j] = 0.0;
            for (int c = 0; c < e; ++c) dv[((size_t)b * e + c) * si + j] = 0.0;
            for (int h = 0; h < nlat_out; ++h)
                for (int w = 0; w < nlon_out; ++w) {
                    if (!member(&C, h, w, hp, win)) continue;
                    size_t i = (size_t)h * nlon_out + w;
                    double dot = 0.0, gv = 0.0;
                    for (int l = 0; l < d; ++l) dot += qb[l * so + i] * kb[l * si + j];
                    for (int c = 0; c < e; ++c) gv += gb[c * so + i] * vb[c * si + j];
                    double p = exp(dot * scale + C.logw[hp] - lse[(size_t)b * so + i]);
                    double dS = p * (gv - D[(size_t)b * so + i]);
                    for (int l = 0; l < d; ++l) dk[((size_t)b * d + l) * si + j] += scale * dS * qb[l * so + i];
                    for (int c = 0; c < e; ++c) dv[((size_t)b * e + c) * si + j] += p * gb[c * so + i];
                }
        }
        free(s); free(oi);
    }
    free(lse); free(D);
    ctx_free(&C);
    return 0;
}

/* First-order rounding sensitivity of the forward and backward results (a
 * yardstick for the float32 parity tolerance, not part of the method).
 *
 * Every result of App. B.1 / B.4 is a sum of products of the inputs.  If each
 * elementary product is perturbed by a relative amount of at most u, the
 * result moves by at most u times the sum of the absolute values of those
 * products, each counted once per factor that carries the perturbation:
 *   a_ij    = |scale| sum_l |q_il| |k_jl|                (terms of the logit)
 *   c_lse_i = 1 + sum_j p_ij a_ij                        (d lse = sum_j p_ij d s_ij, + the log)
 *   w_ij    = 1 + a_ij + c_lse_i                         (relative budget of p_ij = exp(s_ij - lse_i))
 *   c_out_ic = sum_j p_ij |v_jc| w_ij
 *   G_ij    = sum_c |dout_ic| |v_jc|,   Dabs_i = sum_c |dout_ic| c_out_ic   (D_i = dout_i . out_i)
 *   t_ij    = |dout_i . v_j - D_i| w_ij + G_ij + Dabs_i  (budget of dS_ij / p_ij)
 *   c_dq_il = |scale| sum_{j in N(i)} p_ij t_ij |k_jl|
 *   c_dk_jl = |scale| sum_{i: j in N(i)} p_ij t_ij |q_il|
 *   c_dv_jc = sum_{i: j in N(i)} p_ij w_ij |dout_ic|
 * With all inputs positive, scale > 0 and w, t replaced by 1 these sums are
 * the results themselves (c_out = out, c_dv = dv); the tests pin the full
 * expressions against a dense evaluation. */
int s2o_nattn_cond(int grid_type, int nlat_in, int nlon_in, int nlat_out, int nlon_out, double theta,
                   int brute, int nbh, int d, int e, double scale,
                   const double *q, const double *k, const double *v, const double *dout,
                   double *c_out, double *c_lse, double *c_dq, double *c_dk, double *c_dv)
{
    s2o_ctx C;
    int rc = ctx_init(&C, grid_type, nlat_in, nlon_in, nlat_out, nlon_out, theta, brute);
    if (rc) { ctx_free(&C); return rc; }
    size_t so = (size_t)nlat_out * nlon_out, si = (size_t)nlat_in * nlon_in;
    long total_o = (long)nbh * (long)so, total_i = (long)nbh * (long)si;
    double *lse = malloc(sizeof(double) * (size_t)total_o);
    double *D = malloc(sizeof(double) * (size_t)total_o);
    double *Dabs = malloc(sizeof(double) * (size_t)total_o);
    double ascale = fabs(scale);
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * si);
        double *oi = malloc(sizeof(double) * e);
        double *ci = malloc(sizeof(double) * e);
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < total_o; ++t) {
            int b = (int)(t / (long)so);
            int i = (int)(t % (long)so);
            int h = i / nlon_out, w = i % nlon_out;
            const double *qb = q + (size_t)b * d * so, *kb = k + (size_t)b * d * si, *vb = v + (size_t)b * e * si;
            const double *gb = dout + (size_t)b * e * so;
            double m = point_logits(&C, d, scale, qb, kb, h, w, s);
            double Z = 0.0;
            for (size_t j = 0; j < si; ++j)
                if (s[j] != -INFINITY) Z += exp(s[j] - m);
            double L = m + log(Z);
            /* c_lse, then out and c_out */
            double cl = 1.0;
            for (size_t j = 0; j < si; ++j) {
                if (s[j] == -INFINITY) continue;
                double a = 0.0;
                for (int l = 0; l < d; ++l) a += fabs(qb[l * so + i]) * fabs(kb[l * si + j]);
                cl += exp(s[j] - L) * ascale * a;
            }
            for (int c = 0; c < e; ++c) { oi[c] = 0.0; ci[c] = 0.0; }
            for (size_t j = 0; j < si; ++j) {
                if (s[j] == -INFINITY) continue;
                double a = 0.0;
                for (int l = 0; l < d; ++l) a += fabs(qb[l * so + i]) * fabs(kb[l * si + j]);
                double p = exp(s[j] - L), wij = 1.0 + ascale * a + cl;
                for (int c = 0; c < e; ++c) {
                    oi[c] += p * vb[c * si + j];
                    ci[c] += p * fabs(vb[c * si + j]) * wij;
                }
            }
            double Di = 0.0, Da = 0.0;
            for (int c = 0; c < e; ++c) {
                Di += gb[c * so + i] * oi[c];
                Da += fabs(gb[c * so + i]) * ci[c];
                c_out[((size_t)b * e + c) * so + i] = ci[c];
            }
            lse[t] = L; D[t] = Di; Dabs[t] = Da;
            c_lse[t] = cl;
            for (int l = 0; l < d; ++l) c_dq[((size_t)b * d + l) * so + i] = 0.0;
            for (size_t j = 0; j < si; ++j) {
                if (s[j] == -INFINITY) continue;
                double a = 0.0, gv = 0.0, G = 0.0;
                for (int l = 0; l < d; ++l) a += fabs(qb[l * so + i]) * fabs(kb[l * si + j]);
                for (int c = 0; c < e; ++c) {
                    gv += gb[c * so + i] * vb[c * si + j];
                    G += fabs(gb[c * so + i]) * fabs(vb[c * si + j]);
                }
                double p = exp(s[j] - L), wij = 1.0 + ascale * a + cl;
                double tij = fabs(gv - Di) * wij + G + Da;
                for (int l = 0; l < d; ++l) c_dq[((size_t)b * d + l) * so + i] += ascale * p * tij * fabs(kb[l * si + j]);
            }
        }
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < total_i; ++t) {
            int b = (int)(t / (long)si);
            size_t j = (size_t)(t % (long)si);
            int hp = (int)(j / nlon_in), win = (int)(j % nlon_in);
            const double *qb = q + (size_t)b * d * so, *kb = k + (size_t)b * d * si, *vb = v + (size_t)b * e * si;
            const double *gb = dout + (size_t)b * e * so;
            for (int l = 0; l < d; ++l) c_dk[((size_t)b * d + l) * si + j] = 0.0;
            for (int c = 0; c < e; ++c) c_dv[((size_t)b * e + c) * si + j] = 0.0;
            for (int h = 0; h < nlat_out; ++h)
                for (int w = 0; w < nlon_out; ++w) {
                    if (!member(&C, h, w, hp, win)) continue;
                    size_t i = (size_t)h * nlon_out + w;
                    double dot = 0.0, a = 0.0, gv = 0.0, G = 0.0;
                    for (int l = 0; l < d; ++l) {
                        dot += qb[l * so + i] * kb[l * si + j];
                        a += fabs(qb[l * so + i]) * fabs(kb[l * si + j]);
                    }
                    for (int c = 0; c < e; ++c) {
                        gv += gb[c * so + i] * vb[c * si + j];
                        G += fabs(gb[c * so + i]) * fabs(vb[c * si + j]);
                    }
                    size_t ti = (size_t)b * so + i;
                    double p = exp(dot * scale + C.logw[hp] - lse[ti]);
                    double wij = 1.0 + ascale * a + c_lse[ti];
                    double tij = fabs(gv - D[ti]) * wij + G + Dabs[ti];
                    for (int l = 0; l < d; ++l) c_dk[((size_t)b * d + l) * si + j] += ascale * p * tij * fabs(qb[l * so + i]);
                    for (int c = 0; c < e; ++c) c_dv[((size_t)b * e + c) * si + j] += p * wij * fabs(gb[c * so + i]);
                }
        }
        free(s); free(oi); free(ci);
    }
    free(lse); free(D); free(Dabs);
    ctx_free(&C);
    return 0;
}

/* ------------------------------------------------------ global attention -- */

static double *global_logw(int grid_type, int nlat, int nlon)
{
    double *c = malloc(sizeof(double) * nlat), *w = malloc(sizeof(double) * nlat);
    if (s2o_grid(grid_type, nlat, c, w)) { free(c); free(w); return NULL; }
    for (int h = 0; h < nlat; ++h) w[h] = log(w[h] * 2.0 * S2O_PI / (double)nlon);
    free(c);
    return w;
}

/* Global forward: softmax over all N = nlat*nlon tokens of q_i.k_j*scale + ln omega_j. */
int s2o_global_fwd(int grid_type, int nlat, int nlon, int nbh, int d, int e, double scale,
                   const double *q, const double *k, const double *v, double *out, double *lse)
{
    double *logw = global_logw(grid_type, nlat, nlon);
    if (!logw) return -1;
    long N = (long)nlat * nlon, total = (long)nbh * N;
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < total; ++t) {
            long b = t / N, i = t % N;
            const double *qi = q + ((size_t)b * N + i) * d;
            const double *kb = k + (size_t)b * N * d, *vb = v + (size_t)b * N * e;
            double m = -INFINITY;
            for (long j = 0; j < N; ++j) {
                double dot = 0.0;
                for (int l = 0; l < d; ++l) dot += qi[l] * kb[j * d + l];
                s[j] = dot * scale + logw[j / nlon];
                if (s[j] > m) m = s[j];
            }
            double Z = 0.0;
            for (long j = 0; j < N; ++j) Z += exp(s[j] - m);
            double L = m + log(Z);
            lse[t] = L;
            double *oi = out + ((size_t)b * N + i) * e;
            for (int c = 0; c < e; ++c) oi[c] = 0.0;
            for (long j = 0; j < N; ++j) {
                double p = exp(s[j] - L);
                for (int c = 0; c < e; ++c) oi[c] += p * vb[j * e + c];
            }
        }
        free(s);
    }
    free(logw);
    return 0;
}

/* Global backward, same formulas as the neighborhood backward with every
 * input point a member of every disk. */
int s2o_global_bwd(int grid_type, int nlat, int nlon, int nbh, int d, int e, double scale,
                   const double *q, const double *k, const double *v, const double *dout,
                   double *dq, double *dk, double *dv)
{
    double *logw = global_logw(grid_type, nlat, nlon);
    if (!logw) return -1;
    long N = (long)nlat * nlon, total = (long)nbh * N;
    double *lse = malloc(sizeof(double) * (size_t)total), *D = malloc(sizeof(double) * (size_t)total);
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * (size_t)N);
        double *oi = malloc(sizeof(double) * e);
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < total; ++t) {
            long b = t / N, i = t % N;
            const double *qi = q + ((size_t)b * N + i) * d, *gi = dout + ((size_t)b * N + i) * e;
            const double *kb = k + (size_t)b * N * d, *vb = v + (size_t)b * N * e;
            double m = -INFINITY;
            for (long j = 0; j < N; ++j) {
                double dot = 0.0;
                for (int l = 0; l < d; ++l) dot += qi[l] * kb[j * d + l];
                s[j] = dot * scale + logw[j / nlon];
                if (s[j] > m) m = s[j];
            }
            double Z = 0.0;
            for (long j = 0; j < N; ++j) Z += exp(s[j] - m);
            double L = m + log(Z);
            for (int c = 0; c < e; ++c) oi[c] = 0.0;
            for (long j = 0; j < N; ++j) {
                double p = exp(s[j] - L);
                for (int c = 0; c < e; ++c) oi[c] += p * vb[j * e + c];
            }
            double Di = 0.0;
            for (int c = 0; c < e; ++c) Di += gi[c] * oi[c];
            lse[t] = L; D[t] = Di;
            double *dqi = dq + ((size_t)b * N + i) * d;
            for (int l = 0; l < d; ++l) dqi[l] = 0.0;
            for (long j = 0; j < N; ++j) {
                double p = exp(s[j] - L), gv = 0.0;
                for (int c = 0; c < e; ++c) gv += gi[c] * vb[j * e + c];
                double dS = p * (gv - Di);
                for (int l = 0; l < d; ++l) dqi[l] += scale * dS * kb[j * d + l];
            }
        }
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < total; ++t) {
            long b = t / N, j = t % N;
            const double *kj = k + ((size_t)b * N + j) * d, *vj = v + ((size_t)b * N + j) * e;
            const double *qb = q + (size_t)b * N * d, *gb = dout + (size_t)b * N * e;
            double *dkj = dk + ((size_t)b * N + j) * d, *dvj = dv + ((size_t)b * N + j) * e;
            for (int l = 0; l < d; ++l) dkj[l] = 0.0;
            for (int c = 0; c < e; ++c) dvj[c] = 0.0;
            double lw = logw[j / nlon];
            for (long i = 0; i < N; ++i) {
                double dot = 0.0, gv = 0.0;
                for (int l = 0; l < d; ++l) dot += qb[i * d + l] * kj[l];
                for (int c = 0; c < e; ++c) gv += gb[i * e + c] * vj[c];
                double p = exp(dot * scale + lw - lse[b * N + i]);
                double dS = p * (gv - D[b * N + i]);
                for (int l = 0; l < d; ++l) dkj[l] += scale * dS * qb[i * d + l];
                for (int c = 0; c < e; ++c) dvj[c] += p * gb[i * e + c];
            }
        }
        free(s); free(oi);
    }
    free(lse); free(D);
    free(logw);
    return 0;
}
