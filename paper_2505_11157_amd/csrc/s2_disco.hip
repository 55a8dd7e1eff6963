// Discrete-continuous (DISCO) convolution on the sphere (App. B.3, first equation), float32, on the same compact
// form of the indicator as the attention kernels: for output latitude h the disk meets the input latitudes of its
// band in arcs of consecutive longitude offsets, and the filter basis is tabulated per (h, band row, offset):
//     z[b, c, k, h, w] = sum_{h', w'} psi_k[h, h', w'] x[b, c, h', (w' + w pscale) mod nlon_in]
//     y[b, o, h, w]    = sum_{c, k} weight[o, c, k] z[b, c, k, h, w] + bias[o]
// psi_k = hat_k(r) * omega[h'] with K piecewise-linear hats of the geodesic distance r (hat_k(r) = max(0,
// 1 - |r K / theta_cutoff - k|): isotropic filters that vanish on the rim of the disk); the paper leaves the basis
// open.  Equal longitude counts (at least 64, a multiple of 16; batch * channels a multiple of 16) run the contraction
// with psi on the fp32 matrix cores (disco_z_band, disco_dx_band below); other shapes use a gather per point (lanes on
// consecutive longitudes, the basis values of a (latitude, offset) uniform over a wavefront).  The channel mixing is a
// channel matrix on the fp32 matrix cores.  Backward: dx goes through the transposed neighborhood (no atomics), dweight
// is the split-K weight-gradient product summed in a fixed order.
#include <cmath>
#include <new>

#include "s2_nattn_kernels.h"

struct s2_disco {
    const s2_grid_t *g;
    int K;
    float *dev_psi = nullptr;     // [entry][KP], KP = K rounded up to a multiple of 4; entry = poff[h * band_max + b] + offset
    int *dev_poff = nullptr;      // [nlat_out * band_max]
    // matrix-core path (equal longitude counts): the same values with 16 floats per offset and every arc padded with
    // zero entries to a multiple of four offsets; row pitch (floats) of the staged input rows
    float *dev_psi16 = nullptr;
    int *dev_poff16 = nullptr;
    int pitch16 = 0;
    int dx_lds_bytes = 0;         // dynamic LDS of the matrix-core dx kernel (0: not available)
};

namespace {

constexpr int kMaxBasis = 16;     // a 4 x 4 planar kernel's worth of basis functions (App. C)

__device__ __forceinline__ int wrapn(int x, int n)
{
    x = x < 0 ? x + n : x;
    return x >= n ? x - n : x;
}

// z[bc][k][h][w]: one lane per output point, block -> (64 longitudes, latitude, bc).  KP: the basis count rounded up to
// a multiple of four; the basis table holds KP values per arc offset (zeros behind the K-th).
template <int KP>
__global__ void __launch_bounds__(64)
disco_z_fwd(S2DeviceTables t, const float *__restrict__ psi, const int *__restrict__ poff, int K,
            const float *__restrict__ x, float *__restrict__ z)
{
    const int w = blockIdx.x * 64 + threadIdx.x, h = blockIdx.y, bc = blockIdx.z;
    if (w >= t.nlon_out) return;
    const size_t si = size_t(t.nlat_in) * t.nlon_in, so = size_t(t.nlat_out) * t.nlon_out;
    float acc[KP];
#pragma unroll
    for (int k = 0; k < KP; ++k) acc[k] = 0.f;
    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    for (int b = 0; b < nb; ++b) {
        const int c = t.cnt[h * t.band_max + b];
        const int first = w * t.pscale + (c == t.nlon_in ? 0 : -((c - 1) >> 1));
        const float *xr = x + size_t(bc) * si + size_t(hp0 + b) * t.nlon_in;
        const float *pr = psi + size_t(poff[h * t.band_max + b]) * KP;
        int col = wrapn(first, t.nlon_in);
        for (int tt = 0; tt < c; ++tt) {
            const float xv = xr[col];
#pragma unroll
            for (int k = 0; k < KP; ++k) acc[k] = fmaf(pr[tt * KP + k], xv, acc[k]);
            col = col + 1 == t.nlon_in ? 0 : col + 1;
        }
    }
#pragma unroll
    for (int k = 0; k < KP; ++k)
        if (k < K) z[(size_t(bc) * K + k) * so + size_t(h) * t.nlon_out + w] = acc[k];
}

// dz[bc][k][n] -> dzt[bc][n][KP] (zeros behind the K-th value): the gather of disco_dx then reads the K values of an
// output point as KP/4 16-byte loads instead of K loads from K planes
template <int KP>
__global__ void __launch_bounds__(256)
disco_dz_transpose(int K, size_t so, const float *__restrict__ dz, float *__restrict__ dzt)
{
    const size_t n = size_t(blockIdx.x) * 256 + threadIdx.x;
    const int bc = blockIdx.y;
    if (n >= so) return;
    float v[KP];
#pragma unroll
    for (int k = 0; k < KP; ++k) v[k] = k < K ? dz[(size_t(bc) * K + k) * so + n] : 0.f;
    float4 *o = reinterpret_cast<float4 *>(dzt + (size_t(bc) * so + n) * KP);
#pragma unroll
    for (int q = 0; q < KP / 4; ++q) o[q] = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}

// dx[bc][h'][w_in] = sum over the output points (h, w) whose disk holds the input point, and over k, of
// psi_k[h, h', w_in - w pscale] dz[bc][k][h][w]: one lane per input point; dzt is dz with the basis index innermost
template <int KP, bool PS1>      // PS1: equal longitude counts (no division in the walk over the arc)
__global__ void __launch_bounds__(64)
disco_dx(S2DeviceTables t, const float *__restrict__ psi, const int *__restrict__ poff,
         const float *__restrict__ dzt, float *__restrict__ dx)
{
    const int win = blockIdx.x * 64 + threadIdx.x, hp = blockIdx.y, bc = blockIdx.z;
    if (win >= t.nlon_in) return;
    const size_t si = size_t(t.nlat_in) * t.nlon_in, so = size_t(t.nlat_out) * t.nlon_out;
    float acc = 0.f;
    const int ps = PS1 ? 1 : t.pscale;
    const int nb = t.omega_rel[hp] > 0.f ? t.tband_n[hp] : 0;       // a latitude of weight zero receives nothing
    const int h0 = t.tband_lo[hp];
    for (int b = 0; b < nb; ++b) {
        const int h = h0 + b;
        const int bf = hp - t.band_lo[h];                            // row of h' in the band of h
        const int c = t.cnt[h * t.band_max + bf];
        const int lo = c == t.nlon_in ? 0 : -((c - 1) >> 1);
        const float *pr = psi + size_t(poff[h * t.band_max + bf]) * KP;
        const float *dr = dzt + (size_t(bc) * so + size_t(h) * t.nlon_out) * KP;
        // offset tt of the arc of output w is input column w ps + lo + tt: w ps = win - lo - tt (mod nlon_in)
        int xw = wrapn(win - lo, t.nlon_in);
        for (int tt = 0; tt < c; ++tt) {
            if (PS1 || xw % ps == 0) {
                const int w = PS1 ? xw : xw / ps;
                const float4 *dp = reinterpret_cast<const float4 *>(dr + size_t(w) * KP);
#pragma unroll
                for (int q = 0; q < KP / 4; ++q) {
                    const float4 v = dp[q];
                    acc = fmaf(pr[tt * KP + 4 * q + 0], v.x, acc);
                    acc = fmaf(pr[tt * KP + 4 * q + 1], v.y, acc);
                    acc = fmaf(pr[tt * KP + 4 * q + 2], v.z, acc);
                    acc = fmaf(pr[tt * KP + 4 * q + 3], v.w, acc);
                }
            }
            xw = xw == 0 ? t.nlon_in - 1 : xw - 1;
        }
    }
    dx[size_t(bc) * si + size_t(hp) * t.nlon_in + win] = acc;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// z on the fp32 matrix cores (equal longitude counts).  For ONE output point the contraction over the offsets of an
// arc is a small dense product: Z[k][c] += sum_d psi[d][k] x[c][w + lo + d] -- basis index k as the row dimension
// of v_mfma_f32_16x16x4_f32 (16 rows: the basis count padded), 16 channels as its columns, four offsets per
// instruction.  No mask is needed (the arcs are exact; only their length is padded to a multiple of four, with zero
// basis values) and A = psi[d0 + g][k = lane & 15] is one coalesced 256-byte read shared by every output point of the
// latitude.  A wavefront owns 16 consecutive output longitudes (16 accumulators), a workgroup 64 longitudes x 16
// channels of one latitude; each input row of the band is copied to LDS once (channel-major, pitch 4 mod 64 words:
// B = x[c = lane & 15][w + lo + d0 + g] is conflict-free).  Lane (c, g) ends with z[k = 4 g + 0..3][c] of its 16
// points: 64 contiguous bytes per (k, c).
__global__ void __launch_bounds__(256)
disco_z_band(S2DeviceTables t, const float *__restrict__ psi16, const int *__restrict__ poff16, int K, int pitch,
             const float *__restrict__ x, float *__restrict__ z)
{
    extern __shared__ __attribute__((aligned(16))) float xs[];       // [16 channels][pitch]
    const int nlon = t.nlon_in;
    const int h = blockIdx.y, bc0 = blockIdx.z * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int w0g = blockIdx.x * 64, w0 = w0g + 16 * wave;
    const bool active = w0 < nlon;
    const size_t si = size_t(t.nlat_in) * nlon, so = size_t(t.nlat_out) * nlon;
    f32x4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    const int sc = tid >> 4, sp = tid & 15;         // staging: channel, first 16-byte piece
    for (int b = 0; b < nb; ++b) {
        const int cnt = t.cnt[h * t.band_max + b];
        const int lo = cnt == nlon ? 0 : -((cnt - 1) >> 1), npad = (cnt + 3) & ~3;
        const int Xs = (w0g + lo + nlon) & ~3;                                // first staged column (unwrapped)
        const int np4 = (w0g + 63 + lo + nlon + npad - Xs + 3) >> 2;           // 16-byte pieces per channel row
        __syncthreads();                            // the previous row has been consumed
        const float *xr = x + size_t(bc0 + sc) * si + size_t(hp0 + b) * nlon;
        for (int pc = sp; pc < np4; pc += 16) {
            int col = Xs + 4 * pc;
            col = col >= 2 * nlon ? col - 2 * nlon : col;
            col = col >= nlon ? col - nlon : col;
            col = col >= nlon ? col - nlon : col;
            *reinterpret_cast<f32x4 *>(xs + sc * pitch + 4 * pc) = *reinterpret_cast<const f32x4 *>(xr + col);
        }
        __syncthreads();
        if (!active) continue;
        const float *pa = psi16 + size_t(poff16[h * t.band_max + b]) * 16 + lane;
        const float *xb = xs + n * pitch + (w0 + lo + nlon - Xs) + g;
        float a = pa[0];
        for (int d0 = 0; d0 < npad; d0 += 4) {
            const float an = d0 + 4 < npad ? pa[(d0 + 4) * 16] : 0.f;          // next step's basis values
#pragma unroll
            for (int wi = 0; wi < 16; ++wi)
                acc[wi] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, xb[d0 + wi], acc[wi], 0, 0, 0);
            a = an;
        }
    }
    if (!active) return;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int k = 4 * g + rr;
        if (k < K) {
            float *zo = z + (size_t(bc0 + n) * K + k) * so + size_t(h) * nlon + w0;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<f32x4 *>(zo + 4 * q) =
                    f32x4{acc[4 * q][rr], acc[4 * q + 1][rr], acc[4 * q + 2][rr], acc[4 * q + 3][rr]};
        }
    }
}

// dx on the fp32 matrix cores (equal longitude counts, at most 512 longitudes).  For 16 consecutive input
// longitudes x of latitude h' and 16 channels, one output latitude h of the transposed band contributes
//     dx[c][x] += sum_{w, k} dz[c][h][w][k] psi[h, h'][x - w - lo][k],
// a product of the 16 x (w, k) slab of dz (basis index innermost: A = dzt[c = lane & 15][w][4 q + g], one LDS word per
// lane) with the banded matrix psi[x - w - lo][k] (B, taken from a copy of the arc's basis values in LDS that carries
// 16 zero entries on either side, so that offsets outside the arc need no mask; entry stride 20 words: the 16 x 4
// words a wavefront reads fall into 64 different banks).  dz is walked in chunks of 32 output longitudes; a
// wavefront skips the output longitudes whose arcs miss its 16 inputs.  No atomics: every dx element is owned by one
// lane.
template <int KP>
__global__ void __launch_bounds__(256)
disco_dx_band(S2DeviceTables t, const float *__restrict__ psi, const int *__restrict__ poff,
              const float *__restrict__ dzt, float *__restrict__ dx)
{
    constexpr int kChunk = 32, kPitchG = kChunk * KP + 4, kStride = 20, kMargin = 16, kQ = KP / 4;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *G = lds, *P = lds + 16 * kPitchG;            // dz chunk [16 channels][32 w * KP]; basis values of the arc
    const int nlon = t.nlon_in;
    const int hp = blockIdx.y, bc0 = blockIdx.z * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int x0g = blockIdx.x * 64, x0 = x0g + 16 * wave;
    const bool active = x0 < nlon;
    const size_t si = size_t(t.nlat_in) * nlon, so = size_t(t.nlat_out) * nlon;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const int nb = t.omega_rel[hp] > 0.f ? t.tband_n[hp] : 0;       // a latitude of weight zero receives nothing
    const int h0 = t.tband_lo[hp];
    const int sc = tid >> 4, sp = tid & 15;
    for (int b = 0; b < nb; ++b) {
        const int h = h0 + b;
        const int bf = hp - t.band_lo[h];
        const int cnt = t.cnt[h * t.band_max + bf];
        const int lo = cnt == nlon ? 0 : -((cnt - 1) >> 1);
        const float *pr = psi + size_t(poff[h * t.band_max + bf]) * KP;
        __syncthreads();                               // the previous row's basis values are no longer read
        for (int i = tid; i < (cnt + 2 * kMargin) * kStride; i += 256) P[i] = 0.f;
        __syncthreads();
        for (int i = tid; i < cnt * KP; i += 256) P[(i / KP + kMargin) * kStride + i % KP] = pr[i];
        // output longitudes (unwrapped, offset by 2 nlon so that they stay positive) whose arcs meet the workgroup's /
        // the wavefront's inputs: x - w - lo in [0, cnt)
        const int base = 2 * nlon;
        const int wg_lo = base + x0g - lo - cnt + 1, wg_hi = base + x0g + 63 - lo;
        const int wv_lo = base + x0 - lo - cnt + 1, wv_hi = base + x0 + 15 - lo;
        for (int wc = wg_lo; wc <= wg_hi; wc += kChunk) {
            __syncthreads();                           // the previous chunk has been consumed (and P is complete)
            {
                const float *src = dzt + (size_t(bc0 + sc) * so + size_t(h) * nlon) * KP;
#pragma unroll
                for (int j = 0; j < KP / 2; ++j) {
                    const int pc = sp + 16 * j, wo = pc / kQ, part = pc % kQ;
                    int wphys = wc + wo;
                    wphys -= (wphys / nlon) * nlon;
                    *reinterpret_cast<f32x4 *>(G + sc * kPitchG + wo * KP + 4 * part) =
                        *reinterpret_cast<const f32x4 *>(src + size_t(wphys) * KP + 4 * part);
                }
            }
            __syncthreads();
            if (!active) continue;
            const int a = max(wc, wv_lo), e = min(wc + kChunk - 1, wv_hi);
            for (int w = a; w <= e; ++w) {
                const float *ga = G + n * kPitchG + (w - wc) * KP + g;
                const float *pb = P + (base + x0 + n - w - lo + kMargin) * kStride + g;
#pragma unroll
                for (int q = 0; q < kQ; ++q) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ga[4 * q], pb[4 * q], acc, 0, 0, 0);
            }
        }
    }
    if (!active) return;
    // lane (x = n, g) holds channels 4 g + 0..3
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) dx[size_t(bc0 + 4 * g + rr) * si + size_t(hp) * nlon + x0 + n] = acc[rr];
}

int check(const s2_disco_t *dc, int batch, int cin, int cout, const void *ws, size_t ws_bytes)
{
    if (!dc) return s2_fail(S2_ERR_INVALID_ARG, "disco handle is NULL");
    if (batch < 1 || cin < 1 || cout < 1) return s2_fail(S2_ERR_INVALID_ARG, "batch and channel counts must be >= 1");
    const size_t n_out = size_t(dc->g->nlat_out) * dc->g->nlon_out;
    if ((cin * dc->K) % 16 != 0 || cout % 16 != 0 || n_out % 16 != 0)
        return s2_fail(S2_ERR_UNSUPPORTED, "channels_in * nbasis, channels_out and the number of output points must be multiples of 16");
    if (long(batch) * cin > 65535) return s2_fail(S2_ERR_INVALID_ARG, "batch * channels_in too large");
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < s2_disco_workspace_bytes(dc, batch, cin, cout))
        return s2_fail(S2_ERR_WORKSPACE, "workspace missing, not 256-byte aligned or smaller than s2_disco_workspace_bytes()");
    return S2_OK;
}

inline int padded(int K) { return (K + 3) / 4 * 4; }

template <class F>
void by_basis(int K, F f)       // f(KP), KP = the basis count rounded up to a multiple of four
{
    if (K <= 4) f(std::integral_constant<int, 4>());
    else if (K <= 8) f(std::integral_constant<int, 8>());
    else if (K <= 12) f(std::integral_constant<int, 12>());
    else f(std::integral_constant<int, 16>());
}

int raise_dx_lds(int K, int bytes)
{
    int rc = 0;
    by_basis(K, [&](auto KP) {
        rc = hipFuncSetAttribute(reinterpret_cast<const void *>(disco_dx_band<decltype(KP)::value>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess;
    });
    return rc;
}

}  // namespace

extern "C" int s2_disco_init(const s2_grid_t *g, int nbasis, s2_disco_t **out)
{
    if (!out) return s2_fail(S2_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!g) return s2_fail(S2_ERR_INVALID_ARG, "grid is NULL");
    if (nbasis < 1 || nbasis > kMaxBasis) return s2_fail(S2_ERR_INVALID_ARG, "nbasis must lie in [1, 16]");
    if (g->upscale > 1) return s2_fail(S2_ERR_UNSUPPORTED, "the DISCO convolution covers equal grids and downsampling");
    s2_disco *dc = new (std::nothrow) s2_disco();
    if (!dc) return s2_fail(S2_ERR_ALLOC, "out of host memory");
    dc->g = g;
    dc->K = nbasis;
    // basis values along the arcs of the kernels' tables (zero-weight latitudes are not in them)
    const double kPi = 3.141592653589793238462643383279502884, dr = g->theta / nbasis;
    const int KP = padded(nbasis);      // values per arc offset in the table (zeros behind the last basis function)
    std::vector<int> poff(size_t(g->nlat_out) * g->band_max, 0);
    std::vector<float> psi;
    for (int h = 0; h < g->nlat_out; ++h)
        for (int b = 0; b < g->band_n[h]; ++b) {
            const int hp = g->band_lo[h] + b, c = g->cnt[size_t(h) * g->band_max + b];
            const int lo = c == g->nlon_in ? 0 : -((c - 1) / 2);
            poff[size_t(h) * g->band_max + b] = int(psi.size() / KP);
            for (int tt = 0; tt < c; ++tt) {
                const int wp = ((lo + tt) % g->nlon_in + g->nlon_in) % g->nlon_in;
                const double r = s2_great_circle(g->colat_out[h], g->colat_in[hp], 2.0 * kPi * wp / g->nlon_in);
                for (int k = 0; k < KP; ++k)
                    psi.push_back(k < nbasis ? float(std::max(0.0, 1.0 - std::fabs(r / dr - k)) * g->omega_in[hp]) : 0.f);
            }
        }
    // matrix-core path: 16 floats per offset, arcs padded to a multiple of four offsets
    std::vector<int> poff16(poff.size(), 0);
    std::vector<float> psi16;
    int maxnpad = 4;
    const bool band_ok = g->pscale == 1 && g->nlon_in == g->nlon_out && g->nlon_in % 16 == 0 && g->nlon_in >= 64 &&
                         g->nlon_in <= 2048;
    if (band_ok)
        for (int h = 0; h < g->nlat_out; ++h)
            for (int b = 0; b < g->band_n[h]; ++b) {
                const int c = g->cnt[size_t(h) * g->band_max + b], npad = (c + 3) / 4 * 4;
                const size_t src = size_t(poff[size_t(h) * g->band_max + b]) * KP;
                poff16[size_t(h) * g->band_max + b] = int(psi16.size() / 16);
                maxnpad = std::max(maxnpad, npad);
                for (int tt = 0; tt < npad; ++tt)
                    for (int k = 0; k < 16; ++k) psi16.push_back(tt < c && k < nbasis ? psi[src + size_t(tt) * KP + k] : 0.f);
            }
    dc->pitch16 = band_ok ? (64 + maxnpad + 8 + 63) / 64 * 64 + 4 : 0;
    if (band_ok && g->nlon_in <= 512) dc->dx_lds_bytes = (16 * (32 * KP + 4) + (maxnpad + 32) * 20) * int(sizeof(float));
    if (g->on_device) {
        if (band_ok) {
            if (hipMalloc(&dc->dev_psi16, std::max<size_t>(psi16.size(), 1) * sizeof(float)) != hipSuccess ||
                hipMalloc(&dc->dev_poff16, poff16.size() * sizeof(int)) != hipSuccess ||
                hipMemcpy(dc->dev_psi16, psi16.data(), psi16.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
                hipMemcpy(dc->dev_poff16, poff16.data(), poff16.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess ||
                hipFuncSetAttribute(reinterpret_cast<const void *>(disco_z_band), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    16 * dc->pitch16 * int(sizeof(float))) != hipSuccess ||
                (dc->dx_lds_bytes && raise_dx_lds(nbasis, dc->dx_lds_bytes))) {
                (void)hipGetLastError();
                s2_disco_destroy(dc);
                return s2_fail(S2_ERR_ALLOC, "set-up of the matrix-core basis tables failed");
            }
        }
        if (hipMalloc(&dc->dev_psi, std::max<size_t>(psi.size(), 1) * sizeof(float)) != hipSuccess ||
            hipMalloc(&dc->dev_poff, poff.size() * sizeof(int)) != hipSuccess) {
            (void)hipGetLastError();
            s2_disco_destroy(dc);
            return s2_fail(S2_ERR_ALLOC, "hipMalloc of the basis tables failed");
        }
        if (hipMemcpy(dc->dev_psi, psi.data(), psi.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
            hipMemcpy(dc->dev_poff, poff.data(), poff.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipGetLastError();
            s2_disco_destroy(dc);
            return s2_fail(S2_ERR_DEVICE, "upload of the basis tables failed");
        }
    }
    *out = dc;
    return S2_OK;
}

extern "C" void s2_disco_destroy(s2_disco_t *dc)
{
    if (!dc) return;
    if (dc->dev_psi) (void)hipFree(dc->dev_psi);
    if (dc->dev_poff) (void)hipFree(dc->dev_poff);
    if (dc->dev_psi16) (void)hipFree(dc->dev_psi16);
    if (dc->dev_poff16) (void)hipFree(dc->dev_poff16);
    delete dc;
}

extern "C" size_t s2_disco_workspace_bytes(const s2_disco_t *dc, int batch, int cin, int cout)
{
    if (!dc || batch < 1 || cin < 1 || cout < 1) return 0;
    const size_t n_out = size_t(dc->g->nlat_out) * dc->g->nlon_out;
    auto up = [](size_t x) { return (x + 63) / 64 * 64; };
    // z, dz: [batch][cin * K][n_out]; dz with the basis index innermost [batch * cin][n_out][KP]; partial sums of the
    // weight gradient
    return (2 * up(size_t(batch) * cin * dc->K * n_out) + up(size_t(batch) * cin * padded(dc->K) * n_out) +
            up(s2_wgrad_part_floats(cout, cin * dc->K))) * sizeof(float);
}

extern "C" int s2_disco_fwd(const s2_disco_t *dc, int batch, int cin, int cout, const float *x, const float *weight,
                            const float *bias, float *y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check(dc, batch, cin, cout, workspace, workspace_bytes);
    if (rc) return rc;
    if (!x || !weight || !y) return s2_fail(S2_ERR_INVALID_ARG, "NULL tensor pointer");
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(weight) | reinterpret_cast<uintptr_t>(y)) % 16 != 0)
        return s2_fail(S2_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    const s2_grid_t *g = dc->g;
    if (!g->on_device) return s2_fail(S2_ERR_DEVICE, "grid handle has no device tables (no HIP device at init)");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    float *z = static_cast<float *>(workspace);
    const int n_out = g->nlat_out * g->nlon_out, K = dc->K;
    {
        S2TraceScope tr("disco_z_fwd", 0.0, st);
        if (dc->dev_psi16 && (batch * cin) % 16 == 0) {
            const dim3 grid((g->nlon_out + 63) / 64, g->nlat_out, batch * cin / 16);
            hipLaunchKernelGGL(disco_z_band, grid, dim3(256), size_t(16) * dc->pitch16 * sizeof(float), st, g->dt,
                               dc->dev_psi16, dc->dev_poff16, K, dc->pitch16, x, z);
        } else {
            const dim3 grid((g->nlon_out + 63) / 64, g->nlat_out, batch * cin);
            by_basis(K, [&](auto KB) {
                hipLaunchKernelGGL((disco_z_fwd<decltype(KB)::value>), grid, dim3(64), 0, st, g->dt, dc->dev_psi, dc->dev_poff, K, x, z);
            });
        }
    }
    S2TraceScope tr("disco_mix", 0.0, st);
    s2_gemm_f32(false, cout, n_out, cin * K, batch, weight, z, bias, nullptr, y, false, st);
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}

extern "C" int s2_disco_bwd(const s2_disco_t *dc, int batch, int cin, int cout, const float *x, const float *weight,
                            const float *dy, float *dx, float *dweight, float *dbias, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    (void)x;       // z = psi * x was kept in the workspace by the forward pass
    int rc = check(dc, batch, cin, cout, workspace, workspace_bytes);
    if (rc) return rc;
    if (!weight || !dy || !dx) return s2_fail(S2_ERR_INVALID_ARG, "NULL tensor pointer");
    if ((reinterpret_cast<uintptr_t>(weight) | reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(dx)) % 16 != 0)
        return s2_fail(S2_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    const s2_grid_t *g = dc->g;
    if (!g->on_device) return s2_fail(S2_ERR_DEVICE, "grid handle has no device tables (no HIP device at init)");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int n_out = g->nlat_out * g->nlon_out, K = dc->K;
    auto up = [](size_t v) { return (v + 63) / 64 * 64; };
    float *z = static_cast<float *>(workspace), *dz = z + up(size_t(batch) * cin * K * n_out);
    float *dzt = dz + up(size_t(batch) * cin * K * n_out), *part = dzt + up(size_t(batch) * cin * padded(K) * n_out);
    {
        S2TraceScope tr("disco_bwd mix", 0.0, st);
        if (dweight) s2_wgrad_f32(cout, cin * K, n_out, batch, dy, z, part, dweight, st);
        if (dbias) s2_channel_sum_f32(batch, cout, n_out, dy, dbias, part, s2_wgrad_part_floats(cout, cin * K), st);
        s2_gemm_f32(true, cin * K, n_out, cout, batch, weight, dy, nullptr, nullptr, dz, false, st);
    }
    S2TraceScope tr("disco_dx", 0.0, st);
    const dim3 grid((g->nlon_in + 63) / 64, g->nlat_in, batch * cin);
    by_basis(K, [&](auto KP) {
        const dim3 tgrid(unsigned((size_t(n_out) + 255) / 256), batch * cin);
        hipLaunchKernelGGL((disco_dz_transpose<decltype(KP)::value>), tgrid, dim3(256), 0, st, K, size_t(n_out), dz, dzt);
        if (dc->dx_lds_bytes && (batch * cin) % 16 == 0) {
            const dim3 bgrid((g->nlon_in + 63) / 64, g->nlat_in, batch * cin / 16);
            hipLaunchKernelGGL((disco_dx_band<decltype(KP)::value>), bgrid, dim3(256), size_t(dc->dx_lds_bytes), st, g->dt,
                               dc->dev_psi, dc->dev_poff, dzt, dx);
        } else if (g->pscale == 1)
            hipLaunchKernelGGL((disco_dx<decltype(KP)::value, true>), grid, dim3(64), 0, st, g->dt, dc->dev_psi, dc->dev_poff, dzt, dx);
        else
            hipLaunchKernelGGL((disco_dx<decltype(KP)::value, false>), grid, dim3(64), 0, st, g->dt, dc->dev_psi, dc->dev_poff, dzt, dx);
    });
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}
