// Generic float32 kernels for spherical neighborhood attention: any head
// dimension up to 128, any grid ratio.  One lane owns one output point (forward,
// dq) or one input point (dk/dv); the geodesic disk is walked as latitude rows
// times a centred longitude arc (App. B.3), operands come straight from
// global memory with lanes on consecutive longitudes.
//
// These are the shape-agnostic path.  The tuned kernels in s2_nattn_tiled.hip
// take over for the head dimensions and grids they are specialised for.
#include <type_traits>

#include "s2_nattn_kernels.h"

namespace {

constexpr int kChunk = 8;   // logits evaluated together before one softmax rescale

// Storage type of the tensors: float, or bf16 (raw 16-bit words; arithmetic is float32 either way, results are
// rounded to nearest even on the store).
typedef unsigned short bf16raw;
__device__ __forceinline__ float ldf(const float *p) { return *p; }
__device__ __forceinline__ float ldf(const bf16raw *p) { return __builtin_bit_cast(float, unsigned(*p) << 16); }
__device__ __forceinline__ void stf(float *p, float x) { *p = x; }
__device__ __forceinline__ void stf(bf16raw *p, float x)
{
    const __bf16 b = (__bf16)x;
    *p = __builtin_bit_cast(bf16raw, b);
}

__device__ __forceinline__ int wrap(int x, int n)
{
    x = x < 0 ? x + n : x;
    return x >= n ? x - n : x;
}

// Arc of output point (h, w) on band row b: first input column (may be negative) and length.  Equal grids and
// downsampling: the centred arc around input column w*pscale.  Upsampling (w = upscale*m + s): the arc of class s
// relative to input column m.
__device__ __forceinline__ void arc_of(const S2DeviceTables &t, int h, int w, int b, int &first, int &c)
{
    if (t.upscale > 1) {
        const int m = w / t.upscale, sc = w - m * t.upscale;
        const int at = (h * t.upscale + sc) * t.band_max + b;
        c = t.ucnt[at];
        first = m + t.ulo[at];
    } else {
        c = t.cnt[h * t.band_max + b];
        first = w * t.pscale + ((c == t.nlon_in) ? 0 : -((c - 1) >> 1));
    }
}

// Forward: App. B.1 (second equation) in the index form of App. B.3, with an
// online softmax in base 2.  q is pre-multiplied by scale*log2(e).  The
// quadrature weight enters as a factor omega[h']/omega_ref on exp2(s - m)
// rather than as an additive log term: the running maximum is taken over the
// bare logits, whose magnitude is a few units, so float32 rounding of the
// logit stays near 1e-7 instead of growing with |log2 omega| ~ 10..20.
template <int DMAX, typename T>
__global__ void __launch_bounds__(64)
nattn_fwd_generic(S2DeviceTables t, int nbh, int first_row, int d, int e, float qscale,
                  const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                  T *__restrict__ out, float *__restrict__ lse)
{
    const int ntile = (t.nlon_out + 63) / 64;
    int id = blockIdx.x;
    const int tile = id % ntile; id /= ntile;
    const int bh = id % nbh;
    const int h = t.row_order[first_row + id / nbh];
    const int w = tile * 64 + threadIdx.x;
    if (w >= t.nlon_out) return;

    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t io = size_t(h) * t.nlon_out + w;
    const T *qb = q + size_t(bh) * d * so + io;
    float qr[DMAX], acc[DMAX];
#pragma unroll
    for (int l = 0; l < DMAX; ++l) {
        qr[l] = l < d ? ldf(qb + l * so) * qscale : 0.f;
        acc[l] = 0.f;
    }
    float m = -INFINITY, lsum = 0.f;
    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    for (int b = 0; b < nb; ++b) {
        const int hp = hp0 + b;
        int first, c;
        arc_of(t, h, w, b, first, c);
        const float wq = t.omega_rel[hp];
        const T *kb = k + size_t(bh) * d * si + size_t(hp) * t.nlon_in;
        const T *vb = v + size_t(bh) * e * si + size_t(hp) * t.nlon_in;
        for (int t0 = 0; t0 < c; t0 += kChunk) {
            float s[kChunk];
            int col[kChunk];
            float mc = -INFINITY;
            // channel by channel: the chunk's eight columns of one channel row are neighbours in memory, so the
            // eight loads of a channel hit the same cache lines (offsets past the arc re-read its last column)
#pragma unroll
            for (int j = 0; j < kChunk; ++j) {
                col[j] = wrap(first + min(t0 + j, c - 1), t.nlon_in);
                s[j] = 0.f;
            }
#pragma unroll
            for (int l = 0; l < DMAX; ++l)
                if (l < d) {
                    const T *kr = kb + l * si;
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) s[j] = fmaf(qr[l], ldf(kr + col[j]), s[j]);
                }
#pragma unroll
            for (int j = 0; j < kChunk; ++j) {
                s[j] = t0 + j < c ? s[j] : -INFINITY;
                mc = fmaxf(mc, s[j]);
            }
            const float m_new = fmaxf(m, mc);
            const float corr = __builtin_amdgcn_exp2f(m - m_new);
            m = m_new;
            lsum *= corr;
            float p[kChunk];
#pragma unroll
            for (int j = 0; j < kChunk; ++j) {
                p[j] = wq * __builtin_amdgcn_exp2f(s[j] - m_new);      // 0 past the arc
                lsum += p[j];
            }
#pragma unroll
            for (int l = 0; l < DMAX; ++l)
                if (l < e) {
                    const T *vr = vb + l * si;
                    float a = acc[l] * corr;
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) a = fmaf(p[j], ldf(vr + col[j]), a);
                    acc[l] = a;
                } else {
                    acc[l] = 0.f;
                }
        }
    }
    const float inv = 1.f / lsum;
    T *ob = out + size_t(bh) * e * so + io;
#pragma unroll
    for (int l = 0; l < DMAX; ++l)
        if (l < e) stf(ob + l * so, acc[l] * inv);
    lse[size_t(bh) * so + io] = (m + log2f(lsum * t.omega_ref)) * 0.6931471805599453f;
}

// Backward, query side (App. B.4): D_i = dout_i.out_i, then
// dq_i = scale * sum_j p_ij (dout_i.v_j - D_i) k_j over the same lists as the
// forward pass, p_ij recomputed from the saved logsumexp.  Also stores D_i.
template <int DMAX, typename T>
__global__ void __launch_bounds__(64)
nattn_bwd_dq_generic(S2DeviceTables t, int nbh, int d, int e, float scale,
                     const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                     const T *__restrict__ o, const float *__restrict__ lse, const T *__restrict__ go,
                     T *__restrict__ dq, float *__restrict__ Dws)
{
    const int ntile = (t.nlon_out + 63) / 64;
    int id = blockIdx.x;
    const int tile = id % ntile; id /= ntile;
    const int bh = id % nbh;
    const int h = t.row_order[id / nbh];
    const int w = tile * 64 + threadIdx.x;
    if (w >= t.nlon_out) return;

    const float qscale = scale * 1.4426950408889634f;
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t io = size_t(h) * t.nlon_out + w;
    float qr[DMAX], gr[DMAX], dqr[DMAX];
    float Di = 0.f;
#pragma unroll
    for (int l = 0; l < DMAX; ++l) {
        qr[l] = l < d ? ldf(q + (size_t(bh) * d + l) * so + io) * qscale : 0.f;
        gr[l] = l < e ? ldf(go + (size_t(bh) * e + l) * so + io) : 0.f;
        if (l < e) Di = fmaf(gr[l], ldf(o + (size_t(bh) * e + l) * so + io), Di);
        dqr[l] = 0.f;
    }
    Dws[size_t(bh) * so + io] = Di;
    // base-2 logsumexp relative to omega_ref: p_ij = omega_rel_j * exp2(s_ij - lse2)
    const float lse2 = (lse[size_t(bh) * so + io] - t.ln_omega_ref) * 1.4426950408889634f;
    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    for (int b = 0; b < nb; ++b) {
        const int hp = hp0 + b;
        int first, c;
        arc_of(t, h, w, b, first, c);
        const float wq = t.omega_rel[hp];
        const T *kb = k + size_t(bh) * d * si + size_t(hp) * t.nlon_in;
        const T *vb = v + size_t(bh) * e * si + size_t(hp) * t.nlon_in;
        for (int t0 = 0; t0 < c; t0 += kChunk) {
            // channel by channel over a chunk of eight columns (see the forward); K rows are read twice, the
            // second time from the cache
            int col[kChunk];
            float dot[kChunk], gv[kChunk];
#pragma unroll
            for (int j = 0; j < kChunk; ++j) {
                col[j] = wrap(first + min(t0 + j, c - 1), t.nlon_in);
                dot[j] = 0.f;
                gv[j] = -Di;
            }
#pragma unroll
            for (int l = 0; l < DMAX; ++l)
                if (l < d) {
                    const T *kr = kb + l * si;
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) dot[j] = fmaf(qr[l], ldf(kr + col[j]), dot[j]);
                }
#pragma unroll
            for (int l = 0; l < DMAX; ++l)
                if (l < e) {
                    const T *vr = vb + l * si;
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) gv[j] = fmaf(gr[l], ldf(vr + col[j]), gv[j]);
                }
#pragma unroll
            for (int j = 0; j < kChunk; ++j)
                dot[j] = t0 + j < c ? wq * __builtin_amdgcn_exp2f(dot[j] - lse2) * gv[j] : 0.f;      // dS
#pragma unroll
            for (int l = 0; l < DMAX; ++l)
                if (l < d) {
                    const T *kr = kb + l * si;
                    float a = dqr[l];
#pragma unroll
                    for (int j = 0; j < kChunk; ++j) a = fmaf(dot[j], ldf(kr + col[j]), a);
                    dqr[l] = a;
                }
        }
    }
#pragma unroll
    for (int l = 0; l < DMAX; ++l)
        if (l < d) stf(dq + (size_t(bh) * d + l) * so + io, dqr[l] * scale);
}

// Backward, key/value side (App. B.4): one lane per INPUT point j gathers
//   dk_j = scale * sum_i dS_ij q_i,   dv_j = sum_i p_ij dout_i
// over the output points whose disk contains j.  By the symmetry of the
// distance these are, on output latitude h, the longitudes w with
// |w*pscale - w_in| <= half-width(h, h') on the circle.
template <int DMAX, typename T>
__global__ void __launch_bounds__(64)
nattn_bwd_dkdv_generic(S2DeviceTables t, int nbh, int d, int e, float scale,
                       const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                       const float *__restrict__ lse, const T *__restrict__ go, const float *__restrict__ Dws,
                       T *__restrict__ dk, T *__restrict__ dv)
{
    const int ntile = (t.nlon_in + 63) / 64;
    int id = blockIdx.x;
    const int tile = id % ntile; id /= ntile;
    const int bh = id % nbh;
    const int hp = t.trow_order[id / nbh];
    const int win = tile * 64 + threadIdx.x;
    if (win >= t.nlon_in) return;

    const float log2e = 1.4426950408889634f;
    const float qscale = scale * log2e;
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t ii = size_t(hp) * t.nlon_in + win;
    float kr[DMAX], vr[DMAX], dkr[DMAX], dvr[DMAX];
#pragma unroll
    for (int l = 0; l < DMAX; ++l) {
        kr[l] = l < d ? ldf(k + (size_t(bh) * d + l) * si + ii) * qscale : 0.f;
        vr[l] = l < e ? ldf(v + (size_t(bh) * e + l) * si + ii) : 0.f;
        dkr[l] = 0.f;
        dvr[l] = 0.f;
    }
    const float wq = t.omega_rel[hp];
    const float lref2 = t.ln_omega_ref * log2e;
    const int ps = t.pscale;
    const int nb = t.tband_n[hp], h0 = t.tband_lo[hp];
    for (int b = 0; b < nb; ++b) {
        const int h = h0 + b;
        const int c = t.tcnt[hp * t.tband_max + b];
        // x = w*pscale runs over the multiples of pscale in [win-hw, win+hw] (whole circle if c == nlon_in)
        // (whole circle: start at the lane's own longitude so that the summation order is shift invariant)
        const int hw = (c == t.nlon_in) ? 0 : (c - 1) >> 1;
        int x = win - hw + t.nlon_in;             // shifted by nlon_in (a multiple of pscale) to stay positive
        const int r = x % ps;
        if (r) x += ps - r;
        const int x_end = (c == t.nlon_in) ? x + t.nlon_in - ps : win + hw + t.nlon_in;
        const T *qb = q + size_t(bh) * d * so + size_t(h) * t.nlon_out;
        const T *gb = go + size_t(bh) * e * so + size_t(h) * t.nlon_out;
        const float *lb = lse + size_t(bh) * so + size_t(h) * t.nlon_out;
        const float *Db = Dws + size_t(bh) * so + size_t(h) * t.nlon_out;
        auto visit = [&](int w) {
            float qr[DMAX], gr[DMAX];
            const float lse2 = fmaf(lb[w], log2e, -lref2);
            float dot = 0.f, gv = -Db[w];
#pragma unroll
            for (int l = 0; l < DMAX; ++l) {
                qr[l] = l < d ? ldf(qb + l * so + w) : 0.f;
                gr[l] = l < e ? ldf(gb + l * so + w) : 0.f;
                dot = fmaf(qr[l], kr[l], dot);
                gv = fmaf(gr[l], vr[l], gv);
            }
            const float p = wq * __builtin_amdgcn_exp2f(dot - lse2);
            const float dS = p * gv;
#pragma unroll
            for (int l = 0; l < DMAX; ++l) {
                dkr[l] = fmaf(dS, qr[l], dkr[l]);
                dvr[l] = fmaf(p, gr[l], dvr[l]);
            }
        };
        if (t.upscale > 1) {
            // upsampling: output longitude w = upscale*m + s holds this input point iff win - m lies in the arc
            // of class s, i.e. m = win - lo - tt for tt = 0 .. c-1
            const int bf = hp - t.band_lo[h];
            for (int sc = 0; sc < t.upscale; ++sc) {
                const int at = (h * t.upscale + sc) * t.band_max + bf;
                const int cu = t.ucnt[at], lo = t.ulo[at];
                for (int tt = 0; tt < cu; ++tt) {
                    int m = (win - lo - tt) % t.nlon_in;
                    m = m < 0 ? m + t.nlon_in : m;
                    visit(m * t.upscale + sc);
                }
            }
        } else {
            for (; x <= x_end; x += ps) {
                int w = x / ps;
                w = w >= t.nlon_out ? w - t.nlon_out : w;
                w = w >= t.nlon_out ? w - t.nlon_out : w;
                visit(w);
            }
        }
    }
#pragma unroll
    for (int l = 0; l < DMAX; ++l) {
        if (l < d) stf(dk + (size_t(bh) * d + l) * si + ii, dkr[l] * scale);
        if (l < e) stf(dv + (size_t(bh) * e + l) * si + ii, dvr[l]);
    }
}

// Input latitudes of weight zero: every p_ij of theirs is zero, so dk = dv = 0 there.  The dk/dv kernels above and
// in the tuned files form 0 * exp2(.) for them, which is not a number once the exponential overflows; this fill,
// enqueued after them, writes the exact result.  x: [rows][nlat_in][nlon_in], one block per (row, 256 columns).
template <typename T>
__global__ void __launch_bounds__(256)
zero_latitude(T *__restrict__ x, int lat, int rows, int nlon_in, size_t si)
{
    const int w = blockIdx.x * 256 + threadIdx.x;
    if (w >= nlon_in) return;
    for (int r = blockIdx.y; r < rows; r += gridDim.y) x[size_t(r) * si + size_t(lat) * nlon_in + w] = T(0);
}

template <int DMAX, typename T>
int launch_fwd(const S2DeviceTables &t, int nbh, int d, int e, float scale, const T *q, const T *k, const T *v, T *out,
               float *lse, hipStream_t st)
{
    const int ntile = (t.nlon_out + 63) / 64;
    const long nblk = long(ntile) * nbh * t.nlat_out;
    S2TraceScope tr("nattn_fwd_generic", nbh * (t.fwd_pairs[0] + t.fwd_pairs[1] + t.fwd_pairs[2] + t.fwd_pairs[3]), st);
    hipLaunchKernelGGL((nattn_fwd_generic<DMAX, T>), dim3((unsigned)nblk), dim3(64), 0, st, t, nbh, 0, d, e,
                       scale * 1.4426950408889634f, q, k, v, out, lse);
    return 0;
}

template <int DMAX, typename T>
int launch_dq(const S2DeviceTables &t, int nbh, int d, int e, float scale, const T *q, const T *k, const T *v,
              const T *o, const float *lse, const T *go, T *dq, float *Dws, hipStream_t st)
{
    const int nto = (t.nlon_out + 63) / 64;
    S2TraceScope tr("nattn_bwd_dq_generic", nbh * (t.fwd_pairs[0] + t.fwd_pairs[1] + t.fwd_pairs[2] + t.fwd_pairs[3]), st);
    hipLaunchKernelGGL((nattn_bwd_dq_generic<DMAX, T>), dim3((unsigned)(long(nto) * nbh * t.nlat_out)), dim3(64), 0, st,
                       t, nbh, d, e, scale, q, k, v, o, lse, go, dq, Dws);
    return 0;
}

template <int DMAX, typename T>
int launch_dkdv(const S2DeviceTables &t, int nbh, int d, int e, float scale, const T *q, const T *k, const T *v,
                const float *lse, const T *go, const float *Dws, T *dk, T *dv, hipStream_t st)
{
    const int nti = (t.nlon_in + 63) / 64;
    S2TraceScope tr("nattn_bwd_dkdv_generic", nbh * (t.fwd_pairs[0] + t.fwd_pairs[1] + t.fwd_pairs[2] + t.fwd_pairs[3]), st);
    hipLaunchKernelGGL((nattn_bwd_dkdv_generic<DMAX, T>), dim3((unsigned)(long(nti) * nbh * t.nlat_in)), dim3(64), 0, st,
                       t, nbh, d, e, scale, q, k, v, lse, go, Dws, dk, dv);
    return 0;
}

// the kernels are instantiated for channel counts up to 8, 16, 32, 64, 128
template <typename F>
int by_width(int d, int e, F f)
{
    const int dm = d > e ? d : e;
    if (dm <= 8) return f(std::integral_constant<int, 8>());
    if (dm <= 16) return f(std::integral_constant<int, 16>());
    if (dm <= 32) return f(std::integral_constant<int, 32>());
    if (dm <= 64) return f(std::integral_constant<int, 64>());
    return f(std::integral_constant<int, 128>());
}

}  // namespace

void s2_nattn_zero_latitude(const S2DeviceTables &t, int lat, int rows, void *x, bool bf16, hipStream_t st)
{
    const dim3 grid((t.nlon_in + 255) / 256, rows < 65535 ? rows : 65535);
    const size_t si = size_t(t.nlat_in) * t.nlon_in;
    if (bf16)
        hipLaunchKernelGGL(zero_latitude<bf16raw>, grid, dim3(256), 0, st, static_cast<bf16raw *>(x), lat, rows, t.nlon_in, si);
    else
        hipLaunchKernelGGL(zero_latitude<float>, grid, dim3(256), 0, st, static_cast<float *>(x), lat, rows, t.nlon_in, si);
}

int s2_nattn_fwd_generic(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q,
                         const float *k, const float *v, float *out, float *lse, hipStream_t st)
{
    return by_width(d, e, [&](auto W) { return launch_fwd<decltype(W)::value, float>(t, nbh, d, e, scale, q, k, v, out, lse, st); });
}

int s2_nattn_bwd_dkdv_generic(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q,
                              const float *k, const float *v, const float *lse, const float *go, const float *Dws,
                              float *dk, float *dv, hipStream_t st)
{
    return by_width(d, e, [&](auto W) {
        return launch_dkdv<decltype(W)::value, float>(t, nbh, d, e, scale, q, k, v, lse, go, Dws, dk, dv, st);
    });
}

int s2_nattn_bwd_generic(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q,
                         const float *k, const float *v, const float *o, const float *lse, const float *go,
                         float *dq, float *dk, float *dv, float *Dws, hipStream_t st)
{
    return by_width(d, e, [&](auto W) {
        constexpr int DM = decltype(W)::value;
        launch_dq<DM, float>(t, nbh, d, e, scale, q, k, v, o, lse, go, dq, Dws, st);
        return launch_dkdv<DM, float>(t, nbh, d, e, scale, q, k, v, lse, go, Dws, dk, dv, st);
    });
}

// bf16 tensors (raw 16-bit words), float32 arithmetic, float32 lse and D
int s2_nattn_fwd_generic_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q, const void *k,
                              const void *v, void *out, float *lse, hipStream_t st)
{
    return by_width(d, e, [&](auto W) {
        return launch_fwd<decltype(W)::value, bf16raw>(t, nbh, d, e, scale, static_cast<const bf16raw *>(q),
                                                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(v),
                                                       static_cast<bf16raw *>(out), lse, st);
    });
}

int s2_nattn_bwd_dq_generic_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q,
                                 const void *k, const void *v, const void *o, const float *lse, const void *go, void *dq,
                                 float *Dws, hipStream_t st)
{
    return by_width(d, e, [&](auto W) {
        return launch_dq<decltype(W)::value, bf16raw>(
            t, nbh, d, e, scale, static_cast<const bf16raw *>(q), static_cast<const bf16raw *>(k),
            static_cast<const bf16raw *>(v), static_cast<const bf16raw *>(o), lse, static_cast<const bf16raw *>(go),
            static_cast<bf16raw *>(dq), Dws, st);
    });
}

int s2_nattn_bwd_dkdv_generic_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q,
                                   const void *k, const void *v, const float *lse, const void *go, const float *Dws,
                                   void *dk, void *dv, hipStream_t st)
{
    return by_width(d, e, [&](auto W) {
        return launch_dkdv<decltype(W)::value, bf16raw>(
            t, nbh, d, e, scale, static_cast<const bf16raw *>(q), static_cast<const bf16raw *>(k),
            static_cast<const bf16raw *>(v), lse, static_cast<const bf16raw *>(go), Dws, static_cast<bf16raw *>(dk),
            static_cast<bf16raw *>(dv), st);
    });
}
