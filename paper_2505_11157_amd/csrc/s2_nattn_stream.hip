// Streaming float32 kernels for the light latitudes of spherical neighborhood
// attention on gfx950 (App. B.1 second equation in the index form of App. B.3;
// gradients of App. B.4).
//
// Away from the poles a disk meets about nine input latitudes on short arcs,
// and neighbouring output latitudes share eight of those nine.  Here a
// workgroup walks DOWN a range of consecutive output latitudes for one strip of
// 128 longitudes and one (batch, head): input latitude r is copied into LDS
// once (all 32 K channels and all 32 V channels of the strip plus a halo of 32
// columns on each side, LDS-direct loads, double buffered) and consumed by
// every wavefront whose current output latitude has r in its band.  Wavefront
// w owns output latitudes first + w, first + w + NW, ...; NW is chosen on the
// host so that the band of latitude h + NW begins no earlier than the last row
// of the band of h, hence a wavefront never carries two softmax states.  Each K
// and V row is fetched from memory once per workgroup instead of once per
// (output latitude, run), which removes the re-reads that bound the one-wave
// kernels.
//
// Inside a row the arc of a latitude pair is cut into runs that start at a
// multiple of four window columns, so a lane's strip of a channel row is a few
// aligned ds_read_b128 and is reused from registers for its four outputs; the
// (at most three) offsets in front of the arc get a logit of -inf.
#include <cstdlib>

#include "s2_nattn_kernels.h"

namespace {

constexpr int kD = 32;          // head dimension (both)
constexpr int kSegS = 128;      // output longitudes per workgroup (forward: per wavefront)
constexpr int kHalo = 32;       // halo columns on each side of the strip: arcs of up to 65 offsets
constexpr int kWin = kSegS + 2 * kHalo;   // 192 window columns = three 64-lane loads per channel row
constexpr int kPitchS = kWin + 8;         // 8 mod 16: rows four apart start 32 banks apart
constexpr int kSlot = 2 * kD * kPitchS;   // floats per ring slot: 32 K rows, then 32 V rows
constexpr int kMaxWaves = 8;
constexpr int kNTS = 8;         // longest run of window offsets handled at once

typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

__device__ __forceinline__ float dpp_swap_pair(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, true));
}

__device__ __forceinline__ int wrap2(int x, int n)
{
    x = x >= n ? x - n : x;
    return x >= n ? x - n : x;
}

// Read of a grid table entry through the scalar cache.  The tables are never written by a kernel, but the
// compiler cannot know that once the kernel has stored results, and would fall back to vector loads whose
// completion wait (vmcnt) also waits for the LDS-direct copies in flight.
__device__ __forceinline__ int table_i(const int *p, int idx)
{
    int v;
    const int *a = p + idx;
    asm("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(a));
    return v;
}
__device__ __forceinline__ float table_f(const float *p, int idx)
{
    return __builtin_bit_cast(float, table_i(reinterpret_cast<const int *>(p), idx));
}

// channel held by (lane half, register index i): groups of four alternate between the halves, so the
// two lanes of a pair read LDS rows four apart
__device__ __forceinline__ constexpr int chan_fwd(int half, int i) { return (i >> 2) * 8 + half * 4 + (i & 3); }

// This wavefront's share of the copy of input latitude r into a ring slot: channel rows wave, wave + nw, ...
// of the 64 (K then V), three 64-column pieces each.  voff = byte offsets of the lane's column in each piece.
__device__ __forceinline__ void stage_row(const float *kb, const float *vb, size_t si, unsigned (&voff)[3],
                                          float *slot, int wave, int nw)
{
#pragma unroll
    for (int a = 0; a < 3; ++a) asm volatile("" : "+v"(voff[a]));   // keep the 32-bit offsets: no widened lane addresses
    for (int rr = wave; rr < 2 * kD; rr += nw) {
        const bool isv = rr >= kD;
        const char *rb = reinterpret_cast<const char *>((isv ? vb : kb) + size_t(isv ? rr - kD : rr) * si);
        asm volatile("" : "+s"(rb));
        float *dst = slot + rr * kPitchS;
#pragma unroll
        for (int a = 0; a < 3; ++a)
            __builtin_amdgcn_global_load_lds((gptr_t)(rb + voff[a]), (lptr_t)(dst + 64 * a), 4, 0, 0);
    }
}

// Strip of SL4 float4 from the lane's i-th channel row (p already includes the lane's row and column base).
template <int SL4>
__device__ __forceinline__ void read_strip(const float *p, int i, float (&st)[4 * SL4])
{
#pragma unroll
    for (int a = 0; a < SL4; ++a) {
        const float4 x = *reinterpret_cast<const float4 *>(p + chan_fwd(0, i) * kPitchS + 4 * a);
        st[4 * a] = x.x; st[4 * a + 1] = x.y; st[4 * a + 2] = x.z; st[4 * a + 3] = x.w;
    }
}

// One run of NT window offsets starting at an aligned window column (soff already includes it): logits,
// online softmax update, P.V.  The first `lead` offsets lie in front of the arc.
template <int NT>
__device__ __forceinline__ void stream_run_fwd(const float *slot, int soff, int lead, float wq,
                                               const float (&q)[4][kD / 2], float (&acc)[4][kD / 2],
                                               float (&mref)[4], float (&lsum)[4])
{
    constexpr int SL4 = (NT + 3 + 3) / 4;
    float s[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) s[r][tt] = 0.f;
    const float *kp = slot + soff;
    // One strip at a time, fenced: pulling several channels' strips to the front does not fit in the
    // registers next to q, the accumulator and the logits (a spill reload waits on the vector-memory counter
    // and with it on the LDS-direct copies of the next row, which costs far more than the LDS latency hidden).
#pragma unroll
    for (int i = 0; i < kD / 2; ++i) {
        float st[4 * SL4];
        read_strip<SL4>(kp, i, st);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) s[r][tt] = fmaf(q[r][i], st[r + tt], s[r][tt]);
        __builtin_amdgcn_sched_barrier(0);
    }
    float cmax[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        cmax[r] = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            s[r][tt] += dpp_swap_pair(s[r][tt]);
            if (tt < 3) s[r][tt] = tt < lead ? -INFINITY : s[r][tt];
            cmax[r] = fmaxf(cmax[r], s[r][tt]);
        }
    }
    // The reference maximum only moves when exceeded by 2^8, so corr is almost always exactly 1; the
    // accumulator is multiplied unconditionally all the same: a branch here makes the compiler keep two
    // copies of the 64 accumulator registers alive, which costs more than the multiplies.
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float m_new = cmax[r] > mref[r] + 8.f ? cmax[r] : mref[r];
        const float corr = __builtin_amdgcn_exp2f(mref[r] - m_new);
        mref[r] = m_new;
        lsum[r] *= corr;
#pragma unroll
        for (int c = 0; c < kD / 2; ++c) acc[r][c] *= corr;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            s[r][tt] = wq * __builtin_amdgcn_exp2f(s[r][tt] - mref[r]);
            lsum[r] += s[r][tt];
        }
    const float *vp = kp + kD * kPitchS;
#pragma unroll
    for (int i = 0; i < kD / 2; ++i) {
        float st[4 * SL4];
        read_strip<SL4>(vp, i, st);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r][i] = fmaf(s[r][tt], st[r + tt], acc[r][i]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Segment `sl` of `nsl` equal-cost pieces of the latitude range [lo, hi): cum[i] is the running cost of the
// first i latitudes.  Boundary j is the first latitude whose running cost reaches j / nsl of the total.
__device__ __forceinline__ void segment_bounds(int sl, int nsl, int lo, int hi, const int *cum, int &a, int &b)
{
    const int n = hi - lo;
    const long total = cum[n];
    const long ta = total * sl / nsl, tb = total * (sl + 1) / nsl;
    a = b = n;
    for (int i = n - 1; i >= 0; --i) {
        const int c = cum[i];
        if (c >= ta) a = i;
        if (c >= tb) b = i;
    }
    if (sl == nsl - 1) b = n;
    a += lo; b += lo;
}

__global__ void __launch_bounds__(64 * kMaxWaves)
nattn_fwd_stream(S2DeviceTables t, int nbh, int nsl, float qscale, const float *__restrict__ q,
                 const float *__restrict__ k, const float *__restrict__ v, float *__restrict__ out,
                 float *__restrict__ lse)
{
    constexpr int DH = kD / 2;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int nw = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;

    const int nseg = (t.nlon_out + kSegS - 1) / kSegS;
    int id = blockIdx.x;
    const int seg = id % nseg; id /= nseg;
    const int bh = id % nbh;
    int h_lo, h_hi;
    segment_bounds(id / nbh, nsl, t.st_lo, t.st_hi, t.st_cum, h_lo, h_hi);
    if (h_lo >= h_hi) return;   // (more segments than latitudes)

    const int nlon = t.nlon_in;   // equal longitude counts on both grids
    const int p = lane >> 1, half = lane & 1;
    const int w0 = seg * kSegS + 4 * p;
    const bool active = w0 < t.nlon_out;
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    // lane's strip base in a slot: its channel rows start at row 4*half, its columns at 4*p
    const int sbase = half * 4 * kPitchS + 4 * p;

    // window = columns seg*128 - 32 .. seg*128 + 159 (mod nlon)
    unsigned voff[3];
    {
        const int xw = wrap2(seg * kSegS - kHalo + nlon, nlon);
#pragma unroll
        for (int a = 0; a < 3; ++a) voff[a] = 4u * unsigned(wrap2(wrap2(xw + lane, nlon) + 64 * a, nlon));
    }
    const float *kslice = k + size_t(bh) * kD * si, *vslice = v + size_t(bh) * kD * si;

    const int r_first = t.band_lo[h_lo];
    const int r_last = t.band_lo[h_hi - 1] + t.band_n[h_hi - 1] - 1;

    float qr[4][DH], acc[4][DH], mref[4], lsum[4];
    int h = h_lo + wave;
    // q / out addressing: a uniform running pointer over the channel rows plus one 32-bit lane offset, kept
    // opaque so that sixteen 64-bit lane addresses are not computed up front and parked in registers
    unsigned lane_off = unsigned((size_t(half) * 4 * so + w0) * sizeof(float));
    const size_t row_bytes = so * sizeof(float);
    auto load_q = [&](int hh) {
        const char *rb = reinterpret_cast<const char *>(q + size_t(bh) * kD * so + size_t(hh) * t.nlon_out);
        asm volatile("" : "+s"(rb));
        asm volatile("" : "+v"(lane_off));
#pragma unroll
        for (int i = 0; i < DH; ++i) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (active) x = *reinterpret_cast<const float4 *>(rb + lane_off);
            rb += (i & 3) == 3 ? 5 * row_bytes : row_bytes;
            qr[0][i] = x.x * qscale; qr[1][i] = x.y * qscale; qr[2][i] = x.z * qscale; qr[3][i] = x.w * qscale;
            acc[0][i] = acc[1][i] = acc[2][i] = acc[3][i] = 0.f;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) { mref[r] = -INFINITY; lsum[r] = 0.f; }
    };
    auto store_out = [&](int hh) {
        if (!active) return;
        char *rb = reinterpret_cast<char *>(out + size_t(bh) * kD * so + size_t(hh) * t.nlon_out);
        asm volatile("" : "+s"(rb));
        asm volatile("" : "+v"(lane_off));
        float inv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) inv[r] = 1.f / lsum[r];
#pragma unroll
        for (int i = 0; i < DH; ++i) {
            *reinterpret_cast<float4 *>(rb + lane_off) =
                make_float4(acc[0][i] * inv[0], acc[1][i] * inv[1], acc[2][i] * inv[2], acc[3][i] * inv[3]);
            rb += (i & 3) == 3 ? 5 * row_bytes : row_bytes;
        }
        if (half == 0) {
            float L[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) L[r] = (mref[r] + log2f(lsum[r] * t.omega_ref)) * 0.6931471805599453f;
            *reinterpret_cast<float4 *>(lse + size_t(bh) * so + size_t(hh) * t.nlon_out + w0) =
                make_float4(L[0], L[1], L[2], L[3]);
        }
    };
    if (h < h_hi) load_q(h);

    stage_row(kslice + size_t(r_first) * nlon, vslice + size_t(r_first) * nlon, si, voff, smem, wave, nw);
    for (int r = r_first; r <= r_last; ++r) {
        const int cur = (r - r_first) & 1;
        // row r has landed (everything this wavefront had in flight) and, after the barrier, everybody's share
        // of it; everybody is also done with row r - 1, whose slot takes row r + 1
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (r < r_last)
            stage_row(kslice + size_t(r + 1) * nlon, vslice + size_t(r + 1) * nlon, si, voff,
                      smem + (cur ^ 1) * kSlot, wave, nw);
        const float *slot = smem + cur * kSlot;
        const float wq = table_f(t.omega_rel, r);
        while (h < h_hi) {
            const int b = r - table_i(t.band_lo, h), nb = table_i(t.band_n, h);
            if (b < 0) break;
            if (b < nb) {
                const int c = table_i(t.cnt, h * t.band_max + b);
                const int a = kHalo - ((c - 1) >> 1);
                int A = a & ~3, lead = a - A, span = a + c - A;
                int soff = sbase + A;
                while (span > kNTS) {
                    stream_run_fwd<kNTS>(slot, soff, lead, wq, qr, acc, mref, lsum);
                    lead = 0; soff += kNTS; span -= kNTS;
                }
#define S2_RUN(N) case N: stream_run_fwd<N>(slot, soff, lead, wq, qr, acc, mref, lsum); break;
                switch (span) {
                    S2_RUN(1) S2_RUN(2) S2_RUN(3) S2_RUN(4) S2_RUN(5) S2_RUN(6) S2_RUN(7) S2_RUN(8)
                }
#undef S2_RUN
            }
            if (b < nb - 1) break;
            // last row of this latitude: write it out and take the next one (whose band may start on this row)
            store_out(h);
            __builtin_amdgcn_sched_barrier(0);   // the new q must not be requested while the old state is still live
            h += nw;
            if (h < h_hi) load_q(h);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

}  // namespace

bool s2_nattn_stream_supported(const S2DeviceTables &t, int d, int e)
{
    return d == kD && e == kD && t.pscale == 1 && t.nlon_in == t.nlon_out && t.nlon_in % 4 == 0 && t.nlon_in >= kWin &&
           t.st_nw >= 1 && t.st_hi > t.st_lo;
}

int s2_nattn_fwd_stream(const S2DeviceTables &t, int nbh, float qscale, const float *q, const float *k,
                        const float *v, float *out, float *lse, hipStream_t st)
{
    const int nw = t.st_nw;
    const int nseg = (t.nlon_out + kSegS - 1) / kSegS;
    // equal-cost latitude segments; one workgroup fills a compute unit, so aim at one workgroup per unit
    static const int ncu = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        return n;
    }();
    const int per = nbh * nseg;
    int nsl = (ncu + per / 2) / per;
    nsl = nsl < 1 ? 1 : nsl;
    const int max_nsl = (t.st_hi - t.st_lo + nw - 1) / nw;
    nsl = nsl > max_nsl ? max_nsl : nsl;
    const size_t lds = 2 * size_t(kSlot) * sizeof(float);
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(nattn_fwd_stream),
                                hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)) != hipSuccess)
            return -1;
        configured = true;
    }
    S2TraceScope tr("nattn_fwd_stream", nbh * t.fwd_pairs[3], st);
    hipLaunchKernelGGL(nattn_fwd_stream, dim3(unsigned(nsl * nbh * nseg)), dim3(64 * nw), lds, st, t, nbh, nsl, qscale, q,
                       k, v, out, lse);
    return 0;
}
