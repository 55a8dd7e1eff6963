// Streaming float32 kernels for the light latitudes of spherical neighborhood
// attention on gfx950 (App. B.1 second equation in the index form of App. B.3;
// gradients of App. B.4).
//
// Away from the poles a disk meets about nine input latitudes on short arcs,
// and neighbouring output latitudes share eight of those nine.  Here a
// workgroup walks DOWN a range of consecutive output latitudes for one strip of
// 128 longitudes and one (batch, head): input latitude r is copied into LDS
// once (all 32 K channels and all 32 V channels of the strip plus a halo of 32
// columns on each side, LDS-direct loads into a ring of three slots) and consumed by
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

    // Ring of three slots, rows requested two steps ahead.  A step is: barrier (row r is complete for everybody,
    // everybody is done with row r - 1), work on row r, wait for this wavefront's share of row r + 1 (requested a
    // whole step ago), request row r + 2 into the slot row r - 1 occupied.  Wavefronts with little work in a
    // step reach the request early, so their copies overlap the arithmetic of the busy ones.
    stage_row(kslice + size_t(r_first) * nlon, vslice + size_t(r_first) * nlon, si, voff, smem, wave, nw);
    if (r_first < r_last)
        stage_row(kslice + size_t(r_first + 1) * nlon, vslice + size_t(r_first + 1) * nlon, si, voff, smem + kSlot,
                  wave, nw);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    int cur = 0;
    for (int r = r_first; r <= r_last; ++r) {
        __syncthreads();
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
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const int nxt2 = cur == 0 ? 2 : cur - 1;   // (cur + 2) % 3
        if (r + 2 <= r_last)
            stage_row(kslice + size_t(r + 2) * nlon, vslice + size_t(r + 2) * nlon, si, voff, smem + nxt2 * kSlot, wave,
                      nw);
        cur = cur == 2 ? 0 : cur + 1;
    }
}


// ------------------------------------------------------------- backward ----------
//
// Same streaming structure with the register budget of the gradient kernels: FOUR adjacent lanes share four
// consecutive points and each carries 8 of the 32 channels (channel 4 i + quarter, so the four lanes read
// adjacent LDS rows; with a pitch of 16 mod 64 floats their b128 strips cover the 64 banks exactly once).
// A wavefront owns 64 longitudes, a workgroup one strip of 64 longitudes plus the halo (128 window columns).
//   dq    : owners are output points; rows of K and V stream by (s = q.K, dP = dout.V, dq += dS K); stores D_i.
//   dk/dv : owners are INPUT points (transposed neighborhood); rows of q, dout, lse and D stream by.

constexpr int kDL = 8;                    // channels per lane
constexpr int kSegQ = 64;                 // owner longitudes per workgroup
constexpr int kWinQ = kSegQ + 2 * kHalo;  // 128 window columns = two 64-lane loads per row
constexpr int kPitchQ = kWinQ + 16;       // 16 mod 64
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float quad_sum(float x)
{
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, true));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, true));
    return x;
}

// Reduce-scatter over a lane quad: a0..a3 are the lanes' partial sums for the quad's four points; lane qd gets
// the full sum for point qd (b0, b1 = bits of qd).  The softmax arithmetic that follows is then done once per
// (point, offset) by the lane that owns the point and handed back to the other three with quad_bcast, instead
// of being repeated by all four lanes.
__device__ __forceinline__ float quad_reduce_scatter(float a0, float a1, float a2, float a3, bool b0, bool b1)
{
    const float u01 = b0 ? a1 : a0, w01 = b0 ? a0 : a1;
    const float t01 = u01 + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, w01), 0xB1, 0xf, 0xf, true));
    const float u23 = b0 ? a3 : a2, w23 = b0 ? a2 : a3;
    const float t23 = u23 + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, w23), 0xB1, 0xf, 0xf, true));
    const float x = b1 ? t23 : t01, y = b1 ? t01 : t23;
    return x + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, y), 0x4E, 0xf, 0xf, true));
}

template <int R>
__device__ __forceinline__ float quad_bcast(float x)   // value of lane R of the quad
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), R * 0x55, 0xf, 0xf, true));
}

// This wavefront's share of the copy of one streamed latitude into a ring slot: rows wave, wave + nw, ... of
// the nrows rows; row rr comes from base[rr / 32] + (rr % 32) * stride for the 64 channel rows and from
// extra[rr - 64] for the per-point rows (lse, D) behind them.
__device__ __forceinline__ void stage_row_q(const float *a, const float *b, size_t stride, const float *x0,
                                            const float *x1, int nrows, unsigned (&voff)[2], float *slot, int wave,
                                            int nw)
{
#pragma unroll
    for (int c = 0; c < 2; ++c) asm volatile("" : "+v"(voff[c]));
    for (int rr = wave; rr < nrows; rr += nw) {
        const float *src = rr < kD ? a + size_t(rr) * stride
                                   : rr < 2 * kD ? b + size_t(rr - kD) * stride : rr == 2 * kD ? x0 : x1;
        const char *rb = reinterpret_cast<const char *>(src);
        asm volatile("" : "+s"(rb));
        float *dst = slot + rr * kPitchQ;
#pragma unroll
        for (int c = 0; c < 2; ++c)
            __builtin_amdgcn_global_load_lds((gptr_t)(rb + voff[c]), (lptr_t)(dst + 64 * c), 4, 0, 0);
    }
}

// Counting semaphores in LDS for the ring of row slots of the gradient kernels.  The wavefronts of a workgroup
// do very different amounts of work on one streamed row (1 to 9+ offsets, depending on where the row lies in the
// band of their latitude), so a barrier per row leaves them idle for a third of the time.  Instead, every
// wavefront counts "my share of the row in this slot has landed" and "I am done reading this slot"; a wavefront
// waits only for the count it needs, which lets the fast ones run one row ahead of the slow ones.  The waits are
// bounded: if a count never arrives (which would be a bug) the wavefront goes on after about ten milliseconds
// instead of hanging the device, the results are then wrong rather than missing, and the kernel sets a flag in
// device memory that s2_grid_device_flags reports.
__device__ __forceinline__ void sem_signal(unsigned *p, int lane)
{
    if (lane == 0) __hip_atomic_fetch_add(p, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ void sem_wait(unsigned *p, unsigned target, bool &gave_up)
{
    if (gave_up) return;
    for (int spin = 0; spin < (1 << 17); ++spin) {
        const unsigned v = __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (__builtin_amdgcn_readfirstlane(v) >= target) return;
        __builtin_amdgcn_s_sleep(2);
    }
    gave_up = true;   // no further waiting in this wavefront: the kernel ends quickly whatever went wrong
}

template <int SL4>
__device__ __forceinline__ void read_strip_q(const float *p, float (&st)[4 * SL4])
{
#pragma unroll
    for (int a = 0; a < SL4; ++a) {
        const float4 x = *reinterpret_cast<const float4 *>(p + 4 * a);
        st[4 * a] = x.x; st[4 * a + 1] = x.y; st[4 * a + 2] = x.z; st[4 * a + 3] = x.w;
    }
}

// acc[r][tt] += own[r][i] * row_i[r + tt] over the lane's 8 channels (rows 4 i of p).  The next channel's strip is
// requested before this channel's FMAs; the fence keeps the scheduler from pulling more strips to the front
// (without it the kernels spill).
template <int NT>
__device__ __forceinline__ void dot_rows(const float *p, const float (&own)[4][kDL], float (&acc)[4][NT])
{
    constexpr int SL4 = (NT + 6) / 4;
    float st[2][4 * SL4];
    read_strip_q<SL4>(p, st[0]);
#pragma unroll
    for (int i = 0; i < kDL; ++i) {
        if (i + 1 < kDL) read_strip_q<SL4>(p + 4 * (i + 1) * kPitchQ, st[(i + 1) & 1]);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r][tt] = fmaf(own[r][i], st[i & 1][r + tt], acc[r][tt]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// out[r][i] += sum_tt w[r][tt] * row_i[r + tt]
template <int NT>
__device__ __forceinline__ void axpy_rows(const float *p, const float (&w)[4][NT], float (&out)[4][kDL])
{
    constexpr int SL4 = (NT + 6) / 4;
    float st[2][4 * SL4];
    read_strip_q<SL4>(p, st[0]);
#pragma unroll
    for (int i = 0; i < kDL; ++i) {
        if (i + 1 < kDL) read_strip_q<SL4>(p + 4 * (i + 1) * kPitchQ, st[(i + 1) & 1]);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) out[r][i] = fmaf(w[r][tt], st[i & 1][r + tt], out[r][i]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// lse2o, Dro: logsumexp (base 2, relative) and D of the point this lane owns within its quad (point qd)
template <int NT>
__device__ __forceinline__ void stream_run_dq(const float *slot, int soff, int lead, float wq, bool b0, bool b1,
                                              const float (&q)[4][kDL], const float (&go)[4][kDL], float lse2o,
                                              float Dro, float (&dq)[4][kDL])
{
    float s[4][NT], dp[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) { s[r][tt] = 0.f; dp[r][tt] = 0.f; }
    const float *kp = slot + soff, *vp = kp + kD * kPitchQ;
    dot_rows<NT>(kp, q, s);
    dot_rows<NT>(vp, go, dp);
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
        const float sv = quad_reduce_scatter(s[0][tt], s[1][tt], s[2][tt], s[3][tt], b0, b1);
        const float dv = quad_reduce_scatter(dp[0][tt], dp[1][tt], dp[2][tt], dp[3][tt], b0, b1);
        float w = wq * __builtin_amdgcn_exp2f(sv - lse2o) * (dv - Dro);
        if (tt < 3) w = tt < lead ? 0.f : w;   // offsets in front of the arc
        s[0][tt] = quad_bcast<0>(w); s[1][tt] = quad_bcast<1>(w);
        s[2][tt] = quad_bcast<2>(w); s[3][tt] = quad_bcast<3>(w);
    }
    axpy_rows<NT>(kp, s, dq);
}

__global__ void __launch_bounds__(64 * kMaxWaves)
nattn_bwd_dq_stream(S2DeviceTables t, int nbh, int nsl, float scale, const float *__restrict__ q,
                    const float *__restrict__ k, const float *__restrict__ v, const float *__restrict__ o,
                    const float *__restrict__ lse, const float *__restrict__ go, float *__restrict__ dq,
                    float *__restrict__ Dws)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    constexpr int kSlotQ = 2 * kD * kPitchQ;
    const int nw = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nseg = (t.nlon_out + kSegQ - 1) / kSegQ;
    int id = blockIdx.x;
    const int seg = id % nseg; id /= nseg;
    const int bh = id % nbh;
    int h_lo, h_hi;
    segment_bounds(id / nbh, nsl, t.st_lo, t.st_hi, t.st_cum, h_lo, h_hi);
    if (h_lo >= h_hi) return;

    const int nlon = t.nlon_in;
    const int qd = lane & 3, u = lane >> 2;
    const int w0 = seg * kSegQ + 4 * u;
    const bool active = w0 < t.nlon_out;
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const int sbase = qd * kPitchQ + 4 * u;
    const float qscale = scale * kLog2e;
    unsigned voff[2];
    {
        const int xw = wrap2(seg * kSegQ - kHalo + nlon, nlon);
#pragma unroll
        for (int c = 0; c < 2; ++c) voff[c] = 4u * unsigned(wrap2(wrap2(xw + lane, nlon) + 64 * c, nlon));
    }
    const float *kslice = k + size_t(bh) * kD * si, *vslice = v + size_t(bh) * kD * si;
    const int r_first = t.band_lo[h_lo];
    const int r_last = t.band_lo[h_hi - 1] + t.band_n[h_hi - 1] - 1;

    float qr[4][kDL], gr[4][kDL], dqa[4][kDL], lse2[4], Dr[4], lse2o = 0.f, Dro = 0.f;
    const bool b0 = qd & 1, b1 = qd & 2;
    unsigned lane_off = unsigned((size_t(qd) * so + w0) * sizeof(float));
    const size_t row4 = 4 * so * sizeof(float);   // the lane's next channel is four channel rows on
    int h = h_lo + wave;
    auto load_owner = [&](int hh) {
        const size_t rowoff = (size_t(bh) * kD * so + size_t(hh) * t.nlon_out) * sizeof(float);
        const char *pq = reinterpret_cast<const char *>(q) + rowoff;
        const char *pg = reinterpret_cast<const char *>(go) + rowoff;
        const char *po = reinterpret_cast<const char *>(o) + rowoff;
        asm volatile("" : "+s"(pq)); asm volatile("" : "+s"(pg)); asm volatile("" : "+s"(po));
        asm volatile("" : "+v"(lane_off));
#pragma unroll
        for (int r = 0; r < 4; ++r) Dr[r] = 0.f;
#pragma unroll
        for (int i = 0; i < kDL; ++i) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x, z = x;
            if (active) {
                x = *reinterpret_cast<const float4 *>(pq + lane_off);
                y = *reinterpret_cast<const float4 *>(pg + lane_off);
                z = *reinterpret_cast<const float4 *>(po + lane_off);
            }
            pq += row4; pg += row4; po += row4;
            qr[0][i] = x.x * qscale; qr[1][i] = x.y * qscale; qr[2][i] = x.z * qscale; qr[3][i] = x.w * qscale;
            gr[0][i] = y.x; gr[1][i] = y.y; gr[2][i] = y.z; gr[3][i] = y.w;
            Dr[0] = fmaf(y.x, z.x, Dr[0]); Dr[1] = fmaf(y.y, z.y, Dr[1]);
            Dr[2] = fmaf(y.z, z.z, Dr[2]); Dr[3] = fmaf(y.w, z.w, Dr[3]);
            dqa[0][i] = dqa[1][i] = dqa[2][i] = dqa[3][i] = 0.f;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) Dr[r] = quad_sum(Dr[r]);
        const size_t io = size_t(bh) * so + size_t(hh) * t.nlon_out + w0;
        float4 L = make_float4(0.f, 0.f, 0.f, 0.f);
        if (active) L = *reinterpret_cast<const float4 *>(lse + io);
        lse2[0] = (L.x - t.ln_omega_ref) * kLog2e; lse2[1] = (L.y - t.ln_omega_ref) * kLog2e;
        lse2[2] = (L.z - t.ln_omega_ref) * kLog2e; lse2[3] = (L.w - t.ln_omega_ref) * kLog2e;
        if (active && qd == 0) *reinterpret_cast<float4 *>(Dws + io) = make_float4(Dr[0], Dr[1], Dr[2], Dr[3]);
        lse2o = b1 ? (b0 ? lse2[3] : lse2[2]) : (b0 ? lse2[1] : lse2[0]);
        Dro = b1 ? (b0 ? Dr[3] : Dr[2]) : (b0 ? Dr[1] : Dr[0]);
    };
    auto store_owner = [&](int hh) {
        if (!active) return;
        char *pd = reinterpret_cast<char *>(dq) + (size_t(bh) * kD * so + size_t(hh) * t.nlon_out) * sizeof(float);
        asm volatile("" : "+s"(pd));
        asm volatile("" : "+v"(lane_off));
#pragma unroll
        for (int i = 0; i < kDL; ++i) {
            *reinterpret_cast<float4 *>(pd + lane_off) =
                make_float4(dqa[0][i] * scale, dqa[1][i] * scale, dqa[2][i] * scale, dqa[3][i] * scale);
            pd += row4;
        }
    };
    if (h < h_hi) load_owner(h);

    // Ring of four slots, rows requested three steps ahead; see sem_signal / sem_wait.  A step is: wait until row r
    // has landed for everybody, work on it, mark the slot as read, announce this wavefront's share of row r + 2
    // (requested a whole step ago), wait until everybody has read row r - 1 and request row r + 3 into its slot.
    unsigned *arrived = reinterpret_cast<unsigned *>(smem + 4 * kSlotQ), *released = arrived + 4;
    if (threadIdx.x < 8) arrived[threadIdx.x] = 0u;
    __syncthreads();
    auto stage = [&](int rr, int slot_idx) {
        stage_row_q(kslice + size_t(rr) * nlon, vslice + size_t(rr) * nlon, si, nullptr, nullptr, 2 * kD, voff,
                    smem + slot_idx * kSlotQ, wave, nw);
    };
    for (int j = 0; j < 3; ++j)
        if (r_first + j <= r_last) stage(r_first + j, j);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    for (int j = 0; j < 2; ++j)
        if (r_first + j <= r_last) sem_signal(arrived + j, lane);
    int cur = 0;
    bool gave_up = false;
    unsigned fill = unsigned(nw);   // count that completes the current use of slot `cur`
    for (int r = r_first; r <= r_last; ++r) {
        sem_wait(arrived + cur, fill, gave_up);
        const float *slot = smem + cur * kSlotQ;
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
                    stream_run_dq<kNTS>(slot, soff, lead, wq, b0, b1, qr, gr, lse2o, Dro, dqa);
                    lead = 0; soff += kNTS; span -= kNTS;
                }
#define S2_RUN(N) case N: stream_run_dq<N>(slot, soff, lead, wq, b0, b1, qr, gr, lse2o, Dro, dqa); break;
                switch (span) {
                    S2_RUN(1) S2_RUN(2) S2_RUN(3) S2_RUN(4) S2_RUN(5) S2_RUN(6) S2_RUN(7) S2_RUN(8)
                }
#undef S2_RUN
            }
            if (b < nb - 1) break;
            store_owner(h);
            __builtin_amdgcn_sched_barrier(0);
            h += nw;
            if (h < h_hi) load_owner(h);
            __builtin_amdgcn_sched_barrier(0);
        }
        sem_signal(released + cur, lane);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (r + 2 <= r_last) sem_signal(arrived + ((cur + 2) & 3), lane);
        if (r + 3 <= r_last) {
            const int prev = (cur + 3) & 3;   // slot of row r - 1
            // uses of that slot completed so far: one less than `fill / nw` if it lies ahead of `cur` in the ring
            if (r > r_first) sem_wait(released + prev, cur == 0 ? fill - unsigned(nw) : fill, gave_up);
            stage(r + 3, prev);
        }
        cur = (cur + 1) & 3;
        if (cur == 0) fill += unsigned(nw);
    }
    if (gave_up && lane == 0) atomicOr(t.dev_flags, 1u);
}

// xoff: float offset of the quad's first point in the lse / D rows of the slot; qd: the lane's own point
template <int NT>
__device__ __forceinline__ void stream_run_dkdv(const float *slot, int soff, int xoff, int lead, float wq, float lref2,
                                                bool b0, bool b1, int qd, const float (&kr)[4][kDL],
                                                const float (&vr)[4][kDL], float (&dk)[4][kDL], float (&dv)[4][kDL])
{
    float s[4][NT], dp[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) { s[r][tt] = 0.f; dp[r][tt] = 0.f; }
    const float *qp = slot + soff, *gp = qp + kD * kPitchQ;
    dot_rows<NT>(qp, kr, s);
    dot_rows<NT>(gp, vr, dp);
    // the streamed points' logsumexp and D for this lane's own point (rows 64 and 65 of the slot)
    const float *lp = slot + 2 * kD * kPitchQ + xoff + qd, *dp_row = lp + kPitchQ;
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
        const float sv = quad_reduce_scatter(s[0][tt], s[1][tt], s[2][tt], s[3][tt], b0, b1);
        const float dvv = quad_reduce_scatter(dp[0][tt], dp[1][tt], dp[2][tt], dp[3][tt], b0, b1);
        float pr = wq * __builtin_amdgcn_exp2f(sv - fmaf(lp[tt], kLog2e, -lref2));
        if (tt < 3) pr = tt < lead ? 0.f : pr;   // offsets in front of the arc
        const float ds = pr * (dvv - dp_row[tt]);
        s[0][tt] = quad_bcast<0>(ds); s[1][tt] = quad_bcast<1>(ds);
        s[2][tt] = quad_bcast<2>(ds); s[3][tt] = quad_bcast<3>(ds);
        dp[0][tt] = quad_bcast<0>(pr); dp[1][tt] = quad_bcast<1>(pr);
        dp[2][tt] = quad_bcast<2>(pr); dp[3][tt] = quad_bcast<3>(pr);
    }
    axpy_rows<NT>(qp, s, dk);
    axpy_rows<NT>(gp, dp, dv);
}

__global__ void __launch_bounds__(64 * kMaxWaves)
nattn_bwd_dkdv_stream(S2DeviceTables t, int nbh, int nsl, float scale, const float *__restrict__ q,
                      const float *__restrict__ k, const float *__restrict__ v, const float *__restrict__ lse,
                      const float *__restrict__ go, const float *__restrict__ Dws, float *__restrict__ dk,
                      float *__restrict__ dv)
{
    extern __shared__ __attribute__((aligned(16))) float smem[];
    constexpr int kRowsKV = 2 * kD + 2;
    constexpr int kSlotKV = kRowsKV * kPitchQ;
    const int nw = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int nseg = (t.nlon_in + kSegQ - 1) / kSegQ;
    int id = blockIdx.x;
    const int seg = id % nseg; id /= nseg;
    const int bh = id % nbh;
    int h_lo, h_hi;   // input latitudes owned by this workgroup
    segment_bounds(id / nbh, nsl, t.tst_lo, t.tst_hi, t.tst_cum, h_lo, h_hi);
    if (h_lo >= h_hi) return;

    const int nlon = t.nlon_out;   // equal longitude counts: streamed rows are output latitudes
    const int qd = lane & 3, u = lane >> 2;
    const int w0 = seg * kSegQ + 4 * u;
    const bool active = w0 < t.nlon_in;
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const int sbase = qd * kPitchQ + 4 * u, xbase = 4 * u;
    const float qscale = scale * kLog2e, lref2 = t.ln_omega_ref * kLog2e;
    unsigned voff[2];
    {
        const int xw = wrap2(seg * kSegQ - kHalo + nlon, nlon);
#pragma unroll
        for (int c = 0; c < 2; ++c) voff[c] = 4u * unsigned(wrap2(wrap2(xw + lane, nlon) + 64 * c, nlon));
    }
    const float *qslice = q + size_t(bh) * kD * so, *gslice = go + size_t(bh) * kD * so;
    const float *lslice = lse + size_t(bh) * so, *dslice = Dws + size_t(bh) * so;
    const int r_first = t.tband_lo[h_lo];
    const int r_last = t.tband_lo[h_hi - 1] + t.tband_n[h_hi - 1] - 1;

    float kr[4][kDL], vr[4][kDL], dka[4][kDL], dva[4][kDL];
    const bool b0 = qd & 1, b1 = qd & 2;
    unsigned lane_off = unsigned((size_t(qd) * si + w0) * sizeof(float));
    const size_t row4 = 4 * si * sizeof(float);
    int h = h_lo + wave;
    float wq = 0.f;
    auto load_owner = [&](int hh) {
        const size_t rowoff = (size_t(bh) * kD * si + size_t(hh) * t.nlon_in) * sizeof(float);
        const char *pk = reinterpret_cast<const char *>(k) + rowoff;
        const char *pv = reinterpret_cast<const char *>(v) + rowoff;
        asm volatile("" : "+s"(pk)); asm volatile("" : "+s"(pv));
        asm volatile("" : "+v"(lane_off));
#pragma unroll
        for (int i = 0; i < kDL; ++i) {
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x;
            if (active) {
                x = *reinterpret_cast<const float4 *>(pk + lane_off);
                y = *reinterpret_cast<const float4 *>(pv + lane_off);
            }
            pk += row4; pv += row4;
            kr[0][i] = x.x * qscale; kr[1][i] = x.y * qscale; kr[2][i] = x.z * qscale; kr[3][i] = x.w * qscale;
            vr[0][i] = y.x; vr[1][i] = y.y; vr[2][i] = y.z; vr[3][i] = y.w;
            dka[0][i] = dka[1][i] = dka[2][i] = dka[3][i] = 0.f;
            dva[0][i] = dva[1][i] = dva[2][i] = dva[3][i] = 0.f;
        }
        wq = table_f(t.omega_rel, hh);
    };
    auto store_owner = [&](int hh) {
        if (!active) return;
        const size_t rowoff = (size_t(bh) * kD * si + size_t(hh) * t.nlon_in) * sizeof(float);
        char *pk = reinterpret_cast<char *>(dk) + rowoff;
        char *pv = reinterpret_cast<char *>(dv) + rowoff;
        asm volatile("" : "+s"(pk)); asm volatile("" : "+s"(pv));
        asm volatile("" : "+v"(lane_off));
#pragma unroll
        for (int i = 0; i < kDL; ++i) {
            *reinterpret_cast<float4 *>(pk + lane_off) =
                make_float4(dka[0][i] * scale, dka[1][i] * scale, dka[2][i] * scale, dka[3][i] * scale);
            *reinterpret_cast<float4 *>(pv + lane_off) = make_float4(dva[0][i], dva[1][i], dva[2][i], dva[3][i]);
            pk += row4; pv += row4;
        }
    };
    if (h < h_hi) load_owner(h);

    auto stage = [&](int rr, int slot_idx) {
        stage_row_q(qslice + size_t(rr) * nlon, gslice + size_t(rr) * nlon, so, lslice + size_t(rr) * nlon,
                    dslice + size_t(rr) * nlon, kRowsKV, voff, smem + slot_idx * kSlotKV, wave, nw);
    };
    unsigned *arrived = reinterpret_cast<unsigned *>(smem + 4 * kSlotKV), *released = arrived + 4;
    if (threadIdx.x < 8) arrived[threadIdx.x] = 0u;
    __syncthreads();
    for (int j = 0; j < 3; ++j)
        if (r_first + j <= r_last) stage(r_first + j, j);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    for (int j = 0; j < 2; ++j)
        if (r_first + j <= r_last) sem_signal(arrived + j, lane);
    int cur = 0;
    bool gave_up = false;
    unsigned fill = unsigned(nw);
    for (int r = r_first; r <= r_last; ++r) {
        sem_wait(arrived + cur, fill, gave_up);
        const float *slot = smem + cur * kSlotKV;
        while (h < h_hi) {
            const int b = r - table_i(t.tband_lo, h), nb = table_i(t.tband_n, h);
            if (b < 0) break;
            if (b < nb) {
                const int c = table_i(t.tcnt, h * t.tband_max + b);
                const int a = kHalo - ((c - 1) >> 1);
                int A = a & ~3, lead = a - A, span = a + c - A;
                int soff = sbase + A, xoff = xbase + A;
                while (span > kNTS) {
                    stream_run_dkdv<kNTS>(slot, soff, xoff, lead, wq, lref2, b0, b1, qd, kr, vr, dka, dva);
                    lead = 0; soff += kNTS; xoff += kNTS; span -= kNTS;
                }
#define S2_RUN(N) case N: stream_run_dkdv<N>(slot, soff, xoff, lead, wq, lref2, b0, b1, qd, kr, vr, dka, dva); break;
                switch (span) {
                    S2_RUN(1) S2_RUN(2) S2_RUN(3) S2_RUN(4) S2_RUN(5) S2_RUN(6) S2_RUN(7) S2_RUN(8)
                }
#undef S2_RUN
            }
            if (b < nb - 1) break;
            store_owner(h);
            __builtin_amdgcn_sched_barrier(0);
            h += nw;
            if (h < h_hi) load_owner(h);
            __builtin_amdgcn_sched_barrier(0);
        }
        sem_signal(released + cur, lane);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (r + 2 <= r_last) sem_signal(arrived + ((cur + 2) & 3), lane);
        if (r + 3 <= r_last) {
            const int prev = (cur + 3) & 3;
            if (r > r_first) sem_wait(released + prev, cur == 0 ? fill - unsigned(nw) : fill, gave_up);
            stage(r + 3, prev);
        }
        cur = (cur + 1) & 3;
        if (cur == 0) fill += unsigned(nw);
    }
    if (gave_up && lane == 0) atomicOr(t.dev_flags, 1u);
}

}  // namespace

namespace {

int num_compute_units()
{
    static const int ncu = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        return n;
    }();
    return ncu;
}

// equal-cost latitude segments; one workgroup fills a compute unit, so aim at one workgroup per unit
int num_segments(int per, int lo, int hi, int nw)
{
    const int ncu = num_compute_units();
    int nsl = (ncu + per / 2) / per;
    nsl = nsl < 1 ? 1 : nsl;
    const int max_nsl = (hi - lo + nw - 1) / nw;
    return nsl > max_nsl ? max_nsl : nsl;
}

constexpr size_t kLdsFwdStream = 3 * size_t(kSlot) * sizeof(float);
constexpr size_t kLdsDqStream = 4 * size_t(2 * kD * kPitchQ) * sizeof(float) + 8 * sizeof(unsigned);
constexpr size_t kLdsDkdvStream = 4 * size_t((2 * kD + 2) * kPitchQ) * sizeof(float) + 8 * sizeof(unsigned);

}  // namespace


int s2_nattn_stream_configure()
{
    auto raise = [](auto kern, size_t lds) {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   int(lds)) == hipSuccess;
    };
    return raise(nattn_fwd_stream, kLdsFwdStream) && raise(nattn_bwd_dq_stream, kLdsDqStream) &&
           raise(nattn_bwd_dkdv_stream, kLdsDkdvStream) ? 0 : -1;
}

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
    const int nsl = num_segments(nbh * nseg, t.st_lo, t.st_hi, nw);
    const size_t lds = kLdsFwdStream;
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    S2TraceScope tr("nattn_fwd_stream", nbh * t.fwd_pairs[3], st);
    hipLaunchKernelGGL(nattn_fwd_stream, dim3(unsigned(nsl * nbh * nseg)), dim3(64 * nw), lds, st, t, nbh, nsl, qscale, q,
                       k, v, out, lse);
    return 0;
}
bool s2_nattn_stream_dq_supported(const S2DeviceTables &t, int d, int e)
{
    return d == kD && e == kD && t.pscale == 1 && t.nlon_in == t.nlon_out && t.nlon_in % 4 == 0 && t.nlon_in >= kWinQ &&
           t.st_nw >= 1 && t.st_hi > t.st_lo;
}

bool s2_nattn_stream_dkdv_supported(const S2DeviceTables &t, int d, int e)
{
    return d == kD && e == kD && t.pscale == 1 && t.nlon_in == t.nlon_out && t.nlon_in % 4 == 0 && t.nlon_in >= kWinQ &&
           t.tst_nw >= 1 && t.tst_hi > t.tst_lo;
}

int s2_nattn_bwd_dq_stream(const S2DeviceTables &t, int nbh, float scale, const float *q, const float *k,
                           const float *v, const float *o, const float *lse, const float *go, float *dq, float *Dws,
                           hipStream_t st)
{
    const int nseg = (t.nlon_out + kSegQ - 1) / kSegQ;
    const int nsl = num_segments(nbh * nseg, t.st_lo, t.st_hi, t.st_nw);
    const size_t lds = kLdsDqStream;
    S2TraceScope tr("nattn_bwd_dq_stream", nbh * t.fwd_pairs[3], st);
    hipLaunchKernelGGL(nattn_bwd_dq_stream, dim3(unsigned(nsl * nbh * nseg)), dim3(64 * t.st_nw), lds, st, t, nbh, nsl,
                       scale, q, k, v, o, lse, go, dq, Dws);
    return 0;
}

int s2_nattn_bwd_dkdv_stream(const S2DeviceTables &t, int nbh, float scale, const float *q, const float *k,
                             const float *v, const float *lse, const float *go, const float *Dws, float *dk, float *dv,
                             hipStream_t st)
{
    const int nseg = (t.nlon_in + kSegQ - 1) / kSegQ;
    const int nsl = num_segments(nbh * nseg, t.tst_lo, t.tst_hi, t.tst_nw);
    const size_t lds = kLdsDkdvStream;
    S2TraceScope tr("nattn_bwd_dkdv_stream", nbh * t.bwd_pairs[3], st);
    hipLaunchKernelGGL(nattn_bwd_dkdv_stream, dim3(unsigned(nsl * nbh * nseg)), dim3(64 * t.tst_nw), lds, st, t, nbh,
                       nsl, scale, q, k, v, lse, go, Dws, dk, dv);
    return 0;
}
