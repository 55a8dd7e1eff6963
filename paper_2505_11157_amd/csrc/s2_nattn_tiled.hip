// Tuned float32 forward kernel for spherical neighborhood attention on gfx950
// (App. B.1 second equation in the index form of App. B.3).
//
// Mapping.  One wavefront owns 128 consecutive output longitudes of one output
// latitude and one (batch, head).  Two adjacent lanes share four consecutive
// outputs: the even lane carries channels [0, D/2), the odd lane [D/2, D).
// Their partial q.k sums are combined with one DPP add per logit; each lane
// then accumulates its own half of the output channels, so q and the output
// accumulator cost D/2 * 4 registers each and two waves fit per SIMD.
//
// Data path.  The disk is walked as (input latitude, run of <= 12 longitude
// offsets).  For a run, the window of K (then V) columns the 128 outputs touch
// is staged through LDS four channels per half at a time (double buffered,
// next group's global loads in flight while the current one is consumed).
// Each lane then reads ONE contiguous strip of 4*PS-... + NT floats per channel
// with aligned ds_read_b128 and reuses it for all 4 x NT (output, offset)
// pairs from registers: about three FMAs per LDS float, so the kernel is bound
// by the vector ALU, not by LDS or cache bandwidth.
//
// Softmax.  Online, base 2, with the quadrature weight as a factor (see the
// generic kernel); the running reference maximum is only moved when a logit
// exceeds it by more than 2^8, which removes almost all accumulator rescales.
#include "s2_nattn_kernels.h"

namespace {

constexpr int kSeg = 128;    // outputs per wavefront
constexpr int kNTMax = 9;    // longest run of offsets handled at once
constexpr int kCG = 4;       // channels per half staged together
constexpr int kBlk = 72;     // floats per staged block: 8 channel rows x 8 columns + 8 pad

// Staged window geometry.  A stage holds 2*kCG channel rows of the
// kSeg*PS + 8 input columns a run can touch, stored as blocks of 8 columns:
// element (row, col) lives at (col / 8) * kBlk + row * 8 + col % 8.  One
// global_load_lds_dword fills one block (lane = row * 8 + column), and the
// 8-float pad rotates the banks from block to block so that the b128 strip
// reads of a lane pair (rows r and r + 4) and of its neighbours are conflict free.
template <int PS>
struct Geo {
    static constexpr int NBLK = (kSeg * PS + 8) / 8;   // 17 (PS = 1) or 33 (PS = 2)
    static constexpr int TILE = NBLK * kBlk;           // floats per buffer
};

typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

__device__ __forceinline__ float dpp_swap_pair(float x)
{
    // lane <-> lane^1 : quad_perm [1,0,3,2]
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, true));
}

// Byte offsets of the lane's element in each staged block relative to the
// channel-row base: window columns start at the lane's x0 = (first window
// column + lane % 8) mod nlon_in and advance by 8 per block around the circle.
template <int PS>
__device__ __forceinline__ void stage_offsets(unsigned rowterm, int x0, int nlon_in, unsigned (&voff)[Geo<PS>::NBLK])
{
    int x = x0;
#pragma unroll
    for (int u = 0; u < Geo<PS>::NBLK; ++u) {
        voff[u] = rowterm + 4u * unsigned(x);
        x += 8;
        x = x >= nlon_in ? x - nlon_in : x;
    }
}

// Start the asynchronous global -> LDS copy of one stage: kCG channel rows per
// half starting at chan0 (uniform pointer: first channel of the group, input
// latitude h', column 0).  One instruction per block of 8 columns.
template <int PS>
__device__ __forceinline__ void stage_issue(const float *chan0, unsigned (&voff)[Geo<PS>::NBLK], float *buf)
{
#pragma unroll
    for (int u = 0; u < Geo<PS>::NBLK; ++u) {
        asm volatile("" : "+v"(voff[u]));   // keep the offsets as 32-bit registers (no widened copies kept live)
        __builtin_amdgcn_global_load_lds((gptr_t)(reinterpret_cast<const char *>(chan0) + voff[u]),
                                         (lptr_t)(buf + u * kBlk), 4, 0, 0);
    }
}

template <int N>
__device__ __forceinline__ void wait_vm()
{
    if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if constexpr (N == 17) asm volatile("s_waitcnt vmcnt(17)" ::: "memory");
    else if constexpr (N == 33) asm volatile("s_waitcnt vmcnt(33)" ::: "memory");
    else static_assert(N == 0, "unsupported wait count");
}

// Strip of SL4 float4 for the lane's four outputs from channel row `cc` of a stage.
template <int SL4>
__device__ __forceinline__ void read_strip(const float *buf, int bE, int bO, int cc, float (&st)[4 * SL4])
{
#pragma unroll
    for (int a = 0; a < SL4; ++a) {
        const float4 x = *reinterpret_cast<const float4 *>(buf + ((a & 1) ? bO : bE) + (a >> 1) * kBlk + cc * 8);
        st[4 * a] = x.x; st[4 * a + 1] = x.y; st[4 * a + 2] = x.z; st[4 * a + 3] = x.w;
    }
}

// One run of NT offsets on one input latitude: logits, softmax update, P.V.
template <int D, int PS, int NT>
__device__ __forceinline__ void run_chunk(float *buf0, float *buf1, const float *__restrict__ kb,
                                          const float *__restrict__ vb, size_t si, unsigned rowterm, int x0,
                                          int nlon_in, int bE, int bO, float wq, const float (&q)[4][D / 2],
                                          float (&acc)[4][D / 2], float (&mref)[4], float (&lsum)[4])
{
    using G = Geo<PS>;
    constexpr int DH = D / 2, NG = DH / kCG;
    constexpr int SL = 3 * PS + NT, SL4 = (SL + 3) / 4;
    static_assert(NG % 2 == 0, "buffer parity assumes an even number of channel groups");
    float s[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) s[r][tt] = 0.f;
    unsigned voff[G::NBLK];
    stage_offsets<PS>(rowterm, x0, nlon_in, voff);

    stage_issue<PS>(kb, voff, buf0);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        float *cur = (g & 1) ? buf1 : buf0, *nxt = (g & 1) ? buf0 : buf1;
        if (g + 1 < NG) stage_issue<PS>(kb + size_t(g + 1) * kCG * si, voff, nxt);
        else stage_issue<PS>(vb, voff, nxt);
        wait_vm<G::NBLK>();
#pragma unroll
        for (int cc = 0; cc < kCG; ++cc) {
            float st[4 * SL4];
            read_strip<SL4>(cur, bE, bO, cc, st);
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int r = 0; r < 4; ++r) s[r][tt] = fmaf(q[r][g * kCG + cc], st[r * PS + tt], s[r][tt]);
        }
    }
    // combine the two channel halves; both lanes of a pair now hold the full logits
    bool need = false;
    float cmax[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        cmax[r] = -INFINITY;
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            s[r][tt] += dpp_swap_pair(s[r][tt]);
            cmax[r] = fmaxf(cmax[r], s[r][tt]);
        }
        need |= cmax[r] > mref[r] + 8.f;
    }
    if (__any(need)) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float m_new = cmax[r] > mref[r] + 8.f ? cmax[r] : mref[r];
            const float corr = __builtin_amdgcn_exp2f(mref[r] - m_new);
            mref[r] = m_new;
            lsum[r] *= corr;
#pragma unroll
            for (int c = 0; c < DH; ++c) acc[r][c] *= corr;
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            s[r][tt] = wq * __builtin_amdgcn_exp2f(s[r][tt] - mref[r]);
            lsum[r] += s[r][tt];
        }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        float *cur = (g & 1) ? buf1 : buf0, *nxt = (g & 1) ? buf0 : buf1;
        if (g + 1 < NG) {
            stage_issue<PS>(vb + size_t(g + 1) * kCG * si, voff, nxt);
            wait_vm<G::NBLK>();
        } else {
            wait_vm<0>();
        }
#pragma unroll
        for (int cc = 0; cc < kCG; ++cc) {
            float st[4 * SL4];
            read_strip<SL4>(cur, bE, bO, cc, st);
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[r][g * kCG + cc] = fmaf(s[r][tt], st[r * PS + tt], acc[r][g * kCG + cc]);
        }
    }
}

template <int D, int PS>
__global__ void __launch_bounds__(64, 2)
nattn_fwd_tiled(S2DeviceTables t, int nbh, float qscale, const float *__restrict__ q, const float *__restrict__ k,
                const float *__restrict__ v, float *__restrict__ out, float *__restrict__ lse)
{
    using G = Geo<PS>;
    constexpr int DH = D / 2;
    __shared__ __attribute__((aligned(16))) float buf0[G::TILE];
    __shared__ __attribute__((aligned(16))) float buf1[G::TILE];

    const int nseg = (t.nlon_out + kSeg - 1) / kSeg;
    int id = blockIdx.x;
    const int seg = id % nseg; id /= nseg;
    const int bh = id % nbh;
    const int h = t.row_order[id / nbh];
    const int lane = threadIdx.x, p = lane >> 1, half = lane & 1;
    const int w0 = seg * kSeg + 4 * p;
    const bool active = w0 < t.nlon_out;       // nlon_out is a multiple of 4: all four outputs or none

    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t io = size_t(h) * t.nlon_out + w0;
    // staging: lane = (channel row, column within a block of 8); rows 0..3 are the even lanes' channels
    const int srow = lane >> 3;
    const unsigned rowterm = unsigned((srow < kCG ? srow : srow - kCG + DH) * si * sizeof(float));
    // strip bases (floats) for float4 #a: even a -> bE + (a/2)*kBlk, odd a -> bO + (a/2)*kBlk
    const int c0 = 4 * p * PS;
    const int bE = (c0 >> 3) * kBlk + (c0 & 7) + half * (kCG * 8);
    const int bO = ((c0 + 4) >> 3) * kBlk + ((c0 + 4) & 7) + half * (kCG * 8);
    float qr[4][DH], acc[4][DH], mref[4], lsum[4];
#pragma unroll
    for (int c = 0; c < DH; ++c) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (active) x = *reinterpret_cast<const float4 *>(q + (size_t(bh) * D + half * DH + c) * so + io);
        qr[0][c] = x.x * qscale; qr[1][c] = x.y * qscale; qr[2][c] = x.z * qscale; qr[3][c] = x.w * qscale;
        acc[0][c] = acc[1][c] = acc[2][c] = acc[3][c] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) { mref[r] = -INFINITY; lsum[r] = 0.f; }

    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    for (int b = 0; b < nb; ++b) {
        const int hp = hp0 + b;
        const int c = t.cnt[h * t.band_max + b];
        const int lo = (c == t.nlon_in) ? 0 : -((c - 1) >> 1);
        const float wq = t.omega_rel[hp];
        const float *kb = k + size_t(bh) * D * si + size_t(hp) * t.nlon_in;
        const float *vb = v + size_t(bh) * D * si + size_t(hp) * t.nlon_in;
        const int nchunk = (c + kNTMax - 1) / kNTMax;
        const int base = c / nchunk, rem = c - base * nchunk;
        int t0 = 0;
        for (int ci = 0; ci < nchunk; ++ci) {
            const int nt = base + (ci < rem ? 1 : 0);
            int x0 = seg * kSeg * PS + lo + t0 + t.nlon_in + (lane & 7);
            x0 = x0 >= t.nlon_in ? x0 - t.nlon_in : x0;
            x0 = x0 >= t.nlon_in ? x0 - t.nlon_in : x0;
#define S2_RUN(N) case N: run_chunk<D, PS, N>(buf0, buf1, kb, vb, si, rowterm, x0, t.nlon_in, bE, bO, wq, qr, acc, mref, lsum); break;
            switch (nt) {
                S2_RUN(1) S2_RUN(2) S2_RUN(3) S2_RUN(4) S2_RUN(5) S2_RUN(6)
                S2_RUN(7) S2_RUN(8) S2_RUN(9)
            }
#undef S2_RUN
            t0 += nt;
        }
    }
    if (!active) return;
    float inv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) inv[r] = 1.f / lsum[r];
#pragma unroll
    for (int c = 0; c < DH; ++c)
        *reinterpret_cast<float4 *>(out + (size_t(bh) * D + half * DH + c) * so + io) =
            make_float4(acc[0][c] * inv[0], acc[1][c] * inv[1], acc[2][c] * inv[2], acc[3][c] * inv[3]);
    if (half == 0) {
        float L[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) L[r] = (mref[r] + log2f(lsum[r] * t.omega_ref)) * 0.6931471805599453f;
        *reinterpret_cast<float4 *>(lse + size_t(bh) * so + io) = make_float4(L[0], L[1], L[2], L[3]);
    }
}

}  // namespace

bool s2_nattn_fwd_tiled_supported(const S2DeviceTables &t, int d, int e)
{
    return d == 32 && e == 32 && (t.pscale == 1 || t.pscale == 2) && t.nlon_in % 4 == 0 && t.nlon_out % 4 == 0 &&
           t.nlon_out >= 72;   // (window wrap logic handles at most two turns of the circle)
}

int s2_nattn_fwd_tiled(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q, const float *k,
                       const float *v, float *out, float *lse, hipStream_t st)
{
    (void)d; (void)e;
    const int nseg = (t.nlon_out + kSeg - 1) / kSeg;
    const unsigned nblk = unsigned(long(nseg) * nbh * t.nlat_out);
    const float qscale = scale * 1.4426950408889634f;
    if (t.pscale == 1)
        hipLaunchKernelGGL((nattn_fwd_tiled<32, 1>), dim3(nblk), dim3(64), 0, st, t, nbh, qscale, q, k, v, out, lse);
    else
        hipLaunchKernelGGL((nattn_fwd_tiled<32, 2>), dim3(nblk), dim3(64), 0, st, t, nbh, qscale, q, k, v, out, lse);
    return 0;
}
