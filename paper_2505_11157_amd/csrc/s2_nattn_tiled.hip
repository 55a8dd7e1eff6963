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
// Data path.  The disk is walked as (input latitude, run of <= 9 longitude
// offsets).  For a run, the window of K (then V) columns the 128 outputs touch
// is staged through LDS four channels per half at a time (double buffered,
// next group's global -> LDS copies in flight while the current one is consumed).
// Each lane then reads ONE contiguous strip of 3*PS + NT floats per channel
// with aligned ds_read_b128 and reuses it for all 4 x NT (output, offset)
// pairs from registers: about three FMAs per LDS float, so the kernel is bound
// by the vector ALU, not by LDS or cache bandwidth.
//
// Softmax.  Online, base 2, with the quadrature weight as a factor (see the
// generic kernel); the running reference maximum is only moved when a logit
// exceeds it by more than 2^8, which removes almost all accumulator rescales.
#include <cstdlib>

#include "s2_nattn_kernels.h"

namespace {

constexpr int kSeg = 128;    // outputs per wavefront
constexpr int kNTMax = 9;    // longest run of offsets handled at once
constexpr int kCG = 4;       // channels per half staged together
// Staged window geometry.  A stage holds 2*kCG channel rows (kCG per half)
// of the kSeg*PS + 8 input columns a run can touch, row-major with a pitch of
// kSeg*PS + 8 floats.  The pitch is 8 mod 16, so the two rows a lane pair reads
// (r and r + kCG) sit 32 banks apart and the b128 strip reads are conflict free.
// One global_load_lds_dword moves 64 consecutive columns of one row (lane =
// column, any alignment, wrap handled per lane).  The last 8 columns of the 8
// rows are one ordinary load (lane = row * 8 + column) written to LDS when the
// stage is consumed: LDS-direct loads with a partial exec mask proved very slow.
//
// 2:1 grids (PS = 2): runs start at a multiple of four input columns (the up to three offsets in front of
// the arc get a logit of -inf), so a window never has a 16-byte piece astride the longitude seam and one
// global_load_lds_dwordx4 (lane = four columns) copies the 256 columns of a row: a quarter of the copy
// instructions, and the copy path moves 16-byte pieces about 1.5 times faster than dwords.
template <int PS>
struct Geo {
    // PS = 2: the strips of neighbouring lane pairs start 8 floats apart; the rows of the second channel half are
    // moved up by 4 floats (pitch 8 mod 16 puts them 32 banks on, the shift makes it 36), so that the 16 lanes a
    // ds_read_b128 serves together cover the 64 banks once
    static constexpr int PITCH = PS == 2 ? 280 : kSeg * PS + 8;
    static constexpr __host__ __device__ int shift(int row) { return PS == 2 && row >= kCG ? 4 : 0; }
    static constexpr bool ALIGNED = PS == 2;                  // windows start at a multiple of 4 columns
    static constexpr int LCOLS = ALIGNED ? 4 : 1;             // columns per lane and copy instruction
    static constexpr int NFULL = kSeg * PS / (64 * LCOLS);    // full 64-lane copies per row
    static constexpr int NLOAD = 2 * kCG * NFULL + 1;         // vector-memory loads per stage
    static constexpr int TILE = 2 * kCG * PITCH;              // floats per buffer
};

// Runs of one arc of c offsets starting at offset lo.  Unaligned windows: nchunk near-equal runs of at most 9.
// Aligned windows: the first run starts at the multiple of 4 at or below lo (`lead` masked offsets), runs of
// 8, the last one of up to 9.
template <int PS>
__device__ __forceinline__ int num_runs(int c, int lo)
{
    if constexpr (Geo<PS>::ALIGNED) {
        const int span = c + (lo - (lo & ~3));
        const int n = (span + 6) >> 3;
        return n < 1 ? 1 : n;
    } else {
        return (c + kNTMax - 1) / kNTMax;
    }
}
__device__ __forceinline__ int arc_lo(int c, int nlon_in) { return c == nlon_in ? 0 : -((c - 1) >> 1); }

typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

__device__ __forceinline__ float dpp_swap_pair(float x)
{
    // lane <-> lane^1 : quad_perm [1,0,3,2]
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, true));
}

// Byte offsets (within a channel row) of the lane's column in each 64-column
// piece of the window; x0 = (first window column + lane) mod nlon_in.  The last
// entry addresses the lane's element of the 8-column tail, channel row included.
template <int PS>
__device__ __forceinline__ void stage_offsets(int x0, int xt, int nlon_in, unsigned trow,
                                              unsigned (&voff)[Geo<PS>::NFULL + 1])
{
#pragma unroll
    for (int a = 0; a < Geo<PS>::NFULL; ++a) {
        int x = x0 + 64 * Geo<PS>::LCOLS * a;
        x = x >= nlon_in ? x - nlon_in : x;
        x = x >= nlon_in ? x - nlon_in : x;
        voff[a] = 4u * unsigned(x);
    }
    int x = xt + kSeg * PS;
    x = x >= nlon_in ? x - nlon_in : x;
    x = x >= nlon_in ? x - nlon_in : x;
    voff[Geo<PS>::NFULL] = trow + 4u * unsigned(x);
}

// Start the asynchronous global -> LDS copy of one stage: kCG channel rows per
// half starting at chan0 (uniform pointer: first channel of the group for the
// even lanes, input latitude h', column 0); the odd lanes' channels lie DH rows on.
// Returns the lane's tail element (to be stored with stage_tail_store).
template <int D, int PS>
__device__ __forceinline__ float stage_issue(const float *chan0, size_t si, unsigned (&voff)[Geo<PS>::NFULL + 1],
                                             float *buf)
{
    using G = Geo<PS>;
#pragma unroll
    for (int a = 0; a <= G::NFULL; ++a) asm volatile("" : "+v"(voff[a]));   // keep 32-bit offsets, no widened copies
    // walk the channel rows with a running uniform pointer (kept opaque so that the row bases of
    // all stages are not computed up front and parked in scalar registers)
    const char *rb = reinterpret_cast<const char *>(chan0);
    asm volatile("" : "+s"(rb));
    const float tail = *reinterpret_cast<const float *>(rb + voff[G::NFULL]);
    const size_t rs = si * sizeof(float);
#pragma unroll
    for (int r = 0; r < 2 * kCG; ++r) {
#pragma unroll
        for (int a = 0; a < G::NFULL; ++a)
            if constexpr (G::LCOLS == 4)
                __builtin_amdgcn_global_load_lds((gptr_t)(rb + voff[a]), (lptr_t)(buf + r * G::PITCH + G::shift(r) + 256 * a), 16, 0, 0);
            else
                __builtin_amdgcn_global_load_lds((gptr_t)(rb + voff[a]), (lptr_t)(buf + r * G::PITCH + 64 * a), 4, 0, 0);
        rb += (r == kCG - 1) ? rs * (D / 2 - kCG + 1) : rs;
    }
    return tail;
}

template <int N>
__device__ __forceinline__ void wait_vm()
{
    // Besides the copies in flight (vmcnt) this waits for the wavefront's own LDS reads (lgkmcnt): the next
    // LDS-direct copy, issued right after this wait, goes into the buffer the previous step read its strips from, and
    // a read still queued in the LDS pipeline when that copy lands would see the new rows (seen as rare run-to-run
    // differences: 38 of 12000 launches of one small problem without the second wait, none in 12000 with it).
    if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    else if constexpr (N == 17) asm volatile("s_waitcnt vmcnt(17)" ::: "memory");
    else if constexpr (N == 33) asm volatile("s_waitcnt vmcnt(33)" ::: "memory");
    else static_assert(N == 0, "unsupported wait count");
}

// Strip of SL4 float4 for the lane's four outputs from channel row `cc` of a stage.
template <int PS, int SL4>
__device__ __forceinline__ void read_strip(const float *buf, int sbase, int cc, float (&st)[4 * SL4])
{
#pragma unroll
    for (int a = 0; a < SL4; ++a) {
        const float4 x = *reinterpret_cast<const float4 *>(buf + sbase + cc * Geo<PS>::PITCH + 4 * a);
        st[4 * a] = x.x; st[4 * a + 1] = x.y; st[4 * a + 2] = x.z; st[4 * a + 3] = x.w;
    }
}

// One run of NT offsets on one input latitude: logits, softmax update, P.V.
template <int D, int PS, int NT>
__device__ __forceinline__ void run_chunk(float *buf0, float *buf1, const float *__restrict__ kb,
                                          const float *__restrict__ vb, size_t si, int x0, int xt, unsigned trow,
                                          int taddr, int nlon_in, int sbase, float wq, int lead,
                                          const float (&q)[4][D / 2], float (&acc)[4][D / 2], float (&mref)[4],
                                          float (&lsum)[4])
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
    unsigned voff[G::NFULL + 1];
    stage_offsets<PS>(x0, xt, nlon_in, trow, voff);

    float tail = stage_issue<D, PS>(kb, si, voff, buf0);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        float *cur = (g & 1) ? buf1 : buf0, *nxt = (g & 1) ? buf0 : buf1;
        // everything in flight (this stage) must have landed before the next stage is requested: the
        // counter is waited down to zero because LDS-direct loads and ordinary loads (the tail, register
        // spills) are not guaranteed to complete in issue order relative to each other
        wait_vm<0>();
        cur[taddr] = tail;
        if (g + 1 < NG) tail = stage_issue<D, PS>(kb + size_t(g + 1) * kCG * si, si, voff, nxt);
        else tail = stage_issue<D, PS>(vb, si, voff, nxt);
#pragma unroll
        for (int cc = 0; cc < kCG; ++cc) {
            float st[4 * SL4];
            read_strip<PS, SL4>(cur, sbase, cc, st);
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
            if (G::ALIGNED && tt < 3) s[r][tt] = tt < lead ? -INFINITY : s[r][tt];   // offsets in front of the arc
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
        wait_vm<0>();
        cur[taddr] = tail;
        if (g + 1 < NG) tail = stage_issue<D, PS>(vb + size_t(g + 1) * kCG * si, si, voff, nxt);
#pragma unroll
        for (int cc = 0; cc < kCG; ++cc) {
            float st[4 * SL4];
            read_strip<PS, SL4>(cur, sbase, cc, st);
#pragma unroll
            for (int tt = 0; tt < NT; ++tt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    acc[r][g * kCG + cc] = fmaf(s[r][tt], st[r * PS + tt], acc[r][g * kCG + cc]);
        }
    }
}

constexpr int kWaves = 8;          // wavefronts per workgroup
constexpr int kState = 4 * 16 + 8; // floats of softmax state per lane: acc[4][16], mref[4], lsum[4]

// Workgroup = 8 wavefronts working on one output latitude h and one segment of
// 128 longitudes.  Output latitudes are sorted by work and grouped in four
// classes: a latitude of class P in {8, 4, 2, 1} has its list of runs split
// over P wavefronts (their partial softmax states are merged through LDS at
// the end), and the workgroup covers 8 / P different (batch, head) slices.
// Near the poles of an equiangular grid a disk holds over twenty times more
// points than at the equator; without the split those rows set the makespan.
//
// UP (upsampling, nlon_out = U * nlon_in): the output longitudes w = U*u + s of one class s see the input grid
// exactly as the outputs of an equal-grid problem do, with the arc tables of that class.  A wavefront then owns
// 128 consecutive u of one class; its q, out and lse elements lie U floats apart.
template <int D, int PS, int WAVES, bool UP = false>
__global__ void __launch_bounds__(64 * WAVES, 2)
nattn_fwd_tiled(S2DeviceTables t, int nbh, int first_row, float qscale, const float *__restrict__ q,
                const float *__restrict__ k, const float *__restrict__ v, float *__restrict__ out,
                float *__restrict__ lse)
{
    using G = Geo<PS>;
    constexpr int DH = D / 2;
    static_assert(DH == 16, "state layout assumes 16 channels per lane");
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int wave = WAVES == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform by construction
    const int lane = threadIdx.x & 63;
    float *buf0 = smem + wave * 2 * G::TILE, *buf1 = buf0 + G::TILE;

    static_assert(!UP || PS == 1, "class view of an upsampling grid is an equal-grid problem");
    const int U = UP ? t.upscale : 1;
    const int nlon_v = UP ? t.nlon_in : t.nlon_out;       // outputs per class
    const int nseg = ((nlon_v + kSeg - 1) / kSeg) * U;
    int P, seg, h, part, bh;
    if constexpr (WAVES == 1) {
        // one wavefront per workgroup, no split: block -> (latitude by work, slice, segment)
        int id = blockIdx.x;
        seg = id % nseg; id /= nseg;
        bh = id % nbh;
        h = t.row_order[first_row + id / nbh];
        P = 1; part = 0;
    } else {
        // block -> (group of 8 (batch, head) slices, class, output latitude, segment, slices of the group).
        // Slices are the outer loop: the K/V of 8 slices (tens of MB) stay resident in the 256 MB
        // last-level cache while all their latitudes are processed; heavy latitudes come first in a group.
        const int per_group = nseg * (8 * t.fwd_cls[0] + 4 * t.fwd_cls[1] + 2 * t.fwd_cls[2] + (first_row ? 0 : t.fwd_cls[3]));
        const int grp8 = blockIdx.x / per_group;
        int id = blockIdx.x - grp8 * per_group, rows_before = 0;
        P = WAVES;
#pragma unroll
        for (int cls = 0; cls < 3; ++cls) {
            const int Pc = WAVES >> cls;
            const int nblk_c = t.fwd_cls[cls] * nseg * Pc;
            if (P == Pc && id >= nblk_c) { id -= nblk_c; rows_before += t.fwd_cls[cls]; P = Pc >> 1; }
        }
        // within a class: P blocks per (latitude, segment), each covering 8 / P slices
        const int tpb = WAVES / P;
        const int sub = id % P; id /= P;
        seg = id % nseg;
        h = t.row_order[rows_before + id / nseg];
        part = wave & (P - 1);
        bh = grp8 * WAVES + sub * tpb + wave / P;
    }
    const bool wave_active = bh < nbh;

    const int p = lane >> 1, half = lane & 1;
    const int sc = UP ? seg % U : 0;                      // class of the outputs of this workgroup
    if constexpr (UP) seg /= U;
    const int w0 = seg * kSeg + 4 * p;
    const bool active = wave_active && w0 < nlon_v;       // nlon_v is a multiple of 4: all four outputs or none

    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t io = size_t(h) * t.nlon_out + (UP ? w0 * U + sc : w0);
    const int *ctab = (UP ? t.ucnt + size_t(h * U + sc) * t.band_max : t.cnt + size_t(h) * t.band_max);
    const int *ltab = UP ? t.ulo + size_t(h * U + sc) * t.band_max : nullptr;
    // strip base (floats) in a staged buffer: the lane's channel rows start at half*kCG, its columns at 4*p*PS
    const int sbase = half * kCG * G::PITCH + G::shift(half * kCG) + 4 * p * PS;
    // window tail: lane = (channel row, one of the last 8 columns)
    const int trl = lane >> 3;
    const unsigned trow = unsigned((trl < kCG ? trl : trl - kCG + DH) * si * sizeof(float));
    const int taddr = trl * G::PITCH + G::shift(trl) + kSeg * PS + (lane & 7);
    float qr[4][DH], acc[4][DH], mref[4], lsum[4];
#pragma unroll
    for (int c = 0; c < DH; ++c) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (UP) {
            if (active) {
                const float *qp = q + (size_t(bh) * D + half * DH + c) * so + io;
                x = make_float4(qp[0], qp[U], qp[2 * U], qp[3 * U]);
            }
        } else {
            if (active) x = *reinterpret_cast<const float4 *>(q + (size_t(bh) * D + half * DH + c) * so + io);
        }
        qr[0][c] = x.x * qscale; qr[1][c] = x.y * qscale; qr[2][c] = x.z * qscale; qr[3][c] = x.w * qscale;
        acc[0][c] = acc[1][c] = acc[2][c] = acc[3][c] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) { mref[r] = -INFINITY; lsum[r] = 0.f; }

    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    // This wavefront's share of the runs of latitude h: every P-th run.  The P wavefronts then work on neighbouring
    // runs of the same input latitude at the same time, whose windows overlap almost entirely, so a row is fetched
    // into the L2 once and staged from there (with contiguous shares each wavefront walked its own band rows and the
    // workgroup kept eight rows alive).
    int run = 0;
    if (wave_active) {
        // Band rows are visited in a rotated order: first the one whose absolute latitude index is 0 modulo
        // the band size, and so on.  Workgroups of neighbouring latitudes run at the same time and advance at
        // the same pace; with this order they all want the SAME input latitudes at the same moment (one
        // ninth of the slice instead of all of it), so the re-reads hit the 4 MB L2 of the XCD instead of
        // streaming the slice from memory nine times.
        const int rot = (t.band_max - hp0 % t.band_max) % t.band_max % nb;
        for (int bb = 0; bb < nb; ++bb) {
            const int b = bb + rot < nb ? bb + rot : bb + rot - nb;
            const int hp = hp0 + b;
            const int c = ctab[b];
            if (UP && c == 0) continue;                     // this class misses the latitude
            const int lo = UP && c != t.nlon_in ? ltab[b] : arc_lo(c, t.nlon_in);
            const int nchunk = num_runs<PS>(c, lo);
            if (((part - run) & (P - 1)) >= nchunk) { run += nchunk; continue; }   // none of these runs is mine
            const float wq = t.omega_rel[hp];
            const float *kb = k + size_t(bh) * D * si + size_t(hp) * t.nlon_in;
            const float *vb = v + size_t(bh) * D * si + size_t(hp) * t.nlon_in;
            const int base = c / nchunk, rem = c - base * nchunk;
            const int lead0 = G::ALIGNED ? lo - (lo & ~3) : 0, span = c + lead0;
            int t0 = -lead0;
            for (int ci = 0; ci < nchunk; ++ci, ++run) {
                const int nt = G::ALIGNED ? (ci == nchunk - 1 ? span - 8 * ci : 8) : base + (ci < rem ? 1 : 0);
                const int lead = ci == 0 ? lead0 : 0;
                if ((run & (P - 1)) == part) {
                    int xw = seg * kSeg * PS + lo + t0 + 2 * t.nlon_in;      // first window column
                    xw = xw >= t.nlon_in ? xw - t.nlon_in : xw;
                    xw = xw >= t.nlon_in ? xw - t.nlon_in : xw;
                    xw = xw >= t.nlon_in ? xw - t.nlon_in : xw;
                    int x0 = xw + G::LCOLS * lane, xt = xw + (lane & 7);
                    x0 = x0 >= t.nlon_in ? x0 - t.nlon_in : x0;
                    xt = xt >= t.nlon_in ? xt - t.nlon_in : xt;
#define S2_RUN(N) case N: run_chunk<D, PS, N>(buf0, buf1, kb, vb, si, x0, xt, trow, taddr, t.nlon_in, sbase, wq, lead, qr, acc, mref, lsum); break;
                    switch (nt) {
                        S2_RUN(1) S2_RUN(2) S2_RUN(3) S2_RUN(4) S2_RUN(5) S2_RUN(6)
                        S2_RUN(7) S2_RUN(8) S2_RUN(9)
                    }
#undef S2_RUN
                }
                t0 += nt;
            }
        }
    }

    // merge the P partial states pairwise through LDS (the staging buffers are free now)
    if (P > 1) {
        __syncthreads();
        for (int s = 1; s < P; s <<= 1) {
            float *slot = smem + (wave / (2 * s)) * (kState * 64) + lane;
            if ((part & (2 * s - 1)) == s) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
#pragma unroll
                    for (int c = 0; c < DH; ++c) slot[(r * DH + c) * 64] = acc[r][c];
                    slot[(64 + r) * 64] = mref[r];
                    slot[(68 + r) * 64] = lsum[r];
                }
            }
            __syncthreads();
            if ((part & (2 * s - 1)) == 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float mo = slot[(64 + r) * 64], lo2 = slot[(68 + r) * 64];
                    const float M = fmaxf(mref[r], mo);
                    // a part that saw no run has m = -inf, l = 0: its factor must be 0, never NaN
                    const float fa = mref[r] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mref[r] - M);
                    const float fb = mo == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mo - M);
                    mref[r] = M;
                    lsum[r] = lsum[r] * fa + lo2 * fb;
#pragma unroll
                    for (int c = 0; c < DH; ++c) acc[r][c] = acc[r][c] * fa + slot[(r * DH + c) * 64] * fb;
                }
            }
            __syncthreads();
        }
    }
    if (!active || part != 0) return;
    float inv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) inv[r] = 1.f / lsum[r];
#pragma unroll
    for (int c = 0; c < DH; ++c) {
        float *op = out + (size_t(bh) * D + half * DH + c) * so + io;
        if constexpr (UP) {
#pragma unroll
            for (int r = 0; r < 4; ++r) op[r * U] = acc[r][c] * inv[r];
        } else {
            *reinterpret_cast<float4 *>(op) =
                make_float4(acc[0][c] * inv[0], acc[1][c] * inv[1], acc[2][c] * inv[2], acc[3][c] * inv[3]);
        }
    }
    if (half == 0) {
        float L[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) L[r] = (mref[r] + log2f(lsum[r] * t.omega_ref)) * 0.6931471805599453f;
        if constexpr (UP) {
#pragma unroll
            for (int r = 0; r < 4; ++r) lse[size_t(bh) * so + io + r * U] = L[r];
        } else {
            *reinterpret_cast<float4 *>(lse + size_t(bh) * so + io) = make_float4(L[0], L[1], L[2], L[3]);
        }
    }
}

// dynamic LDS of the 8-wave kernel: the wavefronts' staging buffers, reused for the merge of their softmax states
template <int PS>
constexpr size_t fwd_tiled_lds()
{
    constexpr size_t stage_fl = size_t(kWaves) * 2 * Geo<PS>::TILE, merge_fl = size_t(kWaves / 2) * kState * 64;
    return (stage_fl > merge_fl ? stage_fl : merge_fl) * sizeof(float);
}

template <int D, int PS, bool UP = false>
int launch_fwd_tiled(const S2DeviceTables &t, int skip_rows, int nbh, float qscale, const float *q, const float *k,
                     const float *v, float *out, float *lse, hipStream_t st)
{   // t.row_order already points past the skip_rows latitudes another kernel has taken
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    const int nseg = UP ? ((t.nlon_in + kSeg - 1) / kSeg) * t.upscale : (t.nlon_out + kSeg - 1) / kSeg;
    const int nsplit = t.fwd_cls[0] + t.fwd_cls[1] + t.fwd_cls[2];   // latitudes split over several wavefronts
    constexpr int mode = 0;   // 1: everything through the one-wave kernel, 2: everything through the 8-wave kernel
    // heavy latitudes: 8-wave workgroups with an in-LDS merge
    if (mode != 1 && (nsplit > 0 || mode == 2)) {
        const int first_row = mode == 2 ? 0 : 1;   // mode 2: every latitude through the 8-wave kernel
        const long nblk = long((nbh + kWaves - 1) / kWaves) * nseg *
                          (8 * t.fwd_cls[0] + 4 * t.fwd_cls[1] + 2 * t.fwd_cls[2] + (first_row ? 0 : t.fwd_cls[3]));
        const size_t lds = fwd_tiled_lds<PS>();
        auto kern = nattn_fwd_tiled<D, PS, kWaves, UP>;
        S2TraceScope tr("nattn_fwd_tiled<8 waves>",
                        nbh * (t.fwd_pairs[0] + t.fwd_pairs[1] + t.fwd_pairs[2] + (first_row ? 0.0 : t.fwd_pairs[3])), st);
        hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(64 * kWaves), lds, st, t, nbh, first_row, qscale, q, k, v,
                           out, lse);
        if (mode == 2) return 0;
    }
    // the rest: one wavefront per workgroup
    const int first_row = mode == 1 ? 0 : nsplit;
    const long nrows = t.nlat_out - skip_rows - first_row;
    const bool no_stream = s2_debug_flag(S2_DEBUG_NO_STREAM);   // test-only: one-wave kernel instead
    if (!UP && nrows > 0 && mode == 0 && !no_stream && s2_nattn_stream_supported(t, D, D))
        return s2_nattn_fwd_stream(t, nbh, qscale, q, k, v, out, lse, st);
    if (nrows > 0) {
        S2TraceScope tr("nattn_fwd_tiled<1 wave>",
                        nbh * (t.fwd_pairs[3] + (mode == 1 ? t.fwd_pairs[0] + t.fwd_pairs[1] + t.fwd_pairs[2] : 0.0)), st);
        hipLaunchKernelGGL((nattn_fwd_tiled<D, PS, 1, UP>), dim3((unsigned)(nrows * nbh * nseg)), dim3(64),
                           2 * Geo<PS>::TILE * sizeof(float), st, t, nbh, first_row, qscale, q, k, v, out, lse);
    }
    return 0;
}

}  // namespace

int s2_nattn_tiled_configure()
{
    auto raise = [](auto kern, size_t lds) {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   int(lds)) == hipSuccess;
    };
    return raise(nattn_fwd_tiled<32, 1, kWaves, false>, fwd_tiled_lds<1>()) &&
           raise(nattn_fwd_tiled<32, 2, kWaves, false>, fwd_tiled_lds<2>()) &&
           raise(nattn_fwd_tiled<32, 1, kWaves, true>, fwd_tiled_lds<1>()) ? 0 : -1;
}

bool s2_nattn_fwd_tiled_supported(const S2DeviceTables &t, int d, int e)
{
    if (t.upscale > 1) return d == 32 && e == 32 && t.nlon_in % 4 == 0 && t.nlon_in >= 72;
    return d == 32 && e == 32 && (t.pscale == 1 || t.pscale == 2) && t.nlon_in % 4 == 0 && t.nlon_out % 4 == 0 &&
           t.nlon_out >= 72;   // (window wrap logic handles at most two turns of the circle)
}

int s2_nattn_fwd_tiled(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q, const float *k,
                       const float *v, float *out, float *lse, hipStream_t st)
{
    const float qscale = scale * 1.4426950408889634f;
    if (t.upscale > 1) {
        // upsampling: every class of output longitudes is an equal-grid problem for the split vector kernels
        S2DeviceTables tu = t;
        s2_pick_split(tu, true, nbh, ((t.nlon_in + kSeg - 1) / kSeg) * t.upscale, false);
        return launch_fwd_tiled<32, 1, true>(tu, 0, nbh, qscale, q, k, v, out, lse, st);
    }
    // dense polar latitudes go to the matrix-core kernel; the vector kernels see the remaining latitudes
    S2DeviceTables tv = t;
    const int nm = s2_nattn_fwd_mfma_rows(t, d, e);
    if (nm > 0) {
        if (s2_nattn_fwd_mfma(t, nbh, nm, scale, q, k, v, out, lse, st)) return -1;
        tv.row_order = t.row_order + nm;
    }
    if (s2_nattn_stream_supported(t, d, e)) {
        if (nm > 0) {
            tv.fwd_cls[0] = tv.fwd_cls[1] = tv.fwd_cls[2] = 0;
            tv.fwd_pairs[0] = tv.fwd_pairs[1] = tv.fwd_pairs[2] = 0.0;
        }
    } else {
        s2_pick_split(tv, true, nbh, (t.nlon_out + kSeg - 1) / kSeg, nm > 0);
    }
    if (t.pscale == 1) return launch_fwd_tiled<32, 1>(tv, nm, nbh, qscale, q, k, v, out, lse, st);
    return launch_fwd_tiled<32, 2>(tv, nm, nbh, qscale, q, k, v, out, lse, st);
}
