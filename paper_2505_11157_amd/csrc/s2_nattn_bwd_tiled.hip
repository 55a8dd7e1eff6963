// Tuned float32 backward kernels for spherical neighborhood attention on gfx950
// (App. B.4 with the typos of the derivation fixed):
//   p_ij = omega_j exp(s_ij - lse_i),  D_i = dout_i . out_i,  dS_ij = p_ij (dout_i . v_j - D_i)
//   dq_i = scale sum_j dS_ij k_j ;  dk_j = scale sum_i dS_ij q_i ;  dv_j = sum_i p_ij dout_i
//
// Same data path as the tuned forward kernel (runs of <= 9 longitude offsets on
// one latitude, windows staged with LDS-direct loads, one aligned b128 strip
// per channel reused from registers), with a different register budget: the
// backward keeps three (dq) or four (dk/dv) per-point vectors live, so FOUR
// adjacent lanes share four consecutive points and each carries 8 of the 32
// channels; partial dot products are combined with two DPP adds.  A wavefront
// owns 64 consecutive longitudes.
//
//   dq kernel   : owners are output points; K, V windows stream by
//                 (s = q.K, dP = dout.V, then dq += dS K).  Also stores D_i.
//   dk/dv kernel: owners are INPUT points (transposed neighborhood: by symmetry
//                 of the distance, input (h', w) lies in the disks of outputs
//                 (h, w + t), |t| <= half-arc(h, h')); q, dout windows stream by
//                 together with the lse and D rows.  Equal grids only.
// No atomics anywhere; heavy latitudes are split over the wavefronts of a
// workgroup and summed through LDS, as in the forward kernel.
#include <cstdlib>

#include "s2_nattn_kernels.h"

namespace {

constexpr int kSegB = 64;    // points per wavefront
constexpr int kNTMax = 9;    // longest run of offsets handled at once
constexpr int kCGB = 4;      // channels per lane staged together
constexpr int kRows = 16;    // channel rows per stage: 4 lanes x kCGB
constexpr int kDL = 8;       // channels per lane (head dimension 32)
constexpr int kWavesB = 8;
constexpr float kLog2e = 1.4426950408889634f;

// Row-major staged window of kRows channel rows x (64*PS + 8) columns.  PS = 1: the
// pitch is 4 mod 16: the four rows a lane quad reads (r, r+4, r+8, r+12) start
// 16 banks apart, so 4 quads x 4 lanes x b128 cover the 64 banks exactly once.
// PS = 2: the strips of neighbouring quads start 8 floats apart, so the rows of the four lane quarters must start
// at banks 0, 32, 4, 36: pitch 8 mod 16 (quarters 32 banks apart) and the rows of quarters 2 and 3 moved up by 4 floats.
template <int PS>
struct GeoB {
    static constexpr int PITCH = PS == 1 ? 84 : 152;
    static constexpr __host__ __device__ int shift(int row) { return PS == 2 && row >= 8 ? 4 : 0; }
    static constexpr int NFULL = PS;                       // full 64-column loads per row
    static constexpr int NLOAD = kRows * NFULL + 2;        // vector-memory loads per stage (2 = tail)
    static constexpr int TILE = kRows * PITCH;
    static_assert(PITCH >= 64 * PS + 8 + 4, "pitch too small");
};

typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

__device__ __forceinline__ float quad_sum(float x)
{
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, true));
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, true));
    return x;
}

__device__ __forceinline__ int wrap2(int x, int n)
{
    x = x >= n ? x - n : x;
    return x >= n ? x - n : x;
}

// channel (relative to the group's first channel) held by stage row r: lane quarter r/4 owns channels 8*(r/4)..+7
__device__ __forceinline__ int chan_of_row(int r) { return (r >> 2) * kDL + (r & 3); }

struct StageOff {
    unsigned full[2];   // byte offset of the lane's column in each 64-column piece
    unsigned tail[2];   // byte offsets (channel row included) of the lane's two tail elements
};

// xw = first window column (already in [0, ncol)), ncol = longitudes of the streamed grid
// Window column x of the streamed row lies at float x * cmul + cadd of that row (1, 0 except for the class view of
// an upsampling grid, where the outputs of one class are cmul floats apart).
template <int PS>
__device__ __forceinline__ StageOff stage_offsets(int xw, int ncol, size_t sstride, int lane, int cmul = 1, int cadd = 0)
{
    StageOff o;
#pragma unroll
    for (int a = 0; a < 2; ++a) o.full[a] = 4u * unsigned(wrap2(xw + lane + 64 * a, ncol) * cmul + cadd);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int e = lane + 64 * u, row = e >> 3, col = e & 7;
        o.tail[u] = unsigned(chan_of_row(row) * sstride * sizeof(float)) +
                    4u * unsigned(wrap2(xw + 64 * PS + col, ncol) * cmul + cadd);
    }
    return o;
}

// Start the asynchronous copy of one stage (kRows channel rows starting at the
// uniform pointer chan0: channel g*kCGB of lane quarter 0, streamed latitude, column 0).
template <int PS>
__device__ __forceinline__ void stage_issue(const float *chan0, size_t sstride, StageOff &o, float *buf, float (&tail)[2])
{
    using G = GeoB<PS>;
#pragma unroll
    for (int a = 0; a < 2; ++a) { asm volatile("" : "+v"(o.full[a])); asm volatile("" : "+v"(o.tail[a])); }
    const char *rb = reinterpret_cast<const char *>(chan0);
    asm volatile("" : "+s"(rb));
    tail[0] = *reinterpret_cast<const float *>(rb + o.tail[0]);
    tail[1] = *reinterpret_cast<const float *>(rb + o.tail[1]);
    const size_t rs = sstride * sizeof(float);
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
#pragma unroll
        for (int a = 0; a < G::NFULL; ++a)
            __builtin_amdgcn_global_load_lds((gptr_t)(rb + o.full[a]), (lptr_t)(buf + r * G::PITCH + G::shift(r) + 64 * a), 4, 0, 0);
        rb += ((r & 3) == 3) ? rs * (kDL - kCGB + 1) : rs;
    }
}

template <int N>
__device__ __forceinline__ void wait_vm()
{
    // Besides the copies in flight (vmcnt) this waits for the wavefront's own LDS reads (lgkmcnt): the next
    // LDS-direct copy, issued right after this wait, goes into the buffer the previous step read its strips from, and
    // a read still queued in the LDS pipeline when that copy lands would see the new rows (seen as rare run-to-run
    // differences: 38 of 12000 launches of one small problem without the second wait, none in 12000 with it).
    if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    else if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if constexpr (N == 18) asm volatile("s_waitcnt vmcnt(18)" ::: "memory");
    else if constexpr (N == 34) asm volatile("s_waitcnt vmcnt(34)" ::: "memory");
    else static_assert(N == 0, "unsupported wait count");
}

template <int PS>
__device__ __forceinline__ void tail_store(float *buf, const int (&taddr)[2], const float (&tail)[2])
{
    buf[taddr[0]] = tail[0];
    buf[taddr[1]] = tail[1];
}

template <int PS, int SL4>
__device__ __forceinline__ void read_strip(const float *buf, int sbase, int cc, float (&st)[4 * SL4])
{
#pragma unroll
    for (int a = 0; a < SL4; ++a) {
        const float4 x = *reinterpret_cast<const float4 *>(buf + sbase + cc * GeoB<PS>::PITCH + 4 * a);
        st[4 * a] = x.x; st[4 * a + 1] = x.y; st[4 * a + 2] = x.z; st[4 * a + 3] = x.w;
    }
}

// acc[r][t] += own[r][c0 + cc] * window(r, t) over the kCGB channels of one stage
template <int PS, int NT>
__device__ __forceinline__ void dot_stage(const float *buf, int sbase, const float (&own)[4][kDL], int c0, float (&acc)[4][NT])
{
    constexpr int SL4 = (3 * PS + NT + 3) / 4;
#pragma unroll
    for (int cc = 0; cc < kCGB; ++cc) {
        float st[4 * SL4];
        read_strip<PS, SL4>(buf, sbase, cc, st);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r][tt] = fmaf(own[r][c0 + cc], st[r * PS + tt], acc[r][tt]);
    }
}

// out[r][c0 + cc] += sum_t w[r][t] * window(r, t)
template <int PS, int NT>
__device__ __forceinline__ void axpy_stage(const float *buf, int sbase, const float (&w)[4][NT], int c0, float (&out)[4][kDL])
{
    constexpr int SL4 = (3 * PS + NT + 3) / 4;
#pragma unroll
    for (int cc = 0; cc < kCGB; ++cc) {
        float st[4 * SL4];
        read_strip<PS, SL4>(buf, sbase, cc, st);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) out[r][c0 + cc] = fmaf(w[r][tt], st[r * PS + tt], out[r][c0 + cc]);
    }
}

// Per-lane addressing shared by both kernels.
struct LaneGeo {
    int sbase;       // strip base (floats) in a staged buffer
    int taddr[2];    // LDS addresses (floats) of the lane's two tail elements
};

template <int PS>
__device__ __forceinline__ LaneGeo lane_geo(int lane)
{
    using G = GeoB<PS>;
    LaneGeo g;
    g.sbase = (lane & 3) * kCGB * G::PITCH + G::shift((lane & 3) * kCGB) + 4 * (lane >> 2) * PS;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int e = lane + 64 * u;
        g.taddr[u] = (e >> 3) * G::PITCH + G::shift(e >> 3) + 64 * PS + (e & 7);
    }
    return g;
}

// ---------------------------------------------------------------- dq ----------

template <int PS, int NT>
__device__ __forceinline__ void run_chunk_dq(float *buf0, float *buf1, const float *__restrict__ kb,
                                             const float *__restrict__ vb, size_t si, int xw, int nlon_in, int lane,
                                             const LaneGeo &lg, float wq, const float (&q)[4][kDL],
                                             const float (&go)[4][kDL], const float (&lse2)[4], const float (&Dr)[4],
                                             float (&dq)[4][kDL])
{
    float s[4][NT], dp[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) { s[r][tt] = 0.f; dp[r][tt] = 0.f; }
    StageOff so = stage_offsets<PS>(xw, nlon_in, si, lane);
    float ta[2], tb[2];
    const float *k1 = kb + size_t(kCGB) * si, *v1 = vb + size_t(kCGB) * si;

    stage_issue<PS>(kb, si, so, buf0, ta);
    // s = q . K
    wait_vm<0>(); tail_store<PS>(buf0, lg.taddr, ta);
    stage_issue<PS>(k1, si, so, buf1, tb);
    dot_stage<PS, NT>(buf0, lg.sbase, q, 0, s);
    wait_vm<0>(); tail_store<PS>(buf1, lg.taddr, tb);
    stage_issue<PS>(vb, si, so, buf0, ta);
    dot_stage<PS, NT>(buf1, lg.sbase, q, kCGB, s);
    // dP = dout . V
    wait_vm<0>(); tail_store<PS>(buf0, lg.taddr, ta);
    stage_issue<PS>(v1, si, so, buf1, tb);
    dot_stage<PS, NT>(buf0, lg.sbase, go, 0, dp);
    wait_vm<0>(); tail_store<PS>(buf1, lg.taddr, tb);
    stage_issue<PS>(kb, si, so, buf0, ta);
    dot_stage<PS, NT>(buf1, lg.sbase, go, kCGB, dp);
    // dS = p (dP - D)
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            const float sv = quad_sum(s[r][tt]), dv = quad_sum(dp[r][tt]);
            s[r][tt] = wq * __builtin_amdgcn_exp2f(sv - lse2[r]) * (dv - Dr[r]);
        }
    // dq += dS K
    wait_vm<0>(); tail_store<PS>(buf0, lg.taddr, ta);
    stage_issue<PS>(k1, si, so, buf1, tb);
    axpy_stage<PS, NT>(buf0, lg.sbase, s, 0, dq);
    wait_vm<0>(); tail_store<PS>(buf1, lg.taddr, tb);
    axpy_stage<PS, NT>(buf1, lg.sbase, s, kCGB, dq);
}

// Decode a workgroup into (latitude, segment, slice, part): same scheme as the forward kernel.
struct Task { int P, seg, row, part, bh; };

template <int WAVES>
__device__ __forceinline__ Task decode_task(const int (&cls)[4], const int *order, int nseg, int nbh, int first_row,
                                            int wave)
{
    Task t;
    if constexpr (WAVES == 1) {
        int id = blockIdx.x;
        t.seg = id % nseg; id /= nseg;
        t.bh = id % nbh;
        t.row = order[first_row + id / nbh];
        t.P = 1; t.part = 0;
    } else {
        const int per_group = nseg * (8 * cls[0] + 4 * cls[1] + 2 * cls[2] + (first_row ? 0 : cls[3]));
        const int grp8 = blockIdx.x / per_group;
        int id = blockIdx.x - grp8 * per_group, rows_before = 0;
        int P = WAVES;
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            const int Pc = WAVES >> c;
            const int nblk_c = cls[c] * nseg * Pc;
            if (P == Pc && id >= nblk_c) { id -= nblk_c; rows_before += cls[c]; P = Pc >> 1; }
        }
        const int tpb = WAVES / P;
        const int sub = id % P; id /= P;
        t.seg = id % nseg;
        t.row = order[rows_before + id / nseg];
        t.part = wave & (P - 1);
        t.bh = grp8 * WAVES + sub * tpb + wave / P;
        t.P = P;
    }
    return t;
}

// Sum NV per-lane vectors of 4 x kDL floats over the P wavefronts of a task (pairwise through LDS).
template <int NV>
__device__ __forceinline__ void merge_sum(float *smem, int wave, int lane, int P, int part, float (&a)[4][kDL],
                                          float (&b)[4][kDL])
{
    __syncthreads();
    for (int s = 1; s < P; s <<= 1) {
        float *slot = smem + (wave / (2 * s)) * (NV * 4 * kDL * 64) + lane;
        if ((part & (2 * s - 1)) == s) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < kDL; ++c) {
                    slot[(r * kDL + c) * 64] = a[r][c];
                    if (NV == 2) slot[(4 * kDL + r * kDL + c) * 64] = b[r][c];
                }
        }
        __syncthreads();
        if ((part & (2 * s - 1)) == 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < kDL; ++c) {
                    a[r][c] += slot[(r * kDL + c) * 64];
                    if (NV == 2) b[r][c] += slot[(4 * kDL + r * kDL + c) * 64];
                }
        }
        __syncthreads();
    }
}

// UP: class view of an upsampling grid (see the forward kernel): owners are the outputs w = U*u + s of one class.
template <int PS, int WAVES, bool UP = false>
__global__ void __launch_bounds__(64 * WAVES, 2)
nattn_bwd_dq_tiled(S2DeviceTables t, int nbh, int first_row, float scale, const float *__restrict__ q,
                   const float *__restrict__ k, const float *__restrict__ v, const float *__restrict__ o,
                   const float *__restrict__ lse, const float *__restrict__ go, float *__restrict__ dq,
                   float *__restrict__ Dws)
{
    using G = GeoB<PS>;
    constexpr int D = 4 * kDL;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int wave = WAVES == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    float *buf0 = smem + wave * 2 * G::TILE, *buf1 = buf0 + G::TILE;
    static_assert(!UP || PS == 1, "class view of an upsampling grid is an equal-grid problem");
    const int U = UP ? t.upscale : 1;
    const int nlon_v = UP ? t.nlon_in : t.nlon_out;       // outputs per class
    const int nseg = ((nlon_v + kSegB - 1) / kSegB) * U;
    const Task tk = decode_task<WAVES>(t.fwd_cls, t.row_order, nseg, nbh, first_row, wave);
    const int h = tk.row, bh = tk.bh;
    const bool wave_active = bh < nbh;
    const int qd = lane & 3;
    const int sc = UP ? tk.seg % U : 0, seg = UP ? tk.seg / U : tk.seg;
    const int w0 = seg * kSegB + 4 * (lane >> 2);
    const bool active = wave_active && w0 < nlon_v;
    const LaneGeo lg = lane_geo<PS>(lane);
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t io = size_t(h) * t.nlon_out + (UP ? w0 * U + sc : w0);
    const int *ctab = (UP ? t.ucnt + size_t(h * U + sc) * t.band_max : t.cnt + size_t(h) * t.band_max);
    const int *ltab = UP ? t.ulo + size_t(h * U + sc) * t.band_max : nullptr;
    const float qscale = scale * kLog2e;

    float qr[4][kDL], gr[4][kDL], dqa[4][kDL], lse2[4], Dr[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < kDL; ++c) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x, z = x;
        if (active) {
            const size_t off = (size_t(bh) * D + qd * kDL + c) * so + io;
            if constexpr (UP) {
                x = make_float4(q[off], q[off + U], q[off + 2 * U], q[off + 3 * U]);
                y = make_float4(go[off], go[off + U], go[off + 2 * U], go[off + 3 * U]);
                z = make_float4(o[off], o[off + U], o[off + 2 * U], o[off + 3 * U]);
            } else {
                x = *reinterpret_cast<const float4 *>(q + off);
                y = *reinterpret_cast<const float4 *>(go + off);
                z = *reinterpret_cast<const float4 *>(o + off);
            }
        }
        qr[0][c] = x.x * qscale; qr[1][c] = x.y * qscale; qr[2][c] = x.z * qscale; qr[3][c] = x.w * qscale;
        gr[0][c] = y.x; gr[1][c] = y.y; gr[2][c] = y.z; gr[3][c] = y.w;
        Dr[0] = fmaf(y.x, z.x, Dr[0]); Dr[1] = fmaf(y.y, z.y, Dr[1]);
        Dr[2] = fmaf(y.z, z.z, Dr[2]); Dr[3] = fmaf(y.w, z.w, Dr[3]);
        dqa[0][c] = dqa[1][c] = dqa[2][c] = dqa[3][c] = 0.f;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) Dr[r] = quad_sum(Dr[r]);
    {
        float4 L = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (UP) {
            const float *lp = lse + size_t(bh) * so + io;
            if (active) L = make_float4(lp[0], lp[U], lp[2 * U], lp[3 * U]);
        } else {
            if (active) L = *reinterpret_cast<const float4 *>(lse + size_t(bh) * so + io);
        }
        lse2[0] = (L.x - t.ln_omega_ref) * kLog2e; lse2[1] = (L.y - t.ln_omega_ref) * kLog2e;
        lse2[2] = (L.z - t.ln_omega_ref) * kLog2e; lse2[3] = (L.w - t.ln_omega_ref) * kLog2e;
        if (active && qd == 0 && tk.part == 0) {
            if constexpr (UP) {
#pragma unroll
                for (int r = 0; r < 4; ++r) Dws[size_t(bh) * so + io + r * U] = Dr[r];
            } else {
                *reinterpret_cast<float4 *>(Dws + size_t(bh) * so + io) = make_float4(Dr[0], Dr[1], Dr[2], Dr[3]);
            }
        }
    }

    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    int run = 0;   // runs are dealt out to the P wavefronts of a task in turn (see the forward kernel)
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
            const int nchunk = (c + kNTMax - 1) / kNTMax;
            if (((tk.part - run) & (tk.P - 1)) >= nchunk) { run += nchunk; continue; }   // none of these runs is mine
            const int lo = (c == t.nlon_in) ? 0 : UP ? ltab[b] : -((c - 1) >> 1);
            const float wq = t.omega_rel[hp];
            const float *kb = k + size_t(bh) * D * si + size_t(hp) * t.nlon_in;
            const float *vb = v + size_t(bh) * D * si + size_t(hp) * t.nlon_in;
            const int base = c / nchunk, rem = c - base * nchunk;
            int t0 = 0;
            for (int ci = 0; ci < nchunk; ++ci, ++run) {
                const int nt = base + (ci < rem ? 1 : 0);
                if ((run & (tk.P - 1)) == tk.part) {
                    const int xw = wrap2(seg * kSegB * PS + lo + t0 + t.nlon_in, t.nlon_in);
#define S2_RUN(N) case N: run_chunk_dq<PS, N>(buf0, buf1, kb, vb, si, xw, t.nlon_in, lane, lg, wq, qr, gr, lse2, Dr, dqa); break;
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
    if (WAVES > 1 && tk.P > 1) merge_sum<1>(smem, wave, lane, tk.P, tk.part, dqa, dqa);
    if (!active || tk.part != 0) return;
#pragma unroll
    for (int c = 0; c < kDL; ++c) {
        float *dp = dq + (size_t(bh) * D + qd * kDL + c) * so + io;
        if constexpr (UP) {
#pragma unroll
            for (int r = 0; r < 4; ++r) dp[r * U] = dqa[r][c] * scale;
        } else {
            *reinterpret_cast<float4 *>(dp) =
                make_float4(dqa[0][c] * scale, dqa[1][c] * scale, dqa[2][c] * scale, dqa[3][c] * scale);
        }
    }
}

// -------------------------------------------------------------- dk, dv ----------

template <int NT>
__device__ __forceinline__ void run_chunk_dkdv(float *buf0, float *buf1, float *aux, const float *__restrict__ qb,
                                               const float *__restrict__ gb, const float *__restrict__ lrow,
                                               const float *__restrict__ drow, size_t so, int xw, int nlon, int lane,
                                               const LaneGeo &lg, float wq, float lref2, const float (&kr)[4][kDL],
                                               const float (&vr)[4][kDL], float (&dk)[4][kDL], float (&dv)[4][kDL],
                                               int cmul = 1, int cadd = 0)
{
    using G = GeoB<1>;
    float s[4][NT], dp[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) { s[r][tt] = 0.f; dp[r][tt] = 0.f; }
    StageOff of = stage_offsets<1>(xw, nlon, so, lane, cmul, cadd);
    // lse and D rows of the window: 64 columns by LDS-direct load, the last 8 by an ordinary load
    // (every lane fetches one of the 16 tail elements; duplicates store the same value)
    __builtin_amdgcn_global_load_lds((gptr_t)(reinterpret_cast<const char *>(lrow) + of.full[0]), (lptr_t)aux, 4, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr_t)(reinterpret_cast<const char *>(drow) + of.full[0]),
                                     (lptr_t)(aux + G::PITCH), 4, 0, 0);
    const int acol = wrap2(xw + 64 + (lane & 7), nlon) * cmul + cadd;
    const float atail = ((lane >> 3) & 1) ? drow[acol] : lrow[acol];
    float ta[2], tb[2];
    const float *q1 = qb + size_t(kCGB) * so, *g1 = gb + size_t(kCGB) * so;

    stage_issue<1>(qb, so, of, buf0, ta);
    // s = k . Q
    wait_vm<0>(); tail_store<1>(buf0, lg.taddr, ta);
    stage_issue<1>(q1, so, of, buf1, tb);
    aux[((lane >> 3) & 1) * G::PITCH + 64 + (lane & 7)] = atail;
    dot_stage<1, NT>(buf0, lg.sbase, kr, 0, s);
    wait_vm<0>(); tail_store<1>(buf1, lg.taddr, tb);
    stage_issue<1>(gb, so, of, buf0, ta);
    dot_stage<1, NT>(buf1, lg.sbase, kr, kCGB, s);
    // dP = v . dout
    wait_vm<0>(); tail_store<1>(buf0, lg.taddr, ta);
    stage_issue<1>(g1, so, of, buf1, tb);
    dot_stage<1, NT>(buf0, lg.sbase, vr, 0, dp);
    wait_vm<0>(); tail_store<1>(buf1, lg.taddr, tb);
    stage_issue<1>(qb, so, of, buf0, ta);
    dot_stage<1, NT>(buf1, lg.sbase, vr, kCGB, dp);
    // p = omega exp2(s - lse2_i), dS = p (dP - D_i): lse and D of output column (own column + r + t)
    {
        constexpr int SL4 = (3 + NT + 3) / 4;
        float ls[4 * SL4], ds[4 * SL4];
        const int ab = 4 * (lane >> 2);
#pragma unroll
        for (int a = 0; a < SL4; ++a) {
            const float4 x = *reinterpret_cast<const float4 *>(aux + ab + 4 * a);
            const float4 y = *reinterpret_cast<const float4 *>(aux + G::PITCH + ab + 4 * a);
            ls[4 * a] = fmaf(x.x, kLog2e, -lref2); ls[4 * a + 1] = fmaf(x.y, kLog2e, -lref2);
            ls[4 * a + 2] = fmaf(x.z, kLog2e, -lref2); ls[4 * a + 3] = fmaf(x.w, kLog2e, -lref2);
            ds[4 * a] = y.x; ds[4 * a + 1] = y.y; ds[4 * a + 2] = y.z; ds[4 * a + 3] = y.w;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                const float sv = quad_sum(s[r][tt]), dv2 = quad_sum(dp[r][tt]);
                const float p = wq * __builtin_amdgcn_exp2f(sv - ls[r + tt]);
                s[r][tt] = p;
                dp[r][tt] = p * (dv2 - ds[r + tt]);
            }
    }
    // dk += dS Q ; dv += p dout
    wait_vm<0>(); tail_store<1>(buf0, lg.taddr, ta);
    stage_issue<1>(q1, so, of, buf1, tb);
    axpy_stage<1, NT>(buf0, lg.sbase, dp, 0, dk);
    wait_vm<0>(); tail_store<1>(buf1, lg.taddr, tb);
    stage_issue<1>(gb, so, of, buf0, ta);
    axpy_stage<1, NT>(buf1, lg.sbase, dp, kCGB, dk);
    wait_vm<0>(); tail_store<1>(buf0, lg.taddr, ta);
    stage_issue<1>(g1, so, of, buf1, tb);
    axpy_stage<1, NT>(buf0, lg.sbase, s, 0, dv);
    wait_vm<0>(); tail_store<1>(buf1, lg.taddr, tb);
    axpy_stage<1, NT>(buf1, lg.sbase, s, kCGB, dv);
}

// UP (upsampling, nlon_out = U * nlon_in): the outputs of class s (w = U*u + s) that hold input column j on a
// latitude are u = j - ulo - c + 1 .. j - ulo, with (c, ulo) the arc of that class; the kernel walks the classes one
// after the other, streaming every U-th column of the q, dout, lse and D rows.
template <int WAVES, bool UP = false>
__global__ void __launch_bounds__(64 * WAVES, 2)
nattn_bwd_dkdv_tiled(S2DeviceTables t, int nbh, int first_row, float scale, const float *__restrict__ q,
                     const float *__restrict__ k, const float *__restrict__ v, const float *__restrict__ lse,
                     const float *__restrict__ go, const float *__restrict__ Dws, float *__restrict__ dk,
                     float *__restrict__ dv)
{
    using G = GeoB<1>;
    constexpr int D = 4 * kDL;
    constexpr int WSZ = 2 * G::TILE + 2 * G::PITCH;   // floats of LDS per wavefront: two stages + lse/D rows
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int wave = WAVES == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    float *buf0 = smem + wave * WSZ, *buf1 = buf0 + G::TILE, *aux = buf1 + G::TILE;
    const int nlon = t.nlon_in;                       // equal grids: nlon_out == nlon_in; UP: outputs per class
    const int nlon_o = UP ? t.nlon_out : nlon, U = UP ? t.upscale : 1;
    const int nseg = (nlon + kSegB - 1) / kSegB;
    const Task tk = decode_task<WAVES>(t.bwd_cls, t.trow_order, nseg, nbh, first_row, wave);
    const int hp = tk.row, bh = tk.bh;
    const bool wave_active = bh < nbh;
    const int qd = lane & 3;
    const int w0 = tk.seg * kSegB + 4 * (lane >> 2);
    const bool active = wave_active && w0 < nlon;
    const LaneGeo lg = lane_geo<1>(lane);
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t ii = size_t(hp) * nlon + w0;
    const float qscale = scale * kLog2e;
    const float wq = t.omega_rel[hp], lref2 = t.ln_omega_ref * kLog2e;

    float kr[4][kDL], vr[4][kDL], dka[4][kDL], dva[4][kDL];
#pragma unroll
    for (int c = 0; c < kDL; ++c) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x;
        if (active) {
            const size_t off = (size_t(bh) * D + qd * kDL + c) * si + ii;
            x = *reinterpret_cast<const float4 *>(k + off);
            y = *reinterpret_cast<const float4 *>(v + off);
        }
        kr[0][c] = x.x * qscale; kr[1][c] = x.y * qscale; kr[2][c] = x.z * qscale; kr[3][c] = x.w * qscale;
        vr[0][c] = y.x; vr[1][c] = y.y; vr[2][c] = y.z; vr[3][c] = y.w;
        dka[0][c] = dka[1][c] = dka[2][c] = dka[3][c] = 0.f;
        dva[0][c] = dva[1][c] = dva[2][c] = dva[3][c] = 0.f;
    }

    const int nb = t.tband_n[hp], h0 = t.tband_lo[hp];
    // arc of output offsets (count c, first offset lo) on band row b for the outputs of class sc
    auto arc = [&](int b, int sc, int &c, int &lo) {
        if constexpr (UP) {
            const int h = h0 + b;
            const int at = (h * U + sc) * t.band_max + (hp - t.band_lo[h]);
            c = t.ucnt[at];
            lo = (c == nlon) ? 0 : -(t.ulo[at] + c - 1);
        } else {
            c = t.tcnt[hp * t.tband_max + b];
            lo = (c == nlon) ? 0 : -((c - 1) >> 1);
        }
    };
    int run = 0;
    if (wave_active) {
        // rotated band order (see the dq kernel): concurrent workgroups read the same latitudes together
        const int rot = (t.tband_max - h0 % t.tband_max) % t.tband_max % nb;
        for (int bb = 0; bb < nb * U; ++bb) {
            const int bq = UP ? bb / U : bb, sc = UP ? bb - bq * U : 0;
            const int b = bq + rot < nb ? bq + rot : bq + rot - nb;
            const int h = h0 + b;
            int c, lo;
            arc(b, sc, c, lo);
            if (UP && c == 0) continue;                     // no output of this class holds the owners
            const int nchunk = (c + kNTMax - 1) / kNTMax;
            if (((tk.part - run) & (tk.P - 1)) >= nchunk) { run += nchunk; continue; }   // none of these runs is mine
            const float *qb = q + size_t(bh) * D * so + size_t(h) * nlon_o;
            const float *gb = go + size_t(bh) * D * so + size_t(h) * nlon_o;
            const float *lrow = lse + size_t(bh) * so + size_t(h) * nlon_o;
            const float *drow = Dws + size_t(bh) * so + size_t(h) * nlon_o;
            const int base = c / nchunk, rem = c - base * nchunk;
            int t0 = 0;
            for (int ci = 0; ci < nchunk; ++ci, ++run) {
                const int nt = base + (ci < rem ? 1 : 0);
                if ((run & (tk.P - 1)) == tk.part) {
                    const int xw = wrap2(tk.seg * kSegB + lo + t0 + nlon, nlon);
#define S2_RUN(N) case N: run_chunk_dkdv<N>(buf0, buf1, aux, qb, gb, lrow, drow, so, xw, nlon, lane, lg, wq, lref2, kr, vr, dka, dva, U, sc); break;
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
    if (WAVES > 1 && tk.P > 1) merge_sum<2>(smem, wave, lane, tk.P, tk.part, dka, dva);
    if (!active || tk.part != 0) return;
#pragma unroll
    for (int c = 0; c < kDL; ++c) {
        const size_t off = (size_t(bh) * D + qd * kDL + c) * si + ii;
        *reinterpret_cast<float4 *>(dk + off) =
            make_float4(dka[0][c] * scale, dka[1][c] * scale, dka[2][c] * scale, dka[3][c] * scale);
        *reinterpret_cast<float4 *>(dv + off) = make_float4(dva[0][c], dva[1][c], dva[2][c], dva[3][c]);
    }
}

// ------------------------------------------ dk, dv with nlon_in = 2 * nlon_out ----------
//
// Input point (h', w_in) lies in the disk of output (h, w) iff |2w - w_in| <= half-arc(h, h').
// A lane quad owns inputs w_in = 4p .. 4p+3 and walks OUTPUT columns w = 2p + (r >> 1) + jj:
// the slot jj is valid for owner r iff |2 jj - (r & 1)| <= half-arc, which only trims the two
// ends of the slot range for one parity; invalid slots get weight 0.  The window of output
// columns a wavefront touches is at most 31 + 10 wide, so one 64-column load per row fills it.

constexpr int kPitch2 = 68;               // = 4 mod 16, >= 64
constexpr int kTile2 = kRows * kPitch2;

__device__ __forceinline__ void stage_issue2(const float *chan0, size_t sstride, unsigned voff, float *buf)
{
    asm volatile("" : "+v"(voff));
    const char *rb = reinterpret_cast<const char *>(chan0);
    asm volatile("" : "+s"(rb));
    const size_t rs = sstride * sizeof(float);
#pragma unroll
    for (int r = 0; r < kRows; ++r) {
        __builtin_amdgcn_global_load_lds((gptr_t)(rb + voff), (lptr_t)(buf + r * kPitch2), 4, 0, 0);
        rb += ((r & 3) == 3) ? rs * (kDL - kCGB + 1) : rs;
    }
}

template <int NT>
__device__ __forceinline__ void read_strip2(const float *p, float (&st)[NT + 2])
{
#pragma unroll
    for (int a = 0; a < (NT + 2) / 2; ++a) {
        const float2 x = *reinterpret_cast<const float2 *>(p + 2 * a);
        st[2 * a] = x.x; st[2 * a + 1] = x.y;
    }
}

template <int NT>
__device__ __forceinline__ void dot_stage2(const float *buf, int sbase, const float (&own)[4][kDL], int c0, float (&acc)[4][NT])
{
#pragma unroll
    for (int cc = 0; cc < kCGB; ++cc) {
        float st[NT + 2];
        read_strip2<NT>(buf + sbase + cc * kPitch2, st);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r][tt] = fmaf(own[r][c0 + cc], st[(r >> 1) + tt], acc[r][tt]);
    }
}

template <int NT>
__device__ __forceinline__ void axpy_stage2(const float *buf, int sbase, const float (&w)[4][NT], int c0, float (&out)[4][kDL])
{
#pragma unroll
    for (int cc = 0; cc < kCGB; ++cc) {
        float st[NT + 2];
        read_strip2<NT>(buf + sbase + cc * kPitch2, st);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int r = 0; r < 4; ++r) out[r][c0 + cc] = fmaf(w[r][tt], st[(r >> 1) + tt], out[r][c0 + cc]);
    }
}

// one run of NT slots jj0 .. jj0+NT-1 on output latitude h; wv[parity][tt] = omega weight or 0
template <int NT>
__device__ __forceinline__ void run_chunk_dkdv2(float *buf0, float *buf1, float *aux, const float *__restrict__ qb,
                                                const float *__restrict__ gb, const float *__restrict__ lrow,
                                                const float *__restrict__ drow, size_t so, unsigned voff, int sbase,
                                                int abase, const float (&wv)[2][NT], float lref2,
                                                const float (&kr)[4][kDL], const float (&vr)[4][kDL],
                                                float (&dk)[4][kDL], float (&dv)[4][kDL])
{
    float s[4][NT], dp[4][NT];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) { s[r][tt] = 0.f; dp[r][tt] = 0.f; }
    unsigned vo = voff;
    asm volatile("" : "+v"(vo));
    __builtin_amdgcn_global_load_lds((gptr_t)(reinterpret_cast<const char *>(lrow) + vo), (lptr_t)aux, 4, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr_t)(reinterpret_cast<const char *>(drow) + vo), (lptr_t)(aux + kPitch2), 4, 0, 0);
    const float *q1 = qb + size_t(kCGB) * so, *g1 = gb + size_t(kCGB) * so;
    stage_issue2(qb, so, voff, buf0);
    wait_vm<0>();
    stage_issue2(q1, so, voff, buf1);
    dot_stage2<NT>(buf0, sbase, kr, 0, s);
    wait_vm<0>();
    stage_issue2(gb, so, voff, buf0);
    dot_stage2<NT>(buf1, sbase, kr, kCGB, s);
    wait_vm<0>();
    stage_issue2(g1, so, voff, buf1);
    dot_stage2<NT>(buf0, sbase, vr, 0, dp);
    wait_vm<0>();
    stage_issue2(qb, so, voff, buf0);
    dot_stage2<NT>(buf1, sbase, vr, kCGB, dp);
    {
        float ls[NT + 2], ds[NT + 2];
        read_strip2<NT>(aux + abase, ls);
        read_strip2<NT>(aux + kPitch2 + abase, ds);
#pragma unroll
        for (int a = 0; a < NT + 2; ++a) ls[a] = fmaf(ls[a], kLog2e, -lref2);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) {
                const float sv = quad_sum(s[r][tt]), dv2 = quad_sum(dp[r][tt]);
                const float p = wv[r & 1][tt] * __builtin_amdgcn_exp2f(sv - ls[(r >> 1) + tt]);
                s[r][tt] = p;
                dp[r][tt] = p * (dv2 - ds[(r >> 1) + tt]);
            }
    }
    wait_vm<0>();
    stage_issue2(q1, so, voff, buf1);
    axpy_stage2<NT>(buf0, sbase, dp, 0, dk);
    wait_vm<0>();
    stage_issue2(gb, so, voff, buf0);
    axpy_stage2<NT>(buf1, sbase, dp, kCGB, dk);
    wait_vm<0>();
    stage_issue2(g1, so, voff, buf1);
    axpy_stage2<NT>(buf0, sbase, s, 0, dv);
    wait_vm<0>(); axpy_stage2<NT>(buf1, sbase, s, kCGB, dv);
}

template <int WAVES>
__global__ void __launch_bounds__(64 * WAVES, 2)
nattn_bwd_dkdv2_tiled(S2DeviceTables t, int nbh, int first_row, float scale, const float *__restrict__ q,
                      const float *__restrict__ k, const float *__restrict__ v, const float *__restrict__ lse,
                      const float *__restrict__ go, const float *__restrict__ Dws, float *__restrict__ dk,
                      float *__restrict__ dv)
{
    constexpr int D = 4 * kDL;
    constexpr int WSZ = 2 * kTile2 + 2 * kPitch2;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int wave = WAVES == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    float *buf0 = smem + wave * WSZ, *buf1 = buf0 + kTile2, *aux = buf1 + kTile2;
    const int nlon_i = t.nlon_in, nlon_o = t.nlon_out;
    const int nseg = (nlon_i + kSegB - 1) / kSegB;
    const Task tk = decode_task<WAVES>(t.bwd_cls, t.trow_order, nseg, nbh, first_row, wave);
    const int hp = tk.row, bh = tk.bh;
    const bool wave_active = bh < nbh;
    const int qd = lane & 3, pq = lane >> 2;
    const int w0 = tk.seg * kSegB + 4 * pq;
    const bool active = wave_active && w0 < nlon_i;
    const size_t so = size_t(t.nlat_out) * nlon_o, si = size_t(t.nlat_in) * nlon_i;
    const size_t ii = size_t(hp) * nlon_i + w0;
    const float qscale = scale * kLog2e;
    const float wq = t.omega_rel[hp], lref2 = t.ln_omega_ref * kLog2e;
    const int sbase = qd * kCGB * kPitch2 + 2 * pq, abase = 2 * pq;

    float kr[4][kDL], vr[4][kDL], dka[4][kDL], dva[4][kDL];
#pragma unroll
    for (int c = 0; c < kDL; ++c) {
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x;
        if (active) {
            const size_t off = (size_t(bh) * D + qd * kDL + c) * si + ii;
            x = *reinterpret_cast<const float4 *>(k + off);
            y = *reinterpret_cast<const float4 *>(v + off);
        }
        kr[0][c] = x.x * qscale; kr[1][c] = x.y * qscale; kr[2][c] = x.z * qscale; kr[3][c] = x.w * qscale;
        vr[0][c] = y.x; vr[1][c] = y.y; vr[2][c] = y.z; vr[3][c] = y.w;
        dka[0][c] = dka[1][c] = dka[2][c] = dka[3][c] = 0.f;
        dva[0][c] = dva[1][c] = dva[2][c] = dva[3][c] = 0.f;
    }

    // slots per band row: full circle -> nlon_o slots from 0; arc of half-width hw -> hw + 1 slots from -(hw / 2)
    const int nb = t.tband_n[hp], h0 = t.tband_lo[hp];
    auto nslots = [&](int c) { return c == nlon_i ? nlon_o : ((c - 1) >> 1) + 1; };
    // contiguous shares of the run list (dealing the runs out in turn, as the other kernels do, was slower here)
    int nrun = 0;
    for (int b = 0; b < nb; ++b) nrun += (nslots(t.tcnt[hp * t.tband_max + b]) + kNTMax - 1) / kNTMax;
    const int run_lo = tk.part * nrun / tk.P, run_hi = (tk.part + 1) * nrun / tk.P;
    int run = 0;
    if (wave_active) {
        // rotated band order (see the dq kernel): concurrent workgroups read the same latitudes together
        const int rot = (t.tband_max - h0 % t.tband_max) % t.tband_max % nb;
        for (int bb = 0; bb < nb; ++bb) {
            const int b = bb + rot < nb ? bb + rot : bb + rot - nb;
            const int h = h0 + b;
            const int c = t.tcnt[hp * t.tband_max + b];
            const bool full = c == nlon_i;
            const int hw = (c - 1) >> 1, nj = nslots(c);
            const int nchunk = (nj + kNTMax - 1) / kNTMax;
            if (run + nchunk <= run_lo || run >= run_hi) { run += nchunk; continue; }
            const int jlo = full ? 0 : -(hw >> 1);
            const float *qb = q + size_t(bh) * D * so + size_t(h) * nlon_o;
            const float *gb = go + size_t(bh) * D * so + size_t(h) * nlon_o;
            const float *lrow = lse + size_t(bh) * so + size_t(h) * nlon_o;
            const float *drow = Dws + size_t(bh) * so + size_t(h) * nlon_o;
            const int base = nj / nchunk, rem = nj - base * nchunk;
            int t0 = 0;
            for (int ci = 0; ci < nchunk; ++ci, ++run) {
                const int nt = base + (ci < rem ? 1 : 0);
                if (run >= run_lo && run < run_hi) {
                    const int jj0 = jlo + t0;
                    const int xw = wrap2(tk.seg * (kSegB / 2) + jj0 + nlon_o, nlon_o);
                    const unsigned voff = 4u * unsigned(wrap2(xw + lane, nlon_o));
#define S2_RUN(N)                                                                                              \
    case N: {                                                                                                  \
        float wv[2][N];                                                                                        \
        _Pragma("unroll") for (int tt = 0; tt < N; ++tt) {                                                    \
            const int j2 = 2 * (jj0 + tt);                                                                     \
            wv[0][tt] = (full || (j2 <= hw && -j2 <= hw)) ? wq : 0.f;                                           \
            wv[1][tt] = (full || (j2 - 1 <= hw && 1 - j2 <= hw)) ? wq : 0.f;                                    \
        }                                                                                                      \
        run_chunk_dkdv2<N>(buf0, buf1, aux, qb, gb, lrow, drow, so, voff, sbase, abase, wv, lref2, kr, vr, dka, \
                           dva);                                                                               \
    } break;
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
    if (WAVES > 1 && tk.P > 1) merge_sum<2>(smem, wave, lane, tk.P, tk.part, dka, dva);
    if (!active || tk.part != 0) return;
#pragma unroll
    for (int c = 0; c < kDL; ++c) {
        const size_t off = (size_t(bh) * D + qd * kDL + c) * si + ii;
        *reinterpret_cast<float4 *>(dk + off) =
            make_float4(dka[0][c] * scale, dka[1][c] * scale, dka[2][c] * scale, dka[3][c] * scale);
        *reinterpret_cast<float4 *>(dv + off) = make_float4(dva[0][c], dva[1][c], dva[2][c], dva[3][c]);
    }
}

}  // namespace

bool s2_nattn_bwd_tiled_supported(const S2DeviceTables &t, int d, int e)
{
    if (t.upscale > 1) return d == 32 && e == 32 && t.nlon_in % 4 == 0 && t.nlon_in >= 72;
    return d == 32 && e == 32 && (t.pscale == 1 || t.pscale == 2) && t.nlon_in % 4 == 0 && t.nlon_out % 4 == 0 &&
           t.nlon_out >= 72;
}

int s2_nattn_bwd_tiled_configure()
{
    auto raise = [](auto kern, size_t lds_wave, size_t merge) {
        size_t lds = lds_wave * kWavesB;
        if (lds < merge) lds = merge;
        return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   int(lds)) == hipSuccess;
    };
    // 8-wave kernels: per-wavefront staging buffers, reused for the merge of the partial sums
    const size_t mg_q = size_t(kWavesB / 2) * 4 * kDL * 64 * sizeof(float), mg_kv = 2 * mg_q;
    const size_t kv1 = (2 * GeoB<1>::TILE + 2 * GeoB<1>::PITCH) * sizeof(float), kv2 = (2 * kTile2 + 2 * kPitch2) * sizeof(float);
    return raise(nattn_bwd_dq_tiled<1, kWavesB>, 2 * GeoB<1>::TILE * sizeof(float), mg_q) &&
           raise(nattn_bwd_dq_tiled<2, kWavesB>, 2 * GeoB<2>::TILE * sizeof(float), mg_q) &&
           raise(nattn_bwd_dq_tiled<1, kWavesB, true>, 2 * GeoB<1>::TILE * sizeof(float), mg_q) &&
           raise(nattn_bwd_dkdv_tiled<kWavesB>, kv1, mg_kv) && raise(nattn_bwd_dkdv_tiled<kWavesB, true>, kv1, mg_kv) &&
           raise(nattn_bwd_dkdv2_tiled<kWavesB>, kv2, mg_kv) ? 0 : -1;
}

namespace {

// Upsampling grids: the split vector kernels in their class view (no matrix-core or streaming launches).
int bwd_tiled_up(const S2DeviceTables &t_all, int nbh, float scale, const float *q, const float *k, const float *v,
                 const float *o, const float *lse, const float *go, float *dq, float *dk, float *dv, float *Dws,
                 hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    const int nseg_o = ((t_all.nlon_in + kSegB - 1) / kSegB) * t_all.upscale, nseg_i = (t_all.nlon_in + kSegB - 1) / kSegB;
    {
        S2DeviceTables t = t_all;
        s2_pick_split(t, true, nbh, nseg_o, false);
        const int nsplit = t.fwd_cls[0] + t.fwd_cls[1] + t.fwd_cls[2];
        const size_t lds_wave = 2 * GeoB<1>::TILE * sizeof(float);
        if (nsplit > 0) {
            const long nblk = long((nbh + kWavesB - 1) / kWavesB) * nseg_o * (8 * t.fwd_cls[0] + 4 * t.fwd_cls[1] + 2 * t.fwd_cls[2]);
            size_t lds = lds_wave * kWavesB;
            const size_t mg = size_t(kWavesB / 2) * 4 * kDL * 64 * sizeof(float);
            if (lds < mg) lds = mg;
            auto k8 = nattn_bwd_dq_tiled<1, kWavesB, true>;
            S2TraceScope tr("nattn_bwd_dq_tiled<8 waves, classes>", nbh * (t.fwd_pairs[0] + t.fwd_pairs[1] + t.fwd_pairs[2]), st);
            hipLaunchKernelGGL(k8, dim3((unsigned)nblk), dim3(64 * kWavesB), lds, st, t, nbh, 1, scale, q, k, v, o, lse,
                               go, dq, Dws);
        }
        const long nrows = t.nlat_out - nsplit;
        if (nrows > 0) {
            S2TraceScope tr("nattn_bwd_dq_tiled<1 wave, classes>", nbh * t.fwd_pairs[3], st);
            hipLaunchKernelGGL((nattn_bwd_dq_tiled<1, 1, true>), dim3((unsigned)(nrows * nbh * nseg_o)), dim3(64), lds_wave,
                               st, t, nbh, nsplit, scale, q, k, v, o, lse, go, dq, Dws);
        }
    }
    S2DeviceTables t = t_all;
    s2_pick_split(t, false, nbh, nseg_i, false);
    const int nsplit = t.bwd_cls[0] + t.bwd_cls[1] + t.bwd_cls[2];
    const size_t lds_wave = (2 * GeoB<1>::TILE + 2 * GeoB<1>::PITCH) * sizeof(float);
    if (nsplit > 0) {
        const long nblk = long((nbh + kWavesB - 1) / kWavesB) * nseg_i * (8 * t.bwd_cls[0] + 4 * t.bwd_cls[1] + 2 * t.bwd_cls[2]);
        size_t lds = lds_wave * kWavesB;
        const size_t mg = size_t(kWavesB / 2) * 2 * 4 * kDL * 64 * sizeof(float);
        if (lds < mg) lds = mg;
        auto k8 = nattn_bwd_dkdv_tiled<kWavesB, true>;
        S2TraceScope tr("nattn_bwd_dkdv_tiled<8 waves, classes>", nbh * (t.bwd_pairs[0] + t.bwd_pairs[1] + t.bwd_pairs[2]), st);
        hipLaunchKernelGGL(k8, dim3((unsigned)nblk), dim3(64 * kWavesB), lds, st, t, nbh, 1, scale, q, k, v, lse, go, Dws,
                           dk, dv);
    }
    const long nrows = t.nlat_in - nsplit;
    if (nrows > 0) {
        S2TraceScope tr("nattn_bwd_dkdv_tiled<1 wave, classes>", nbh * t.bwd_pairs[3], st);
        hipLaunchKernelGGL((nattn_bwd_dkdv_tiled<1, true>), dim3((unsigned)(nrows * nbh * nseg_i)), dim3(64), lds_wave, st,
                           t, nbh, nsplit, scale, q, k, v, lse, go, Dws, dk, dv);
    }
    return 0;
}

}  // namespace

int s2_nattn_bwd_tiled(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q, const float *k,
                       const float *v, const float *o, const float *lse, const float *go, float *dq, float *dk,
                       float *dv, float *Dws, hipStream_t st)
{
    if (t.upscale > 1) return bwd_tiled_up(t, nbh, scale, q, k, v, o, lse, go, dq, dk, dv, Dws, st);
    const int nseg_o = (t.nlon_out + kSegB - 1) / kSegB;
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    const bool no_stream = s2_debug_flag(S2_DEBUG_NO_STREAM);   // test-only: one-wave kernels instead
    // dense polar latitudes: dq on the matrix cores; the vector kernels see the remaining latitudes
    const S2DeviceTables &t_all = t;
    S2DeviceTables t_dq = t_all;
    const int nm = s2_nattn_fwd_mfma_rows(t_all, d, e);
    if (nm > 0) {
        if (s2_nattn_bwd_dq_mfma(t_all, nbh, nm, scale, q, k, v, o, lse, go, dq, Dws, st)) return -1;
        t_dq.row_order = t_all.row_order + nm;
    }
    if (s2_nattn_stream_dq_supported(t_all, d, e)) {
        if (nm > 0) {
            t_dq.fwd_cls[0] = t_dq.fwd_cls[1] = t_dq.fwd_cls[2] = 0;
            t_dq.fwd_pairs[0] = t_dq.fwd_pairs[1] = t_dq.fwd_pairs[2] = 0.0;
        }
    } else {
        s2_pick_split(t_dq, true, nbh, nseg_o, nm > 0);
    }
    const int nsplit_o = t_dq.fwd_cls[0] + t_dq.fwd_cls[1] + t_dq.fwd_cls[2];
    auto run_dq = [&](auto k8, auto k1, size_t lds_wave) {
        if (nsplit_o > 0) {
            const long nblk = long((nbh + kWavesB - 1) / kWavesB) * nseg_o *
                              (8 * t_dq.fwd_cls[0] + 4 * t_dq.fwd_cls[1] + 2 * t_dq.fwd_cls[2]);
            size_t lds = lds_wave * kWavesB;
            const size_t mg = size_t(kWavesB / 2) * 4 * kDL * 64 * sizeof(float);
            if (lds < mg) lds = mg;
            S2TraceScope tr("nattn_bwd_dq_tiled<8 waves>", nbh * (t_dq.fwd_pairs[0] + t_dq.fwd_pairs[1] + t_dq.fwd_pairs[2]), st);
            hipLaunchKernelGGL(k8, dim3((unsigned)nblk), dim3(64 * kWavesB), lds, st, t_dq, nbh, 1, scale, q, k, v, o, lse,
                               go, dq, Dws);
        }
        const long nrows = t.nlat_out - nm - nsplit_o;
        if (nrows > 0 && !no_stream && s2_nattn_stream_dq_supported(t_dq, d, e))
            return s2_nattn_bwd_dq_stream(t_dq, nbh, scale, q, k, v, o, lse, go, dq, Dws, st);
        if (nrows <= 0) return 0;
        S2TraceScope tr("nattn_bwd_dq_tiled<1 wave>", nbh * t_dq.fwd_pairs[3], st);
        hipLaunchKernelGGL(k1, dim3((unsigned)(nrows * nbh * nseg_o)), dim3(64), lds_wave, st, t_dq, nbh, nsplit_o,
                               scale, q, k, v, o, lse, go, dq, Dws);
        return 0;
    };
    int rc;
    if (t.pscale == 1)
        rc = run_dq(nattn_bwd_dq_tiled<1, kWavesB>, nattn_bwd_dq_tiled<1, 1>, 2 * GeoB<1>::TILE * sizeof(float));
    else
        rc = run_dq(nattn_bwd_dq_tiled<2, kWavesB>, nattn_bwd_dq_tiled<2, 1>, 2 * GeoB<2>::TILE * sizeof(float));
    if (rc) return rc;

    if (t_all.pscale == 2) {
        const int nseg_i = (t_all.nlon_in + kSegB - 1) / kSegB;
        S2DeviceTables t = t_all;
        s2_pick_split(t, false, nbh, nseg_i, false);
        const int nsplit_i = t.bwd_cls[0] + t.bwd_cls[1] + t.bwd_cls[2];
        const size_t lds_wave = (2 * kTile2 + 2 * kPitch2) * sizeof(float);
        if (nsplit_i > 0) {
            const long nblk = long((nbh + kWavesB - 1) / kWavesB) * nseg_i *
                              (8 * t.bwd_cls[0] + 4 * t.bwd_cls[1] + 2 * t.bwd_cls[2]);
            size_t lds = lds_wave * kWavesB;
            const size_t mg = size_t(kWavesB / 2) * 2 * 4 * kDL * 64 * sizeof(float);
            if (lds < mg) lds = mg;
            auto k8 = nattn_bwd_dkdv2_tiled<kWavesB>;
            S2TraceScope tr("nattn_bwd_dkdv2_tiled<8 waves>", nbh * (t.bwd_pairs[0] + t.bwd_pairs[1] + t.bwd_pairs[2]), st);
            hipLaunchKernelGGL(k8, dim3((unsigned)nblk), dim3(64 * kWavesB), lds, st, t, nbh, 1, scale, q, k, v, lse,
                               go, Dws, dk, dv);
        }
        const long nrows = t.nlat_in - nsplit_i;
        if (nrows <= 0) return 0;
        S2TraceScope tr("nattn_bwd_dkdv2_tiled<1 wave>", nbh * t.bwd_pairs[3], st);
        hipLaunchKernelGGL((nattn_bwd_dkdv2_tiled<1>), dim3((unsigned)(nrows * nbh * nseg_i)), dim3(64), lds_wave,
                               st, t, nbh, nsplit_i, scale, q, k, v, lse, go, Dws, dk, dv);
        return 0;
    }
    const int nseg_i = (t.nlon_in + kSegB - 1) / kSegB;
    // dense polar input latitudes: dk/dv on the matrix cores
    S2DeviceTables t_kv = t_all;
    const int nmi = s2_nattn_bwd_dkdv_mfma_rows(t_all, d, e);
    if (nmi > 0) {
        if (s2_nattn_bwd_dkdv_mfma(t_all, nbh, nmi, scale, q, k, v, lse, go, Dws, dk, dv, st)) return -1;
        t_kv.trow_order = t_all.trow_order + nmi;
    }
    if (s2_nattn_stream_dkdv_supported(t_all, d, e)) {
        if (nmi > 0) {
            t_kv.bwd_cls[0] = t_kv.bwd_cls[1] = t_kv.bwd_cls[2] = 0;
            t_kv.bwd_pairs[0] = t_kv.bwd_pairs[1] = t_kv.bwd_pairs[2] = 0.0;
        }
    } else {
        s2_pick_split(t_kv, false, nbh, nseg_i, nmi > 0);
    }
    const int nsplit_i = t_kv.bwd_cls[0] + t_kv.bwd_cls[1] + t_kv.bwd_cls[2];
    const size_t lds_wave = (2 * GeoB<1>::TILE + 2 * GeoB<1>::PITCH) * sizeof(float);
    if (nsplit_i > 0) {
        const long nblk = long((nbh + kWavesB - 1) / kWavesB) * nseg_i *
                          (8 * t_kv.bwd_cls[0] + 4 * t_kv.bwd_cls[1] + 2 * t_kv.bwd_cls[2]);
        size_t lds = lds_wave * kWavesB;
        const size_t mg = size_t(kWavesB / 2) * 2 * 4 * kDL * 64 * sizeof(float);
        if (lds < mg) lds = mg;
        auto k8 = nattn_bwd_dkdv_tiled<kWavesB>;
        S2TraceScope tr("nattn_bwd_dkdv_tiled<8 waves>", nbh * (t_kv.bwd_pairs[0] + t_kv.bwd_pairs[1] + t_kv.bwd_pairs[2]), st);
        hipLaunchKernelGGL(k8, dim3((unsigned)nblk), dim3(64 * kWavesB), lds, st, t_kv, nbh, 1, scale, q, k, v, lse, go,
                           Dws, dk, dv);
    }
    const long nrows = t.nlat_in - nmi - nsplit_i;
    if (nrows > 0 && !no_stream && s2_nattn_stream_dkdv_supported(t_kv, d, e))
        return s2_nattn_bwd_dkdv_stream(t_kv, nbh, scale, q, k, v, lse, go, Dws, dk, dv, st);
    if (nrows <= 0) return 0;
    S2TraceScope tr("nattn_bwd_dkdv_tiled<1 wave>", nbh * t_kv.bwd_pairs[3], st);
    hipLaunchKernelGGL((nattn_bwd_dkdv_tiled<1>), dim3((unsigned)(nrows * nbh * nseg_i)), dim3(64), lds_wave, st,
                           t_kv, nbh, nsplit_i, scale, q, k, v, lse, go, Dws, dk, dv);
    return 0;
}
