// Neighborhood attention (Sec. 3.3, eq. (9)-(10); gradients App. B.4) on the fp32 matrix cores for head dimensions
// other than the hand-tuned 32: band tiles of 16 keys x 16 outputs on v_mfma_f32_16x16x4_f32, float32 throughout.
// Equal grids, d = e in {16, 32, 64}, longitude count a multiple of 16 (at least 64).
//
// Structure.  A workgroup of four wavefronts owns OW = 16 NO consecutive longitudes of FOUR consecutive latitudes, one
// latitude per wavefront (forward and dq: output latitudes; dk/dv: input latitudes, walking the transposed
// neighborhood).  It walks the union of the four bands row by row; a row of the other side is copied to LDS once
// (channel-major, as it lies in memory: no transposition) and serves every wavefront whose band holds it.
//   * Rows with short arcs (half-width of every wavefront <= 28): ONE stage of SW = OW + 64 columns holds the window
//     of all owners; every 16-owner tile walks its own key tiles from the first column of its band rounded down to
//     a multiple of four.
//   * Rows with long arcs or whole circles (near the poles): the window (or, when it would reach around the sphere,
//     the whole circle, every column once) is walked in stages of SW columns with key tiles on a common 16-column
//     grid; distances are taken around the circle.
// For 16 outputs the keys of one row form a band of the keys x outputs score matrix: a tile the band does not touch
// is skipped (wavefront-uniform), a tile it cuts gets a per-element mask, a tile inside it none.
//
// Operands of v_mfma_f32_16x16x4_f32 (A: 16 x 4, one value per lane (row = lane & 15, k = lane >> 4); B: 4 x 16
// (k = lane >> 4, column = lane & 15); C/D: lane holds rows 4 (lane >> 4) + 0..3 of column lane & 15):
//   S^T = K Q^T      A = K[channel 4 kb + g][key column]  (one LDS word per lane), B = q of the lane's output,
//                    kb = 0 .. d/4 - 1: lane (n, g) ends with the logits of keys 4 g + 0..3 for output n;
//   O^T += V P^T     the contraction index of instruction j is key 4 g + j, so B is the lane's own probability j
//                    (no data movement between lanes) and A = V[channel 16 mt + (lane & 15)][keys 4 g + 0..3]:
//                    one 16-byte LDS read serves four instructions.
// Channel row c of a staged tile starts at c * pitch + 4 ((c >> 2) & 3) floats with a pitch of 16 mod 32 words: the four
// rows 4 kb + g of the first read pattern fall into four different groups of 16 banks, and the 16 rows 16 mt + n of
// the second into 16 different groups of four banks, so both are free of bank conflicts.
// Softmax: base 2, ln omega as a bias on the logit, lazy reference maximum (moves when exceeded by 2^8; only then do
// the four lanes of an output exchange maxima).  Every matrix result is consumed in the block that issues it.
#include <hip/hip_runtime.h>

#include "s2_internal.h"
#include "s2_nattn_kernels.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kBig = 1 << 20;        // half-width that stands for a whole circle
constexpr int kShort = 28;           // largest half-width served by a single stage
constexpr float kMinRef = -1e30f;    // start value of the reference maximum: finite, so that x - m needs no guard (exp2(-inf) = 0)

template <int D, int NO>
struct Geo {
    static constexpr int OW = 16 * NO;           // longitudes per workgroup
    static constexpr int SW = OW + 64;           // staged columns
    static constexpr int COLS = SW + 32;         // + zeroed padding (a tile may reach past the window)
    static constexpr int PITCH = (COLS + 16) % 32 == 16 ? COLS + 16 : COLS + 32;      // floats per channel row (16 mod 32); row c starts 4 ((c >> 2) & 3) floats in
    static constexpr int TILE = D * PITCH;       // floats per staged tensor
    static constexpr int P4 = SW / 4;            // 16-byte pieces per channel row
    static constexpr int NP = (D * P4 + 255) / 256;      // pieces per thread and tensor (the last may be partial)
    static constexpr bool EVEN = D * P4 % 256 == 0;
    static_assert(PITCH % 32 == 16, "geometry");
};

// Storage type of the tensors: float, or bf16 bits (arithmetic, staged tiles, logsumexp and D stay float32).
typedef unsigned short bf16raw;
__device__ __forceinline__ float ldx(const float *p) { return *p; }
__device__ __forceinline__ float ldx(const bf16raw *p) { return __builtin_bit_cast(float, unsigned(*p) << 16); }
__device__ __forceinline__ void stx(float *p, float x) { *p = x; }
__device__ __forceinline__ void stx(bf16raw *p, float x)          // round to nearest even
{
    const unsigned u = __builtin_bit_cast(unsigned, x);
    *p = bf16raw((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ f32x4 ld4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
__device__ __forceinline__ f32x4 ld4(const bf16raw *p)
{
    const uint2 w = *reinterpret_cast<const uint2 *>(p);
    return f32x4{__builtin_bit_cast(float, w.x << 16), __builtin_bit_cast(float, w.x & 0xffff0000u),
                 __builtin_bit_cast(float, w.y << 16), __builtin_bit_cast(float, w.y & 0xffff0000u)};
}

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float group_max(float x)     // over the four lanes (g = 0..3) of a point
{
    x = fmaxf(x, __shfl_xor(x, 16));
    return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float group_sum(float x)
{
    x += __shfl_xor(x, 16);
    return x + __shfl_xor(x, 32);
}
__device__ __forceinline__ int wrap3(int col, int nlon)     // columns below 4 nlon
{
    col = col >= 2 * nlon ? col - 2 * nlon : col;
    return col >= nlon ? col - nlon : col;
}

// Rows a workgroup has to stage and their metadata, read from the grid tables once and kept one row per lane (a
// table read inside the row loop would be a vector load whose wait also waits for the prefetch in flight).
struct BandRows {
    int rmin, rmax;
    int hwm_v, hw_v;        // lane i: row rmin + i -- largest half-width among the four latitudes, own half-width (-1: none)
    float lw2_v;            // log2 of the row's relative quadrature weight
    __device__ __forceinline__ void load(const int *blo, const int *bn, const int *cnt, int bmax, const float *omega_rel,
                                         int nlon, int first, int end, int own, bool active, int lane)
    {
        rmin = 1 << 30;
        rmax = -1;
        for (int w = 0; w < 4; ++w) {
            const int hh = first + w;
            if (hh >= end) break;
            if (bn[hh] > 0) {
                rmin = min(rmin, blo[hh]);
                rmax = max(rmax, blo[hh] + bn[hh] - 1);
            }
        }
        const int r = rmin + lane;
        const bool valid = r <= rmax;
        hwm_v = 0;
        hw_v = -1;
        for (int w = 0; w < 4; ++w) {
            const int hh = first + w;
            if (hh >= end) break;
            const int b = r - blo[hh];
            if (valid && b >= 0 && b < bn[hh]) {
                const int c = cnt[hh * bmax + b];
                const int x = c == nlon ? kBig : (c - 1) >> 1;
                hwm_v = max(hwm_v, x);
                if (active && hh == own) hw_v = x;
            }
        }
        lw2_v = valid ? __log2f(omega_rel[r]) : 0.f;
    }
    __device__ __forceinline__ int hwmax(int i) const { return __builtin_amdgcn_readlane(hwm_v, i); }
    __device__ __forceinline__ int hw(int i) const { return __builtin_amdgcn_readlane(hw_v, i); }
    __device__ __forceinline__ float lw2(int i) const
    {
        return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lw2_v), i));
    }
};

// How one row is walked: first staged (unwrapped) column, end of the columns that count, number of stages, and whether
// key tiles lie on the common grid with distances taken around the circle.  Unwrapped columns carry an offset of
// nlon so that they stay non-negative; column X is longitude X mod nlon; the owners sit at Wb .. Wb + OW - 1.
struct RowPlan {
    int Xs0, Xend, nst, multi;
    template <int OW, int SW>
    __device__ __forceinline__ void set(int hwm, int nlon, int Wb)
    {
        if (hwm <= kShort) {
            multi = 0;
            Xs0 = (Wb - hwm) & ~3;
            Xend = Xs0 + SW + 32;
            nst = 1;
        } else {
            multi = 1;
            const bool circle = hwm >= kBig || OW + 2 * hwm + 31 >= nlon;
            Xs0 = circle ? nlon : (Wb - hwm) & ~15;
            Xend = circle ? 2 * nlon : Wb + OW + ((hwm + 15) & ~15);
            nst = (Xend - Xs0 + SW - 1) / SW;
        }
    }
};

template <int D, int NO, int NP, class T>
__device__ __forceinline__ void load_stage(f32x4 (&r)[NP], const T *slice, size_t plane, int lat, int nlon, int Xs,
                                           int tid)
{
    using G = Geo<D, NO>;
    static_assert(NP == G::NP, "pieces per thread");
#pragma unroll
    for (int j = 0; j < G::NP; ++j) {
        const int i = tid + 256 * j, c = i / G::P4, pc = i % G::P4;
        if (G::EVEN || i < D * G::P4) r[j] = ld4(slice + size_t(c) * plane + size_t(lat) * nlon + wrap3(Xs + 4 * pc, nlon));
    }
}
template <int D, int NO, int NP>
__device__ __forceinline__ void store_stage(float *tile, const f32x4 (&r)[NP], int tid)
{
    using G = Geo<D, NO>;
    static_assert(NP == G::NP, "pieces per thread");
#pragma unroll
    for (int j = 0; j < G::NP; ++j) {
        const int i = tid + 256 * j, c = i / G::P4, pc = i % G::P4;
        if (G::EVEN || i < D * G::P4) *reinterpret_cast<f32x4 *>(tile + c * G::PITCH + 4 * ((c >> 2) & 3) + 4 * pc) = r[j];
    }
}

// Position of a key tile relative to the 16 owners at Wo: offset of its first column (taken around the circle on the
// common grid), whether the band of half-width hw touches it, and whether it needs the per-element mask.
struct TilePos {
    int dl;
    bool touch, mask;
    __device__ __forceinline__ void set(int Xt, int Wo, int hw, int nlon, int multi)
    {
        dl = Xt - Wo;
        if (multi) {
            dl = dl >= nlon / 2 ? dl - nlon : dl;
            dl = dl < -nlon / 2 ? dl + nlon : dl;
        }
        const int adl = dl < 0 ? -dl : dl;
        const bool full = hw >= kBig;
        touch = full || adl <= hw + 15;
        mask = !full && adl + 15 > hw;
    }
};
// keep[rr]: is key (tile column 4 g + rr) a neighbor of the lane's output n.  gb = 4 g - n + hw (per lane, fixed for a
// row).  The offset key - output + hw must lie in [0, 2 hw]; on the common grid it is taken modulo nlon.
__device__ __forceinline__ void band_mask(bool (&keep)[4], const TilePos &tp, int hw, int nlon, int multi, int gb)
{
    int uu = tp.dl + gb;
    const unsigned lim = unsigned(2 * hw);
    if (multi) {
        uu = uu < 0 ? uu + nlon : uu;
        uu = uu >= nlon ? uu - nlon : uu;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int v = uu + rr;
            keep[rr] = unsigned(v >= nlon ? v - nlon : v) <= lim;
        }
    } else {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) keep[rr] = unsigned(uu + rr) <= lim;
    }
}
__device__ __forceinline__ float max4(float a, float b, float c, float d)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3\n\tv_max_f32 %0, %0, %4" : "=&v"(r) : "v"(a), "v"(b), "v"(c), "v"(d));
    return r;
}

__device__ __forceinline__ int segment_of(int sk, int nseg)      // polar segments (the heaviest) first, from both ends
{
    return (sk & 1) ? nseg - 1 - (sk >> 1) : (sk >> 1);
}

// ---------------------------------------------------------------------------------------------------------------
// Forward.
template <class T, int D, int NO>
__global__ void __launch_bounds__(256, 2)
nattn_fwd_band(S2DeviceTables t, int nbh, float c2, const T *__restrict__ q, const T *__restrict__ k,
               const T *__restrict__ v, T *__restrict__ out, float *__restrict__ lse)
{
    using G = Geo<D, NO>;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *Kc = lds, *Vc = lds + G::TILE;
    const int nlon = t.nlon_in, ngrp = (nlon + G::OW - 1) / G::OW, nseg = (t.nlat_out + 3) >> 2;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int bh = id % nbh, seg = segment_of(id / nbh, nseg);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int first = 4 * seg, h = first + wave;
    const bool active = h < t.nlat_out;
    const int W0 = grp * G::OW, Wb = nlon + W0;
    const size_t plane = size_t(t.nlat_in) * nlon;
    const T *qs = q + size_t(bh) * D * plane, *ks = k + size_t(bh) * D * plane, *vs = v + size_t(bh) * D * plane;

    float qreg[NO][D / 4];
    f32x4 acc[NO][D / 16];
    float m[NO], l[NO];
#pragma unroll
    for (int o = 0; o < NO; ++o) {
        const bool own = active && W0 + 16 * o < nlon;      // the last group of a latitude may be ragged (by whole tiles)
#pragma unroll
        for (int kb = 0; kb < D / 4; ++kb)
            qreg[o][kb] = own ? ldx(qs + size_t(4 * kb + g) * plane + size_t(h) * nlon + (W0 + 16 * o + n)) : 0.f;
#pragma unroll
        for (int mt = 0; mt < D / 16; ++mt) acc[o][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        m[o] = kMinRef;
        l[o] = 0.f;
    }
    BandRows rows;
    rows.load(t.band_lo, t.band_n, t.cnt, t.band_max, t.omega_rel, nlon, first, t.nlat_out, h, active, lane);
    for (int i = tid; i < 2 * G::TILE; i += 256) lds[i] = 0.f;

    const int nrow = rows.rmax - rows.rmin + 1;
    int ri = 0, s = 0;
    RowPlan cur;
    f32x4 rk[G::NP], rv[G::NP];
    bool more = nrow > 0;
    if (more) {
        cur.template set<G::OW, G::SW>(rows.hwmax(0), nlon, Wb);
        load_stage<D, NO>(rk, ks, plane, rows.rmin, nlon, cur.Xs0, tid);
        load_stage<D, NO>(rv, vs, plane, rows.rmin, nlon, cur.Xs0, tid);
    }
    while (more) {
        __syncthreads();                    // everybody is done with the previous stage (first pass: with the zero fill)
        store_stage<D, NO>(Kc, rk, tid);
        store_stage<D, NO>(Vc, rv, tid);
        __syncthreads();
        const int Xst = cur.Xs0 + s * G::SW;
        const RowPlan now = cur;
        const int rnow = ri;
        if (++s == cur.nst) {
            s = 0;
            ++ri;
            if (ri < nrow) cur.template set<G::OW, G::SW>(rows.hwmax(ri), nlon, Wb);
        }
        more = ri < nrow;
        if (more) {
            load_stage<D, NO>(rk, ks, plane, rows.rmin + ri, nlon, cur.Xs0 + s * G::SW, tid);
            load_stage<D, NO>(rv, vs, plane, rows.rmin + ri, nlon, cur.Xs0 + s * G::SW, tid);
        }
        const int hw = rows.hw(rnow);
        if (hw < 0) continue;
        const float lw2 = rows.lw2(rnow);
        const int Xlim = min(Xst + G::SW + (now.multi ? 0 : 32), now.Xend);
#pragma unroll
        for (int o = 0; o < NO; ++o) {
            if (W0 + 16 * o >= nlon) break;
            const int Wo = Wb + 16 * o;
            const int T0 = now.multi ? Xst : (Wo - hw) & ~3;
            const int Tend = now.multi ? Xlim : Wo + 16 + hw;
            for (int Xt = T0; Xt < Tend; Xt += 16) {
                TilePos tp;
                tp.set(Xt, Wo, hw, nlon, now.multi);
                if (!tp.touch) continue;
                const int col0 = Xt - Xst;
                const float *kp = Kc + g * G::PITCH + col0 + n;
                f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kb = 0; kb < D / 4; ++kb) sc = mfma4(kp[kb * 4 * G::PITCH + 4 * (kb & 3)], qreg[o][kb], sc);
                float x[4];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) x[rr] = fmaf(sc[rr], c2, lw2);
                if (tp.mask) {
                    bool keep[4];
                    band_mask(keep, tp, hw, nlon, now.multi, 4 * g - n + hw);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) x[rr] = keep[rr] ? x[rr] : -INFINITY;
                }
                float mx = max4(x[0], x[1], x[2], x[3]);
                if (__any(mx > m[o] + 8.f)) {
                    mx = group_max(mx);
                    const float m_new = mx > m[o] + 8.f ? mx : m[o];
                    const float corr = __builtin_amdgcn_exp2f(m[o] - m_new);
                    m[o] = m_new;
                    l[o] *= corr;
#pragma unroll
                    for (int mt = 0; mt < D / 16; ++mt)
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) acc[o][mt][rr] *= corr;
                }
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    x[rr] = __builtin_amdgcn_exp2f(x[rr] - m[o]);
                    l[o] += x[rr];
                }
                const float *vp = Vc + n * G::PITCH + 4 * ((n >> 2) & 3) + col0 + 4 * g;
                f32x4 va[D / 16];
#pragma unroll
                for (int mt = 0; mt < D / 16; ++mt) va[mt] = *reinterpret_cast<const f32x4 *>(vp + mt * 16 * G::PITCH);
#pragma unroll
                for (int j = 0; j < 4; ++j)          // consecutive instructions belong to different accumulators
#pragma unroll
                    for (int mt = 0; mt < D / 16; ++mt) acc[o][mt] = mfma4(va[mt][j], x[j], acc[o][mt]);
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int o = 0; o < NO; ++o) {
        if (W0 + 16 * o >= nlon) break;
        const float lt = group_sum(l[o]);
        const float inv = 1.f / lt;
        const size_t at = size_t(h) * nlon + (W0 + 16 * o + n);
        T *ob = out + size_t(bh) * D * plane + at;
#pragma unroll
        for (int mt = 0; mt < D / 16; ++mt)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) stx(ob + size_t(16 * mt + 4 * g + rr) * plane, acc[o][mt][rr] * inv);
        if (g == 0) lse[size_t(bh) * plane + at] = (m[o] + __log2f(lt)) * 0.6931471805599453f + t.ln_omega_ref;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Backward, query side: dq and D_i = dout_i . out_i (written for the key-side launch).
template <class T, int D, int NO>
__global__ void __launch_bounds__(256, 2)
nattn_bwd_dq_band(S2DeviceTables t, int nbh, float scale, const T *__restrict__ q, const T *__restrict__ k,
                  const T *__restrict__ v, const T *__restrict__ o_, const float *__restrict__ lse,
                  const T *__restrict__ go, T *__restrict__ dq, float *__restrict__ Dws)
{
    using G = Geo<D, NO>;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *Kc = lds, *Vc = lds + G::TILE;
    const int nlon = t.nlon_in, ngrp = (nlon + G::OW - 1) / G::OW, nseg = (t.nlat_out + 3) >> 2;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int bh = id % nbh, seg = segment_of(id / nbh, nseg);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int first = 4 * seg, h = first + wave;
    const bool active = h < t.nlat_out;
    const int W0 = grp * G::OW, Wb = nlon + W0;
    const size_t plane = size_t(t.nlat_in) * nlon;
    const T *qs = q + size_t(bh) * D * plane, *ks = k + size_t(bh) * D * plane, *vs = v + size_t(bh) * D * plane;
    const T *os = o_ + size_t(bh) * D * plane, *gs = go + size_t(bh) * D * plane;
    const float c2 = scale * kLog2e;

    float qreg[NO][D / 4], greg[NO][D / 4];
    f32x4 acc[NO][D / 16];
    float L2[NO], Dn[NO];
#pragma unroll
    for (int o = 0; o < NO; ++o) {
#pragma unroll
        for (int mt = 0; mt < D / 16; ++mt) acc[o][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        L2[o] = 0.f;
        Dn[o] = 0.f;
        float dsum = 0.f;
        const size_t at = size_t(h) * nlon + (W0 + 16 * o + n);
        const bool own = active && W0 + 16 * o < nlon;
#pragma unroll
        for (int kb = 0; kb < D / 4; ++kb) {
            const size_t e = size_t(4 * kb + g) * plane + at;
            qreg[o][kb] = own ? ldx(qs + e) : 0.f;
            greg[o][kb] = own ? ldx(gs + e) : 0.f;
            dsum = fmaf(greg[o][kb], own ? ldx(os + e) : 0.f, dsum);
        }
        dsum = group_sum(dsum);
        if (own) {
            if (g == 0) Dws[size_t(bh) * plane + at] = dsum;
            Dn[o] = -dsum;
            L2[o] = (lse[size_t(bh) * plane + at] - t.ln_omega_ref) * kLog2e;
        }
    }
    BandRows rows;
    rows.load(t.band_lo, t.band_n, t.cnt, t.band_max, t.omega_rel, nlon, first, t.nlat_out, h, active, lane);
    for (int i = tid; i < 2 * G::TILE; i += 256) lds[i] = 0.f;

    const int nrow = rows.rmax - rows.rmin + 1;
    int ri = 0, s = 0;
    RowPlan cur;
    f32x4 rk[G::NP], rv[G::NP];
    bool more = nrow > 0;
    if (more) {
        cur.template set<G::OW, G::SW>(rows.hwmax(0), nlon, Wb);
        load_stage<D, NO>(rk, ks, plane, rows.rmin, nlon, cur.Xs0, tid);
        load_stage<D, NO>(rv, vs, plane, rows.rmin, nlon, cur.Xs0, tid);
    }
    while (more) {
        __syncthreads();
        store_stage<D, NO>(Kc, rk, tid);
        store_stage<D, NO>(Vc, rv, tid);
        __syncthreads();
        const int Xst = cur.Xs0 + s * G::SW;
        const RowPlan now = cur;
        const int rnow = ri;
        if (++s == cur.nst) {
            s = 0;
            ++ri;
            if (ri < nrow) cur.template set<G::OW, G::SW>(rows.hwmax(ri), nlon, Wb);
        }
        more = ri < nrow;
        if (more) {
            load_stage<D, NO>(rk, ks, plane, rows.rmin + ri, nlon, cur.Xs0 + s * G::SW, tid);
            load_stage<D, NO>(rv, vs, plane, rows.rmin + ri, nlon, cur.Xs0 + s * G::SW, tid);
        }
        const int hw = rows.hw(rnow);
        if (hw < 0) continue;
        const float lw2 = rows.lw2(rnow);
        const int Xlim = min(Xst + G::SW + (now.multi ? 0 : 32), now.Xend);
#pragma unroll
        for (int o = 0; o < NO; ++o) {
            if (W0 + 16 * o >= nlon) break;
            const int Wo = Wb + 16 * o;
            const int T0 = now.multi ? Xst : (Wo - hw) & ~3;
            const int Tend = now.multi ? Xlim : Wo + 16 + hw;
            const float bias = lw2 - L2[o];
            for (int Xt = T0; Xt < Tend; Xt += 16) {
                TilePos tp;
                tp.set(Xt, Wo, hw, nlon, now.multi);
                if (!tp.touch) continue;
                const int col0 = Xt - Xst;
                const float *kp = Kc + g * G::PITCH + col0 + n, *vp = Vc + g * G::PITCH + col0 + n;
                f32x4 sc = {0.f, 0.f, 0.f, 0.f}, dp = {Dn[o], Dn[o], Dn[o], Dn[o]};
#pragma unroll
                for (int kb = 0; kb < D / 4; ++kb) {
                    sc = mfma4(kp[kb * 4 * G::PITCH + 4 * (kb & 3)], qreg[o][kb], sc);
                    dp = mfma4(vp[kb * 4 * G::PITCH + 4 * (kb & 3)], greg[o][kb], dp);
                }
                float ds[4];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) ds[rr] = __builtin_amdgcn_exp2f(fmaf(sc[rr], c2, bias)) * dp[rr];
                if (tp.mask) {
                    bool keep[4];
                    band_mask(keep, tp, hw, nlon, now.multi, 4 * g - n + hw);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) ds[rr] = keep[rr] ? ds[rr] : 0.f;
                }
                const float *kq = Kc + n * G::PITCH + 4 * ((n >> 2) & 3) + col0 + 4 * g;
                f32x4 ka[D / 16];
#pragma unroll
                for (int mt = 0; mt < D / 16; ++mt) ka[mt] = *reinterpret_cast<const f32x4 *>(kq + mt * 16 * G::PITCH);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int mt = 0; mt < D / 16; ++mt) acc[o][mt] = mfma4(ka[mt][j], ds[j], acc[o][mt]);
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int o = 0; o < NO; ++o) {
        if (W0 + 16 * o >= nlon) break;
        T *ob = dq + size_t(bh) * D * plane + size_t(h) * nlon + (W0 + 16 * o + n);
#pragma unroll
        for (int mt = 0; mt < D / 16; ++mt)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) stx(ob + size_t(16 * mt + 4 * g + rr) * plane, acc[o][mt][rr] * scale);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Backward, key side: owners are input points, the transposed band gives the output latitudes; q, dout, lse and D
// of a stage's outputs are staged together.
template <class T, int D, int NO>
__global__ void __launch_bounds__(256, 2)
nattn_bwd_dkdv_band(S2DeviceTables t, int nbh, float scale, const T *__restrict__ q, const T *__restrict__ k,
                    const T *__restrict__ v, const float *__restrict__ lse, const T *__restrict__ go,
                    const float *__restrict__ Dws, T *__restrict__ dk, T *__restrict__ dv)
{
    using G = Geo<D, NO>;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    float *Qc = lds, *Gc = lds + G::TILE, *Ls = lds + 2 * G::TILE, *Dn = Ls + G::COLS;
    const int nlon = t.nlon_in, ngrp = (nlon + G::OW - 1) / G::OW, nseg = (t.nlat_in + 3) >> 2;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int bh = id % nbh, seg = segment_of(id / nbh, nseg);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int first = 4 * seg, hp = first + wave;
    const bool active = hp < t.nlat_in;
    const int W0 = grp * G::OW, Wb = nlon + W0;
    const size_t plane = size_t(t.nlat_in) * nlon;
    const T *qs = q + size_t(bh) * D * plane, *ks = k + size_t(bh) * D * plane, *vs = v + size_t(bh) * D * plane;
    const T *gs = go + size_t(bh) * D * plane;
    const float *ls = lse + size_t(bh) * plane, *Ds = Dws + size_t(bh) * plane;
    const float c2 = scale * kLog2e, lref = t.ln_omega_ref;
    const float lw2 = active ? __log2f(t.omega_rel[hp]) : 0.f;     // -inf for a latitude of weight zero: p = 0

    float kreg[NO][D / 4], vreg[NO][D / 4];
    f32x4 adk[NO][D / 16], adv[NO][D / 16];
#pragma unroll
    for (int o = 0; o < NO; ++o) {
#pragma unroll
        for (int mt = 0; mt < D / 16; ++mt) adk[o][mt] = adv[o][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < D / 4; ++kb) {
            const size_t e = size_t(4 * kb + g) * plane + size_t(hp) * nlon + (W0 + 16 * o + n);
            kreg[o][kb] = active && W0 + 16 * o < nlon ? ldx(ks + e) : 0.f;
            vreg[o][kb] = active && W0 + 16 * o < nlon ? ldx(vs + e) : 0.f;
        }
    }
    BandRows rows;
    rows.load(t.tband_lo, t.tband_n, t.tcnt, t.tband_max, t.omega_rel, nlon, first, t.nlat_in, hp, active, lane);
    for (int i = tid; i < 2 * G::TILE + 2 * G::COLS; i += 256) lds[i] = 0.f;
    auto load_stat = [&](int lat, int Xs) -> float {      // threads 0 .. SW-1: logsumexp (base 2, relative), SW .. 2 SW-1: -D
        const int j = tid < G::SW ? tid : tid - G::SW;
        const size_t at = size_t(lat) * nlon + wrap3(Xs + j, nlon);
        if (tid >= 2 * G::SW) return 0.f;
        return tid < G::SW ? (ls[at] - lref) * kLog2e : -Ds[at];
    };

    const int nrow = rows.rmax - rows.rmin + 1;
    int ri = 0, s = 0;
    RowPlan cur;
    f32x4 rq[G::NP], rg[G::NP];
    float rs = 0.f;
    bool more = nrow > 0;
    if (more) {
        cur.template set<G::OW, G::SW>(rows.hwmax(0), nlon, Wb);
        load_stage<D, NO>(rq, qs, plane, rows.rmin, nlon, cur.Xs0, tid);
        load_stage<D, NO>(rg, gs, plane, rows.rmin, nlon, cur.Xs0, tid);
        rs = load_stat(rows.rmin, cur.Xs0);
    }
    while (more) {
        __syncthreads();
        store_stage<D, NO>(Qc, rq, tid);
        store_stage<D, NO>(Gc, rg, tid);
        if (tid < 2 * G::SW) (tid < G::SW ? Ls : Dn - G::SW)[tid] = rs;
        __syncthreads();
        const int Xst = cur.Xs0 + s * G::SW;
        const RowPlan now = cur;
        const int rnow = ri;
        if (++s == cur.nst) {
            s = 0;
            ++ri;
            if (ri < nrow) cur.template set<G::OW, G::SW>(rows.hwmax(ri), nlon, Wb);
        }
        more = ri < nrow;
        if (more) {
            load_stage<D, NO>(rq, qs, plane, rows.rmin + ri, nlon, cur.Xs0 + s * G::SW, tid);
            load_stage<D, NO>(rg, gs, plane, rows.rmin + ri, nlon, cur.Xs0 + s * G::SW, tid);
            rs = load_stat(rows.rmin + ri, cur.Xs0 + s * G::SW);
        }
        const int hw = rows.hw(rnow);
        if (hw < 0) continue;
        const int Xlim = min(Xst + G::SW + (now.multi ? 0 : 32), now.Xend);
#pragma unroll
        for (int o = 0; o < NO; ++o) {
            if (W0 + 16 * o >= nlon) break;
            const int Wo = Wb + 16 * o;
            const int T0 = now.multi ? Xst : (Wo - hw) & ~3;
            const int Tend = now.multi ? Xlim : Wo + 16 + hw;
            for (int Xt = T0; Xt < Tend; Xt += 16) {
                TilePos tp;
                tp.set(Xt, Wo, hw, nlon, now.multi);
                if (!tp.touch) continue;
                const int col0 = Xt - Xst;
                const float *qp = Qc + g * G::PITCH + col0 + n, *gp = Gc + g * G::PITCH + col0 + n;
                const f32x4 L = *reinterpret_cast<const f32x4 *>(Ls + col0 + 4 * g);
                f32x4 sc = {0.f, 0.f, 0.f, 0.f}, dp = *reinterpret_cast<const f32x4 *>(Dn + col0 + 4 * g);
#pragma unroll
                for (int kb = 0; kb < D / 4; ++kb) {
                    sc = mfma4(qp[kb * 4 * G::PITCH + 4 * (kb & 3)], kreg[o][kb], sc);
                    dp = mfma4(gp[kb * 4 * G::PITCH + 4 * (kb & 3)], vreg[o][kb], dp);
                }
                float pr[4], ds[4];
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    pr[rr] = __builtin_amdgcn_exp2f(fmaf(sc[rr], c2, lw2 - L[rr]));
                    ds[rr] = pr[rr] * dp[rr];
                }
                if (tp.mask) {
                    bool keep[4];
                    band_mask(keep, tp, hw, nlon, now.multi, 4 * g - n + hw);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        pr[rr] = keep[rr] ? pr[rr] : 0.f;
                        ds[rr] = keep[rr] ? ds[rr] : 0.f;
                    }
                }
                const float *gq = Gc + n * G::PITCH + 4 * ((n >> 2) & 3) + col0 + 4 * g, *qq = Qc + n * G::PITCH + 4 * ((n >> 2) & 3) + col0 + 4 * g;
                f32x4 ga[D / 16], qa[D / 16];
#pragma unroll
                for (int mt = 0; mt < D / 16; ++mt) {
                    ga[mt] = *reinterpret_cast<const f32x4 *>(gq + mt * 16 * G::PITCH);
                    qa[mt] = *reinterpret_cast<const f32x4 *>(qq + mt * 16 * G::PITCH);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int mt = 0; mt < D / 16; ++mt) {
                        adv[o][mt] = mfma4(ga[mt][j], pr[j], adv[o][mt]);
                        adk[o][mt] = mfma4(qa[mt][j], ds[j], adk[o][mt]);
                    }
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int o = 0; o < NO; ++o) {
        if (W0 + 16 * o >= nlon) break;
        const size_t at = size_t(bh) * D * plane + size_t(hp) * nlon + (W0 + 16 * o + n);
#pragma unroll
        for (int mt = 0; mt < D / 16; ++mt)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                stx(dk + at + size_t(16 * mt + 4 * g + rr) * plane, adk[o][mt][rr] * scale);
                stx(dv + at + size_t(16 * mt + 4 * g + rr) * plane, adv[o][mt][rr]);
            }
    }
}

template <int D, int NO>
constexpr size_t fwd_lds() { return size_t(2) * Geo<D, NO>::TILE * sizeof(float); }
template <int D, int NO>
constexpr size_t dkdv_lds() { return (size_t(2) * Geo<D, NO>::TILE + 2 * Geo<D, NO>::COLS) * sizeof(float); }

template <class T, int D, int NO>
int configure_one()
{
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(nattn_fwd_band<T, D, NO>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, int(fwd_lds<D, NO>())) != hipSuccess)
        return -1;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(nattn_bwd_dq_band<T, D, NO>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, int(fwd_lds<D, NO>())) != hipSuccess)
        return -1;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(nattn_bwd_dkdv_band<T, D, NO>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, int(dkdv_lds<D, NO>())) != hipSuccess)
        return -1;
    return 0;
}

template <int D, int NO>
unsigned blocks(const S2DeviceTables &t, int nbh, int nlat)
{
    return unsigned(long((nlat + 3) / 4) * nbh * ((t.nlon_in + Geo<D, NO>::OW - 1) / Geo<D, NO>::OW));
}

// Owner tiles per wavefront.  d = 32 and 64: two (for d = 32 four were measured too: 3.13 against 2.88 ms on workload 3,
// 0.58 against 0.41 ms on workload 2 with its 256 workgroups: smaller tiles in LDS and fewer registers put more
// workgroups on a compute unit, which outweighs staging 96 columns per 32 owners instead of 128 per 64).  d = 16: four
// (two measured the same on workload 8), two while a launch would have fewer than two workgroups per compute unit.
// d = 32 on launches that would still leave the device half empty (fewer than four workgroups per compute unit): one.
inline int num_cus()
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
inline bool tiny32(const S2DeviceTables &t, int nbh, int nlat)
{
    return blocks<32, 2>(t, nbh, nlat) < unsigned(4 * num_cus());
}
inline bool narrow16(const S2DeviceTables &t, int nbh, int nlat)
{
    return blocks<16, 4>(t, nbh, nlat) < unsigned(2 * num_cus());
}

double pair_count(const S2DeviceTables &t, bool fwd_side, int nbh)
{
    const double *p = fwd_side ? t.fwd_pairs : t.bwd_pairs;
    return nbh * (p[0] + p[1] + p[2] + p[3]);
}

template <class T, int D, int NO>
void launch_fwd(const S2DeviceTables &t, int nbh, float scale, const T *q, const T *k, const T *v, T *out, float *lse,
                hipStream_t st)
{
    S2TraceScope tr(sizeof(T) == 2 ? "nattn_fwd_band<bf16>" : "nattn_fwd_band", pair_count(t, true, nbh), st);
    const unsigned nblk = blocks<D, NO>(t, nbh, t.nlat_out);
    const size_t bytes = fwd_lds<D, NO>();
    hipLaunchKernelGGL((nattn_fwd_band<T, D, NO>), dim3(nblk), dim3(256), bytes, st, t, nbh, scale * kLog2e, q, k, v, out,
                       lse);
}
template <class T, int D, int NO>
void launch_dq(const S2DeviceTables &t, int nbh, float scale, const T *q, const T *k, const T *v, const T *o,
               const float *lse, const T *go, T *dq, float *Dws, hipStream_t st)
{
    S2TraceScope tr(sizeof(T) == 2 ? "nattn_bwd_dq_band<bf16>" : "nattn_bwd_dq_band", pair_count(t, true, nbh), st);
    const unsigned nblk = blocks<D, NO>(t, nbh, t.nlat_out);
    const size_t bytes = fwd_lds<D, NO>();
    hipLaunchKernelGGL((nattn_bwd_dq_band<T, D, NO>), dim3(nblk), dim3(256), bytes, st, t, nbh, scale, q, k, v, o, lse, go,
                       dq, Dws);
}
template <class T, int D, int NO>
void launch_dkdv(const S2DeviceTables &t, int nbh, float scale, const T *q, const T *k, const T *v, const float *lse,
                 const T *go, const float *Dws, T *dk, T *dv, hipStream_t st)
{
    S2TraceScope tr(sizeof(T) == 2 ? "nattn_bwd_dkdv_band<bf16>" : "nattn_bwd_dkdv_band", pair_count(t, false, nbh), st);
    const unsigned nblk = blocks<D, NO>(t, nbh, t.nlat_in);
    const size_t bytes = dkdv_lds<D, NO>();
    hipLaunchKernelGGL((nattn_bwd_dkdv_band<T, D, NO>), dim3(nblk), dim3(256), bytes, st, t, nbh, scale, q, k, v, lse, go,
                       Dws, dk, dv);
}

template <class T>
void fwd_by_d(const S2DeviceTables &t, int nbh, int d, float scale, const void *q, const void *k, const void *v, void *out,
              float *lse, hipStream_t st)
{
    const T *Q = static_cast<const T *>(q), *K = static_cast<const T *>(k), *V = static_cast<const T *>(v);
    T *O = static_cast<T *>(out);
    if (d == 16 && narrow16(t, nbh, t.nlat_out)) launch_fwd<T, 16, 2>(t, nbh, scale, Q, K, V, O, lse, st);
    else if (d == 16) launch_fwd<T, 16, 4>(t, nbh, scale, Q, K, V, O, lse, st);
    else if (d == 32 && tiny32(t, nbh, t.nlat_out)) launch_fwd<T, 32, 1>(t, nbh, scale, Q, K, V, O, lse, st);
    else if (d == 32) launch_fwd<T, 32, 2>(t, nbh, scale, Q, K, V, O, lse, st);
    else launch_fwd<T, 64, 2>(t, nbh, scale, Q, K, V, O, lse, st);
}
template <class T>
void dq_by_d(const S2DeviceTables &t, int nbh, int d, float scale, const void *q, const void *k, const void *v,
             const void *o, const float *lse, const void *go, void *dq, float *Dws, hipStream_t st)
{
    const T *Q = static_cast<const T *>(q), *K = static_cast<const T *>(k), *V = static_cast<const T *>(v);
    const T *O = static_cast<const T *>(o), *G = static_cast<const T *>(go);
    T *DQ = static_cast<T *>(dq);
    if (d == 16 && narrow16(t, nbh, t.nlat_out)) launch_dq<T, 16, 2>(t, nbh, scale, Q, K, V, O, lse, G, DQ, Dws, st);
    else if (d == 16) launch_dq<T, 16, 4>(t, nbh, scale, Q, K, V, O, lse, G, DQ, Dws, st);
    else if (d == 32 && tiny32(t, nbh, t.nlat_out)) launch_dq<T, 32, 1>(t, nbh, scale, Q, K, V, O, lse, G, DQ, Dws, st);
    else if (d == 32) launch_dq<T, 32, 2>(t, nbh, scale, Q, K, V, O, lse, G, DQ, Dws, st);
    else launch_dq<T, 64, 2>(t, nbh, scale, Q, K, V, O, lse, G, DQ, Dws, st);
}
template <class T>
void dkdv_by_d(const S2DeviceTables &t, int nbh, int d, float scale, const void *q, const void *k, const void *v,
               const float *lse, const void *go, const float *Dws, void *dk, void *dv, hipStream_t st)
{
    const T *Q = static_cast<const T *>(q), *K = static_cast<const T *>(k), *V = static_cast<const T *>(v);
    const T *G = static_cast<const T *>(go);
    T *DK = static_cast<T *>(dk), *DV = static_cast<T *>(dv);
    if (d == 16 && narrow16(t, nbh, t.nlat_in)) launch_dkdv<T, 16, 2>(t, nbh, scale, Q, K, V, lse, G, Dws, DK, DV, st);
    else if (d == 16) launch_dkdv<T, 16, 4>(t, nbh, scale, Q, K, V, lse, G, Dws, DK, DV, st);
    else if (d == 32 && tiny32(t, nbh, t.nlat_in)) launch_dkdv<T, 32, 1>(t, nbh, scale, Q, K, V, lse, G, Dws, DK, DV, st);
    else if (d == 32) launch_dkdv<T, 32, 2>(t, nbh, scale, Q, K, V, lse, G, Dws, DK, DV, st);
    else launch_dkdv<T, 64, 2>(t, nbh, scale, Q, K, V, lse, G, Dws, DK, DV, st);
}

}  // namespace

int s2_nattn_band_configure()
{
    return configure_one<float, 16, 4>() || configure_one<float, 16, 2>() || configure_one<float, 32, 2>() ||
           configure_one<float, 32, 1>() || configure_one<bf16raw, 32, 1>() ||
           configure_one<float, 64, 2>() || configure_one<bf16raw, 16, 4>() || configure_one<bf16raw, 16, 2>() ||
           configure_one<bf16raw, 32, 2>() || configure_one<bf16raw, 64, 2>();
}

bool s2_nattn_band_supported(const S2DeviceTables &t, int d, int e)
{
    return d == e && (d == 16 || d == 32 || d == 64) && t.upscale == 1 && t.pscale == 1 && t.nlon_in == t.nlon_out &&
           t.nlat_in == t.nlat_out && t.nlon_in % 16 == 0 && t.nlon_in >= 64 && t.band_rows_ok &&
           !s2_debug_flag(S2_DEBUG_NO_MFMA);
}

int s2_nattn_fwd_band(const S2DeviceTables &t, int nbh, int d, int, float scale, const float *q, const float *k,
                      const float *v, float *out, float *lse, hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    fwd_by_d<float>(t, nbh, d, scale, q, k, v, out, lse, st);
    return 0;
}

int s2_nattn_bwd_band(const S2DeviceTables &t, int nbh, int d, int, float scale, const float *q, const float *k,
                      const float *v, const float *o, const float *lse, const float *go, float *dq, float *dk, float *dv,
                      float *Dws, hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    dq_by_d<float>(t, nbh, d, scale, q, k, v, o, lse, go, dq, Dws, st);
    dkdv_by_d<float>(t, nbh, d, scale, q, k, v, lse, go, Dws, dk, dv, st);
    return 0;
}

// bf16 tensors on the same kernels (float32 arithmetic on the fp32 matrix cores, bf16 loads and stores)
int s2_nattn_fwd_band_bf16(const S2DeviceTables &t, int nbh, int d, int, float scale, const void *q, const void *k,
                           const void *v, void *out, float *lse, hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    fwd_by_d<bf16raw>(t, nbh, d, scale, q, k, v, out, lse, st);
    return 0;
}
int s2_nattn_bwd_dq_band_bf16(const S2DeviceTables &t, int nbh, int d, int, float scale, const void *q, const void *k,
                              const void *v, const void *o, const float *lse, const void *go, void *dq, float *Dws,
                              hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    dq_by_d<bf16raw>(t, nbh, d, scale, q, k, v, o, lse, go, dq, Dws, st);
    return 0;
}
int s2_nattn_bwd_dkdv_band_bf16(const S2DeviceTables &t, int nbh, int d, int, float scale, const void *q, const void *k,
                                const void *v, const float *lse, const void *go, const float *Dws, void *dk, void *dv,
                                hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    dkdv_by_d<bf16raw>(t, nbh, d, scale, q, k, v, lse, go, Dws, dk, dv, st);
    return 0;
}
