// Neighborhood attention forward for the latitudes near the poles, on the fp32 matrix cores.
//
// Near a pole the geodesic disk covers whole latitude circles (App. B.3: the indicator row is
// all ones), so for those output latitudes the neighborhood sum IS a dense contraction: every
// output of the row against every input column of 5..9 input rows.  That part of the path runs
// as a flash-style kernel on v_mfma_f32_32x32x2_f32 (products and sums in float32, same
// arithmetic class as the vector path); partial arcs in the same band are handled by masking.
// The rest of the sphere, where a disk cuts ~9 of 256 columns, stays on the vector ALU.
//
// One workgroup = one (batch, head, output latitude); one wavefront = 32 consecutive outputs.
// Input rows are streamed as super-tiles of 64 columns x 32 channels of K and V, staged once
// per workgroup in LDS (LDS-direct loads, double buffered) and shared by all wavefronts.
//
//   S^T = K Q^T   two 32x32 tiles (64 inputs x 32 outputs), 16 MFMAs each (2 channels per MFMA)
//   O^T += V^T P^T  32 MFMAs (2 input columns per MFMA)
//
// Tile row r of S^T tile mt is mapped to super-tile column 32*((r>>2)&1) + 16*mt + 4*(r>>3) + (r&3):
// in the result layout lane (output, half hl) then holds columns 32*hl + 16*mt + i in register i, so
// the probabilities feed the second product straight from registers, and the two halves of a
// wavefront read LDS columns 32 apart (disjoint banks).
#include <cstdlib>

#include "s2_nattn_kernels.h"

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

constexpr int kD = 32;          // channels
constexpr int kTileCols = 64;   // input columns per super-tile
constexpr int kPK = 80;         // K tile pitch: = 16 mod 64, the two channel rows of one MFMA step hit disjoint banks
constexpr int kPV = 65;         // V tile pitch: odd, the 32 channel rows read by one wavefront hit 32 banks
constexpr int kTileFloats = kD * kPK + kD * kPV;

__device__ __forceinline__ f32x16 mfma(float a, float b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Read of a grid table entry through the scalar cache.  The tables are never written by a kernel, but the
// compiler cannot know that once the kernel has stored results, and would use vector loads whose
// completion wait (vmcnt) also waits for the LDS-direct copies of the next tile that were just requested.
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

__device__ __forceinline__ int wrapn(int x, int n)
{
    x = x < 0 ? x + n : x;
    return x >= n ? x - n : x;
}

// Each wavefront copies its share of the 64 channel rows (K: 0..31, V: 32..63) of super-tile
// columns x0 .. x0+63 (mod nlon) of input latitude hp: lane = column.
__device__ __forceinline__ void stage_tile(const float *kb, const float *vb, size_t si, int x0, int nlon, float *tile,
                                           int wave, int nwaves, int lane)
{
    const unsigned voff = 4u * unsigned(wrapn(x0 + lane, nlon));
    for (int r = wave; r < 2 * kD; r += nwaves) {
        const bool isv = r >= kD;
        const int c = isv ? r - kD : r;
        const char *rb = reinterpret_cast<const char *>((isv ? vb : kb) + size_t(c) * si);
        float *dst = isv ? tile + kD * kPK + c * kPV : tile + c * kPK;
        __builtin_amdgcn_global_load_lds((gptr_t)(rb + voff), (lptr_t)dst, 4, 0, 0);
    }
}

// NSUB adjacent super-tiles are staged (and consumed) per barrier: half as many workgroup-wide waits for NSUB = 2.
template <int NSUB>
__global__ void __launch_bounds__(1024)
nattn_fwd_mfma(S2DeviceTables t, int nbh, int nrows, int rgroups, float qscale, const float *__restrict__ q,
               const float *__restrict__ k, const float *__restrict__ v, float *__restrict__ out,
               float *__restrict__ lse)
{
    // rgroups = 2 (launches with fewer workgroups than compute units): the workgroup holds two sets of wavefronts,
    // each set walks half of the band of input latitudes with its own tiles, and the two partial softmax states
    // are merged through LDS at the end: twice the wavefronts per SIMD to overlap the matrix-instruction chains.
    extern __shared__ __attribute__((aligned(16))) float smem_all[];
    const int nwaves = (blockDim.x >> 6) / rgroups;   // wavefronts per set = nlon_out / 32
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int grp = wave_all / nwaves, wave = wave_all - grp * nwaves;
    float *smem = smem_all + grp * (2 * NSUB * kTileFloats);
    const int col = lane & 31, hl = lane >> 5;
    const int nlon = t.nlon_in;                       // equal longitude counts
    const int bh = blockIdx.x / nrows;
    const int h = t.row_order[blockIdx.x - bh * nrows];
    const int w = wave * 32 + col;                    // this lane's output longitude
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t io = size_t(h) * t.nlon_out + w;

    // B operand of S^T = K Q^T: lane (output, hl) supplies channel 2s + hl at step s
    float qop[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) qop[s] = q[(size_t(bh) * kD + 2 * s + hl) * so + io] * qscale;
    f32x16 o = {0};
    float m = -INFINITY, l = 0.f;
    // LDS column (within a super-tile) of S^T tile row `col`, tile mt = 0: see header
    const int arow = 32 * ((col >> 2) & 1) + 4 * (col >> 3) + (col & 3);

    const int nb_all = t.band_n[h];
    const int b_lo = grp * nb_all / rgroups, nb = (grp + 1) * nb_all / rgroups - b_lo;   // this set's band rows
    const int hp0 = t.band_lo[h] + b_lo;
    const int ntile = nlon / (kTileCols * NSUB);
    const int total = nb * ntile, total_max = ((nb_all + rgroups - 1) / rgroups) * ntile;
    // prologue: stage the first super-tile
    if (total > 0) {
        const float *kb = k + size_t(bh) * kD * si + size_t(hp0) * nlon;
        const float *vb = v + size_t(bh) * kD * si + size_t(hp0) * nlon;
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
            stage_tile(kb, vb, si, kTileCols * sub, nlon, smem + sub * kTileFloats, wave, nwaves, lane);
    }
    for (int it = 0; it < total_max; ++it) {
        const int b = it / ntile, xg = (it - b * ntile) * kTileCols * NSUB;
        const int hp = hp0 + b;
        float *tiles = smem + (it & 1) * NSUB * kTileFloats;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();     // tile `it` is complete; everyone has finished reading tile it-1
        if (it >= total) continue;   // (the other set has one more band row)
        if (it + 1 < total) {
            const int b2 = (it + 1) / ntile, x2 = (it + 1 - b2 * ntile) * kTileCols * NSUB;
            const float *kb = k + size_t(bh) * kD * si + size_t(hp0 + b2) * nlon;
            const float *vb = v + size_t(bh) * kD * si + size_t(hp0 + b2) * nlon;
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
                stage_tile(kb, vb, si, x2 + kTileCols * sub, nlon,
                           smem + (((it + 1) & 1) * NSUB + sub) * kTileFloats, wave, nwaves, lane);
        }
        const int c = table_i(t.cnt, h * t.band_max + b_lo + b);
        const bool full = c == nlon;
        const int lo = full ? 0 : -((c - 1) >> 1);
        const float wq = table_f(t.omega_rel, hp);
#pragma unroll 1
        for (int sub = 0; sub < NSUB; ++sub) {
        const int x0 = xg + kTileCols * sub;
        const float *tile = tiles + sub * kTileFloats;
        // does this wavefront's span of outputs touch the super-tile at all?
        if (!full) {
            // columns needed by outputs wave*32 .. wave*32+31: [wave*32 + lo, wave*32 + 31 + lo + c) on the circle
            const int need0 = wrapn(wave * 32 + lo, nlon), len = c + 31;
            const int rel = wrapn(x0 - need0, nlon);          // tile start relative to the needed range
            const bool overlap = rel < len || rel + kTileCols > nlon;
            if (!overlap) continue;
        }
        const float *tk = tile, *tv = tile + kD * kPK;
        f32x16 s0 = {0}, s1 = {0};
        {
            // operands of all 16 steps are requested up front, in two halves: the matrix products of the first half
            // cover the LDS latency of the second
            float a0[16], a1[16];
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                a0[s] = tk[(2 * s + hl) * kPK + arow];
                a1[s] = tk[(2 * s + hl) * kPK + arow + 16];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                s0 = mfma(a0[s], qop[s], s0);
                s1 = mfma(a1[s], qop[s], s1);
            }
        }
        float p[32];
#pragma unroll
        for (int i = 0; i < 16; ++i) { p[i] = s0[i]; p[16 + i] = s1[i]; }
        if (!full) {
            // register i of tile mt is super-tile column 32*hl + 16*mt + i; valid iff its offset from the
            // output's own longitude lies in [lo, lo + c)
            const int base = (x0 + 32 * hl - w - lo + 2 * nlon) % nlon;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                int rel = base + i;           // (16*mt + i) is just i for i in 0..31
                rel = rel >= nlon ? rel - nlon : rel;
                p[i] = rel < c ? p[i] : -INFINITY;
            }
        }
        float mloc = -INFINITY;
#pragma unroll
        for (int i = 0; i < 32; ++i) mloc = fmaxf(mloc, p[i]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        if (__any(mloc > m + 8.f)) {
            const float m_new = mloc > m + 8.f ? mloc : m;
            // m = -inf until this output has seen a valid column: then corr = 0 (or 1 while it still has none)
            const float corr = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m - m_new);
            m = m_new;
            l *= corr;
#pragma unroll
            for (int i = 0; i < 16; ++i) o[i] *= corr;
        }
        const float mm = m == -INFINITY ? 0.f : m;   // all 64 columns masked for this output so far: p = exp2(-inf) = 0
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            p[i] = wq * __builtin_amdgcn_exp2f(p[i] - mm);
            l += p[i];
        }
        // O^T += V^T P^T: step i contracts super-tile columns (32*hl + i); A = V[channel = col][that column]
#pragma unroll
        for (int i = 0; i < 32; ++i) o = mfma(tv[col * kPV + 32 * hl + i], p[i], o);
        }
    }
    if (rgroups > 1) {
        // the second set hands its partial state (o, m, l per lane) to the first through LDS
        __syncthreads();     // everybody is done with the tiles
        float *slot = smem_all + wave * 64 + lane;
        const int pitch = nwaves * 64;
        if (grp == 1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) slot[i * pitch] = o[i];
            slot[16 * pitch] = m;
            slot[17 * pitch] = l;
        }
        __syncthreads();
        if (grp != 0) return;
        const float mo = slot[16 * pitch], lo2 = slot[17 * pitch];
        const float M = fmaxf(m, mo);
        // a set that saw no valid column has m = -inf, l = 0: its factor must be 0, never NaN
        const float fa = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - M);
        const float fb = mo == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mo - M);
        m = M;
        l = l * fa + lo2 * fb;
#pragma unroll
        for (int i = 0; i < 16; ++i) o[i] = o[i] * fa + slot[i * pitch] * fb;
    }
    l += __shfl_xor(l, 32);
    const float inv = 1.f / l;
    // lane (output, hl) holds channels 8*(i/4) + 4*hl + i%4 in register i
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int ch = 8 * (i >> 2) + 4 * hl + (i & 3);
        out[(size_t(bh) * kD + ch) * so + io] = o[i] * inv;
    }
    if (hl == 0) lse[size_t(bh) * so + io] = (m + log2f(l * t.omega_ref)) * 0.6931471805599453f;
}

// ------------------------------------------------------------------ backward, dq ----------
//
// Same tiling for dq_i = scale sum_j dS_ij k_j on the dense latitudes:
//   S^T = K Q^T, dP^T = V dout^T (2 x 32 MFMAs), dS = p (dP - D) in registers,
//   dQ^T += K^T-read-by-channel dS^T (32 MFMAs).
// K is read both ways (by column for S^T, by channel for dQ^T); a pitch of 79 floats keeps both
// patterns (almost) free of bank conflicts: 79 = 15 mod 64 is odd, so 32 channel rows hit 32 banks,
// and the two channel rows of one S^T step are 15 banks apart (one of 16 columns collides).  V is only
// read by column: pitch 80 as in the forward.  With these pitches two workgroups with four tiles each
// (two super-tiles per barrier, double buffered) still fit one compute unit's LDS.

constexpr int kPC = 77;                  // dk/dv kernel: q and dout rows are both read both ways; 77 = 13 mod 64 is
                                         // odd (32 channel rows hit 32 banks) and small enough for four tiles per
                                         // workgroup at two workgroups per compute unit
constexpr int kPQK = 79, kPQV = 80;
constexpr int kTileB = kD * kPQK + kD * kPQV;     // K rows then V rows

__device__ __forceinline__ void stage_tile_b(const float *ab, const float *bb, size_t stride, int x0, int ncol,
                                             float *tile, int wave, int nwaves, int lane)
{
    const unsigned voff = 4u * unsigned(wrapn(x0 + lane, ncol));
    for (int r = wave; r < 2 * kD; r += nwaves) {
        const int c = r >= kD ? r - kD : r;
        const char *rb = reinterpret_cast<const char *>((r >= kD ? bb : ab) + size_t(c) * stride);
        __builtin_amdgcn_global_load_lds((gptr_t)(rb + voff), (lptr_t)(r >= kD ? tile + kD * kPQK + c * kPQV : tile + c * kPQK), 4, 0, 0);
    }
}

template <int NSUB>
__global__ void __launch_bounds__(1024)
nattn_bwd_dq_mfma(S2DeviceTables t, int nbh, int nrows, int rgroups, float scale, const float *__restrict__ q,
                  const float *__restrict__ k, const float *__restrict__ v, const float *__restrict__ outp,
                  const float *__restrict__ lse, const float *__restrict__ go, float *__restrict__ dq,
                  float *__restrict__ Dws)
{
    // rgroups = 2: two sets of wavefronts, each with half of the band rows and its own tiles (see the forward)
    extern __shared__ __attribute__((aligned(16))) float smem_all[];
    const int nwaves = (blockDim.x >> 6) / rgroups;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int grp = wave_all / nwaves, wave = wave_all - grp * nwaves;
    float *smem = smem_all + grp * (2 * NSUB * kTileB);
    const int col = lane & 31, hl = lane >> 5;
    const int nlon = t.nlon_in;
    const int bh = blockIdx.x / nrows;
    const int h = t.row_order[blockIdx.x - bh * nrows];
    const int w = wave * 32 + col;
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t io = size_t(h) * t.nlon_out + w;
    const float qscale = scale * 1.4426950408889634f;

    float qop[16], gop[16], Dp = 0.f;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const size_t off = (size_t(bh) * kD + 2 * s + hl) * so + io;
        qop[s] = q[off] * qscale;
        gop[s] = go[off];
        Dp = fmaf(gop[s], outp[off], Dp);
    }
    const float Di = Dp + __shfl_xor(Dp, 32);        // D_i = dout_i . out_i over all 32 channels
    if (hl == 0 && grp == 0) Dws[size_t(bh) * so + io] = Di;
    const float lse2 = (lse[size_t(bh) * so + io] - t.ln_omega_ref) * 1.4426950408889634f;
    f32x16 acc = {0};
    const int arow = 32 * ((col >> 2) & 1) + 4 * (col >> 3) + (col & 3);

    const int nb_all = t.band_n[h];
    const int b_lo = grp * nb_all / rgroups, nb = (grp + 1) * nb_all / rgroups - b_lo;
    const int hp0 = t.band_lo[h] + b_lo;
    const int ntile = nlon / (kTileCols * NSUB);
    const int total = nb * ntile, total_max = ((nb_all + rgroups - 1) / rgroups) * ntile;
    if (total > 0) {
        const float *kb = k + size_t(bh) * kD * si + size_t(hp0) * nlon;
        const float *vb = v + size_t(bh) * kD * si + size_t(hp0) * nlon;
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
            stage_tile_b(kb, vb, si, kTileCols * sub, nlon, smem + sub * kTileB, wave, nwaves, lane);
    }
    for (int it = 0; it < total_max; ++it) {
        const int b = it / ntile, xg = (it - b * ntile) * kTileCols * NSUB;
        const int hp = hp0 + b;
        float *tiles = smem + (it & 1) * NSUB * kTileB;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (it >= total) continue;   // (the other set has one more band row)
        if (it + 1 < total) {
            const int b2 = (it + 1) / ntile, x2 = (it + 1 - b2 * ntile) * kTileCols * NSUB;
            const float *kb = k + size_t(bh) * kD * si + size_t(hp0 + b2) * nlon;
            const float *vb = v + size_t(bh) * kD * si + size_t(hp0 + b2) * nlon;
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
                stage_tile_b(kb, vb, si, x2 + kTileCols * sub, nlon, smem + (((it + 1) & 1) * NSUB + sub) * kTileB, wave,
                             nwaves, lane);
        }
        const int c = table_i(t.cnt, h * t.band_max + b_lo + b);
        const bool full = c == nlon;
        const int lo = full ? 0 : -((c - 1) >> 1);
        const float wq = table_f(t.omega_rel, hp);
#pragma unroll 1
        for (int sub = 0; sub < NSUB; ++sub) {
        const int x0 = xg + kTileCols * sub;
        const float *tile = tiles + sub * kTileB;
        if (!full) {
            const int need0 = wrapn(wave * 32 + lo, nlon), len = c + 31;
            const int rel = wrapn(x0 - need0, nlon);
            if (!(rel < len || rel + kTileCols > nlon)) continue;
        }
        const float *tk = tile, *tv = tile + kD * kPQK;
        const int base = (x0 + 32 * hl - w - lo + 2 * nlon) % nlon;
        // the two 32 x 32 tiles of the super-tile one after the other: half the logits live at a time
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f32x16 sm = {0}, dm = {0};
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                sm = mfma(tk[(2 * s + hl) * kPQK + arow + 16 * mt], qop[s], sm);
                dm = mfma(tv[(2 * s + hl) * kPQV + arow + 16 * mt], gop[s], dm);
            }
            float ds[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) ds[i] = wq * __builtin_amdgcn_exp2f(sm[i] - lse2) * (dm[i] - Di);
            if (!full) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    int rel = base + 16 * mt + i;
                    rel = rel >= nlon ? rel - nlon : rel;
                    ds[i] = rel < c ? ds[i] : 0.f;
                }
            }
            // dQ^T += K dS^T: A = K[channel = col][super-tile column 32*hl + 16*mt + i]
#pragma unroll
            for (int i = 0; i < 16; ++i) acc = mfma(tk[col * kPQK + 32 * hl + 16 * mt + i], ds[i], acc);
        }
        }
    }
    if (rgroups > 1) {
        // the second set hands its partial sums to the first through LDS
        __syncthreads();
        float *slot = smem_all + wave * 64 + lane;
        const int pitch = nwaves * 64;
        if (grp == 1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) slot[i * pitch] = acc[i];
        }
        __syncthreads();
        if (grp != 0) return;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] += slot[i * pitch];
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int ch = 8 * (i >> 2) + 4 * hl + (i & 3);
        dq[(size_t(bh) * kD + ch) * so + io] = acc[i] * scale;
    }
}

// --------------------------------------------------------------- backward, dk and dv ----------
//
// Transposed roles for the dense INPUT latitudes: a wavefront owns 32 input points (k_j, v_j as B
// operands), output latitudes stream by as super-tiles of q and dout (plus their lse and D rows):
//   S = Q K^T, dP = dout V^T  (lane = owner, registers = output columns),
//   p = omega exp2(s - lse_i), dS = p (dP - D_i),
//   dK^T += Q-read-by-channel dS,  dV^T += dout-read-by-channel p.
// Output (h, w) holds input (h', w_in) iff (w - w_in) mod nlon lies in the arc of (h, h'): same mask.

constexpr int kTileC = 2 * kD * kPC + 2 * kTileCols;     // q rows, dout rows (pitch kPC), lse row, D row (64 each)

__device__ __forceinline__ void stage_tile_c(const float *qb, const float *gb, const float *lrow, const float *drow,
                                             size_t stride, int x0, int ncol, float *tile, int wave, int nwaves, int lane)
{
    const unsigned voff = 4u * unsigned(wrapn(x0 + lane, ncol));
    for (int r = wave; r < 2 * kD + 2; r += nwaves) {
        const char *rb;
        if (r < kD) rb = reinterpret_cast<const char *>(qb + size_t(r) * stride);
        else if (r < 2 * kD) rb = reinterpret_cast<const char *>(gb + size_t(r - kD) * stride);
        else rb = reinterpret_cast<const char *>(r == 2 * kD ? lrow : drow);
        float *dst = r < 2 * kD ? tile + r * kPC : tile + 2 * kD * kPC + (r - 2 * kD) * kTileCols;
        __builtin_amdgcn_global_load_lds((gptr_t)(rb + voff), (lptr_t)dst, 4, 0, 0);
    }
}

template <int NSUB>
__global__ void __launch_bounds__(1024)
nattn_bwd_dkdv_mfma(S2DeviceTables t, int nbh, int nrows, int rgroups, float scale, const float *__restrict__ q,
                    const float *__restrict__ k, const float *__restrict__ v, const float *__restrict__ lse,
                    const float *__restrict__ go, const float *__restrict__ Dws, float *__restrict__ dk,
                    float *__restrict__ dv)
{
    // rgroups = 2: two sets of wavefronts, each with half of the (transposed) band rows and its own tiles
    extern __shared__ __attribute__((aligned(16))) float smem_all[];
    const int nwaves = (blockDim.x >> 6) / rgroups;
    const int wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int grp = wave_all / nwaves, wave = wave_all - grp * nwaves;
    float *smem = smem_all + grp * (2 * NSUB * kTileC);
    const int col = lane & 31, hl = lane >> 5;
    const int nlon = t.nlon_in;                       // equal grids
    const int bh = blockIdx.x / nrows;
    const int hp = t.trow_order[blockIdx.x - bh * nrows];
    const int w = wave * 32 + col;                    // owner's input longitude
    const size_t so = size_t(t.nlat_out) * t.nlon_out, si = size_t(t.nlat_in) * t.nlon_in;
    const size_t ii = size_t(hp) * nlon + w;
    const float log2e = 1.4426950408889634f;
    const float qscale = scale * log2e, lref2 = t.ln_omega_ref * log2e, wq = t.omega_rel[hp];

    float kop[16], vop[16];
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const size_t off = (size_t(bh) * kD + 2 * s + hl) * si + ii;
        kop[s] = k[off] * qscale;
        vop[s] = v[off];
    }
    f32x16 adk = {0}, adv = {0};
    const int arow = 32 * ((col >> 2) & 1) + 4 * (col >> 3) + (col & 3);

    const int nb_all = t.tband_n[hp];
    const int b_lo = grp * nb_all / rgroups, nb = (grp + 1) * nb_all / rgroups - b_lo;
    const int h0 = t.tband_lo[hp] + b_lo;
    const int ntile = nlon / (kTileCols * NSUB);
    const int total = nb * ntile, total_max = ((nb_all + rgroups - 1) / rgroups) * ntile;
    auto issue = [&](int itx, float *dst) {
        const int b2 = itx / ntile, x2 = (itx - b2 * ntile) * kTileCols * NSUB;
        const size_t rowoff = size_t(h0 + b2) * nlon;
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
            stage_tile_c(q + size_t(bh) * kD * so + rowoff, go + size_t(bh) * kD * so + rowoff,
                         lse + size_t(bh) * so + rowoff, Dws + size_t(bh) * so + rowoff, so, x2 + kTileCols * sub, nlon,
                         dst + sub * kTileC, wave, nwaves, lane);
    };
    if (total > 0) issue(0, smem);
    for (int it = 0; it < total_max; ++it) {
        const int b = it / ntile, xg = (it - b * ntile) * kTileCols * NSUB;
        float *tiles = smem + (it & 1) * NSUB * kTileC;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (it >= total) continue;   // (the other set has one more band row)
        if (it + 1 < total) issue(it + 1, smem + ((it + 1) & 1) * NSUB * kTileC);
        const int c = table_i(t.tcnt, hp * t.tband_max + b_lo + b);
        const bool full = c == nlon;
        const int lo = full ? 0 : -((c - 1) >> 1);
#pragma unroll 1
        for (int sub = 0; sub < NSUB; ++sub) {
        const int x0 = xg + kTileCols * sub;
        const float *tile = tiles + sub * kTileC;
        if (!full) {
            const int need0 = wrapn(wave * 32 + lo, nlon), len = c + 31;
            const int rel = wrapn(x0 - need0, nlon);
            if (!(rel < len || rel + kTileCols > nlon)) continue;
        }
        const float *tq = tile, *tg = tile + kD * kPC, *tl = tile + 2 * kD * kPC, *td = tl + kTileCols;
        const int base = (x0 + 32 * hl - w - lo + 2 * nlon) % nlon;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f32x16 s = {0}, d = {0};
#pragma unroll
            for (int st = 0; st < 16; ++st) {
                const int ro = (2 * st + hl) * kPC + arow + 16 * mt;
                s = mfma(tq[ro], kop[st], s);
                d = mfma(tg[ro], vop[st], d);
            }
            float p[16], ds[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int j = 32 * hl + 16 * mt + i;          // super-tile column of this register
                const float pi = wq * __builtin_amdgcn_exp2f(s[i] - fmaf(tl[j], log2e, -lref2));
                p[i] = pi;
                ds[i] = pi * (d[i] - td[j]);
            }
            if (!full) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    int rel = base + 16 * mt + i;
                    rel = rel >= nlon ? rel - nlon : rel;
                    if (rel >= c) { p[i] = 0.f; ds[i] = 0.f; }
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int ao = col * kPC + 32 * hl + 16 * mt + i;
                adk = mfma(tq[ao], ds[i], adk);
                adv = mfma(tg[ao], p[i], adv);
            }
        }
        }
    }
    if (rgroups > 1) {
        // the second set hands its partial sums to the first through LDS
        __syncthreads();
        float *slot = smem_all + wave * 64 + lane;
        const int pitch = nwaves * 64;
        if (grp == 1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) { slot[i * pitch] = adk[i]; slot[(16 + i) * pitch] = adv[i]; }
        }
        __syncthreads();
        if (grp != 0) return;
#pragma unroll
        for (int i = 0; i < 16; ++i) { adk[i] += slot[i * pitch]; adv[i] += slot[(16 + i) * pitch]; }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int ch = 8 * (i >> 2) + 4 * hl + (i & 3);
        const size_t off = (size_t(bh) * kD + ch) * si + ii;
        dk[off] = adk[i] * scale;
        dv[off] = adv[i];
    }
}

}  // namespace

int s2_nattn_mfma_configure()
{
    auto raise = [](auto kern, size_t floats) {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   int(floats * sizeof(float))) == hipSuccess;
    };
    // <2>: two super-tiles per barrier, double buffered, for up to two sets of wavefronts; <1>: one per barrier
    return raise(nattn_fwd_mfma<2>, 8 * size_t(kTileFloats)) && raise(nattn_fwd_mfma<1>, 4 * size_t(kTileFloats)) &&
           raise(nattn_bwd_dq_mfma<2>, 8 * size_t(kTileB)) && raise(nattn_bwd_dq_mfma<1>, 4 * size_t(kTileB)) &&
           raise(nattn_bwd_dkdv_mfma<2>, 8 * size_t(kTileC)) && raise(nattn_bwd_dkdv_mfma<1>, 4 * size_t(kTileC)) ? 0 : -1;
}

// latitudes whose disk holds more than 260 points per output (the three heaviest classes) take the matrix-core path
int s2_nattn_fwd_mfma_rows(const S2DeviceTables &t, int d, int e)
{
    const int nw = t.nlon_out / 32;
    if (d != 32 || e != 32 || t.pscale != 1 || t.nlon_in % kTileCols != 0 || t.nlon_out % 32 != 0 || nw < 2 || nw > 16)
        return 0;
    if (s2_debug_flag(S2_DEBUG_NO_MFMA)) return 0;   // test-only: force the vector kernels
    return t.fwd_cls[0] + t.fwd_cls[1] + t.fwd_cls[2];
}

// Two sets of wavefronts per workgroup (each with half of the band rows) when the launch has no more workgroups
// than the device has compute units: with one workgroup of nlon/32 wavefronts per compute unit a SIMD would hold a
// single wavefront and every matrix-instruction chain would run exposed.
static int row_groups(const S2DeviceTables &t, int nbh, int nrows)
{
    static int ncu = 0;
    if (ncu == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu <= 0)
            ncu = 256;
    }
    const bool off = s2_debug_flag(S2_DEBUG_NO_ROW_GROUPS);   // test-only
    const bool fits = t.nlon_out * 4 <= 1024 && t.nlon_in % (2 * kTileCols) == 0;
    return (!off && fits && long(nrows) * nbh <= ncu) ? 2 : 1;
}

int s2_nattn_fwd_mfma(const S2DeviceTables &t, int nbh, int nrows, float scale, const float *q, const float *k,
                      const float *v, float *out, float *lse, hipStream_t st)
{
    const bool two = t.nlon_in % (2 * kTileCols) == 0;
    const int rgroups = row_groups(t, nbh, nrows);
    const size_t lds = rgroups * (two ? 4 : 2) * size_t(kTileFloats) * sizeof(float);
    S2TraceScope tr("nattn_fwd_mfma", nbh * (t.fwd_pairs[0] + t.fwd_pairs[1] + t.fwd_pairs[2]), st);
    if (two)
        hipLaunchKernelGGL(nattn_fwd_mfma<2>, dim3((unsigned)(long(nrows) * nbh)), dim3(t.nlon_out * 2 * rgroups), lds, st, t,
                           nbh, nrows, rgroups, scale * 1.4426950408889634f, q, k, v, out, lse);
    else
        hipLaunchKernelGGL(nattn_fwd_mfma<1>, dim3((unsigned)(long(nrows) * nbh)), dim3(t.nlon_out * 2 * rgroups), lds, st, t,
                           nbh, nrows, rgroups, scale * 1.4426950408889634f, q, k, v, out, lse);
    return 0;
}

int s2_nattn_bwd_dq_mfma(const S2DeviceTables &t, int nbh, int nrows, float scale, const float *q, const float *k,
                         const float *v, const float *o, const float *lse, const float *go, float *dq, float *Dws,
                         hipStream_t st)
{
    const bool two = t.nlon_in % (2 * kTileCols) == 0;
    const int rgroups = row_groups(t, nbh, nrows);
    const size_t lds = rgroups * (two ? 4 : 2) * size_t(kTileB) * sizeof(float);
    S2TraceScope tr("nattn_bwd_dq_mfma", nbh * (t.fwd_pairs[0] + t.fwd_pairs[1] + t.fwd_pairs[2]), st);
    if (two)
        hipLaunchKernelGGL(nattn_bwd_dq_mfma<2>, dim3((unsigned)(long(nrows) * nbh)), dim3(t.nlon_out * 2 * rgroups), lds, st,
                           t, nbh, nrows, rgroups, scale, q, k, v, o, lse, go, dq, Dws);
    else
        hipLaunchKernelGGL(nattn_bwd_dq_mfma<1>, dim3((unsigned)(long(nrows) * nbh)), dim3(t.nlon_out * 2 * rgroups), lds, st,
                           t, nbh, nrows, rgroups, scale, q, k, v, o, lse, go, dq, Dws);
    return 0;
}

int s2_nattn_bwd_dkdv_mfma_rows(const S2DeviceTables &t, int d, int e)
{
    const int nw = t.nlon_in / 32;
    if (d != 32 || e != 32 || t.pscale != 1 || t.nlon_in % kTileCols != 0 || nw < 2 || nw > 16) return 0;
    if (s2_debug_flag(S2_DEBUG_NO_MFMA)) return 0;
    return t.bwd_cls[0] + t.bwd_cls[1] + t.bwd_cls[2];
}

int s2_nattn_bwd_dkdv_mfma(const S2DeviceTables &t, int nbh, int nrows, float scale, const float *q, const float *k,
                           const float *v, const float *lse, const float *go, const float *Dws, float *dk, float *dv,
                           hipStream_t st)
{
    const bool two = t.nlon_in % (2 * kTileCols) == 0;
    const int rgroups = row_groups(t, nbh, nrows);
    const size_t lds = rgroups * (two ? 4 : 2) * size_t(kTileC) * sizeof(float);
    S2TraceScope tr("nattn_bwd_dkdv_mfma", nbh * (t.bwd_pairs[0] + t.bwd_pairs[1] + t.bwd_pairs[2]), st);
    if (two)
        hipLaunchKernelGGL(nattn_bwd_dkdv_mfma<2>, dim3((unsigned)(long(nrows) * nbh)), dim3(t.nlon_in * 2 * rgroups), lds, st,
                           t, nbh, nrows, rgroups, scale, q, k, v, lse, go, Dws, dk, dv);
    else
        hipLaunchKernelGGL(nattn_bwd_dkdv_mfma<1>, dim3((unsigned)(long(nrows) * nbh)), dim3(t.nlon_in * 2 * rgroups), lds, st,
                           t, nbh, nrows, rgroups, scale, q, k, v, lse, go, Dws, dk, dv);
    return 0;
}
