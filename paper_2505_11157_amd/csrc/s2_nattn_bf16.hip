// Neighborhood attention on bf16 tensors with the bf16 matrix cores of gfx950 (App. B.1 second equation in the
// index form of App. B.3; gradients of App. B.4), float32 softmax, accumulation, logsumexp and D.
//
// Band tiles.  The disk of an output point meets input latitude h' in an arc of longitude offsets [-hw, hw] (or the
// whole circle), so for 16 consecutive outputs of one latitude the keys of h' lie in a window of 16 + 2 hw columns:
// a band of the (keys x outputs) score matrix.  The window is cut into tiles of 16 keys; a tile of
// 16 keys x 16 outputs is one v_mfma_f32_16x16x32_bf16 (all 32 channels in one instruction); tiles that the band
// does not touch are skipped, tiles it cuts get a per-element mask, tiles inside it none.  The tile grid of a row is
// shifted by 8 columns when that saves a tile (1 <= hw mod 16 <= 8).  The same kernels take the dense polar
// latitudes (whole circles, no masks) and the light ones.
//
// Orientation.  Scores are produced transposed (S^T = K Q^T: lane = (output n, key group g), four keys per lane),
// so the softmax is a per-lane loop and the probabilities of two key tiles, packed to bf16, are the B operand of the
// next matrix instruction (O^T += V P^T) without moving data between lanes.  The four lanes of an output share the
// running reference maximum, which moves only when a logit exceeds it by more than 2^8.
//
// Staging.  A workgroup of four wavefronts owns 128 consecutive points of one latitude (32 per wavefront, two
// 16-point tiles; the kernels carry the tile count as a template parameter) and streams the other side in stages of 64 columns through LDS, double buffered, one barrier per
// stage.  Operands contracted over channels (K for the scores, V for dP, q and dout in the dk/dv kernel) are needed
// token-major (a key's 32 channels contiguous), but the tensors are channel-major: the 16-byte pieces a thread
// loads (8 columns of one channel) are scattered into a token-major tile with eight 2-byte LDS writes; the operands
// contracted over tokens are copied as they are.  Row pitches of 80 and 144 bytes keep the operand reads of the 16
// lanes that are served together on 64 different banks.
#include "s2_nattn_kernels.h"

namespace {

typedef unsigned short bf16raw;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kD = 32;                     // channels (d = e)
constexpr int kPitchT = 80;                // bytes per row of a token-major tile: 64 bytes of channels + 16
constexpr int kPitchC = 144;               // bytes per row of a channel-major tile: 128 bytes of columns + 16
constexpr int kTokBytes = 64 * kPitchT;    // 64 tokens
constexpr int kChanBytes = kD * kPitchC;   // 32 channel rows of 64 columns
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ __bf16 raw_to_bf16(bf16raw x) { return __builtin_bit_cast(__bf16, x); }
__device__ __forceinline__ bf16raw bf16_bits(float x)
{
    const __bf16 b = (__bf16)x;
    return __builtin_bit_cast(bf16raw, b);
}

// ---- staging: thread tid of 256 handles channel tid >> 3 and the eight columns X0 + 8 (tid & 7) .. + 7 ------------
// X0 is an unwrapped column (>= 0, a multiple of 8); longitude counts are multiples of 8, so a piece never straddles
// the seam and is 16-byte aligned.
__device__ __forceinline__ uint4 load_piece(const bf16raw *slice, size_t plane, int lat, int nlon, int X0, int tid)
{
    int col = X0 + 8 * (tid & 7);              // below 3 nlon
    col = col >= nlon ? col - nlon : col;
    col = col >= nlon ? col - nlon : col;
    return *reinterpret_cast<const uint4 *>(slice + size_t(tid >> 3) * plane + size_t(lat) * nlon + col);
}

__device__ __forceinline__ void store_chan(char *tile, uint4 v, int tid)
{
    *reinterpret_cast<uint4 *>(tile + (tid >> 3) * kPitchC + 16 * (tid & 7)) = v;
}

// token-major: row = column within the stage, 16-byte piece (channel group) swizzled by the row's 16-block
__device__ __forceinline__ void store_tok(char *tile, uint4 v, int tid)
{
    const int c = tid >> 3, p = tid & 7;
    char *dst = tile + 8 * p * kPitchT + (((c >> 3) ^ (p >> 1)) << 4) + 2 * (c & 7);
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int u = 0; u < 8; ++u)
        *reinterpret_cast<bf16raw *>(dst + u * kPitchT) = bf16raw(w[u >> 1] >> (16 * (u & 1)));
}

// ---- operand reads (lane = (m = lane & 15, g = lane >> 4)) ---------------------------------------------------------
// A operand for a contraction over channels: token 16 kt + m of the stage, channels 8 g .. 8 g + 7
__device__ __forceinline__ bf16x8 tok_operand(const char *tile, int kt, int lane)
{
    const int m = lane & 15, g = lane >> 4;
    return *reinterpret_cast<const bf16x8 *>(tile + (16 * kt + m) * kPitchT + ((g ^ kt) << 4));
}
// A operand for a contraction over tokens: channel 16 mt + m; contraction index 8 g + r is token 4 g + r of tile ta,
// 8 g + 4 + r token 4 g + r of tile tb (the order in which the packed probabilities of the two tiles hold them)
__device__ __forceinline__ bf16x8 chan_operand(const char *tile, int mt, int ta, int tb, int lane)
{
    const int m = lane & 15, g = lane >> 4;
    const char *row = tile + (16 * mt + m) * kPitchC + 8 * g;
    const uint2 a = *reinterpret_cast<const uint2 *>(row + 32 * ta);
    const uint2 b = *reinterpret_cast<const uint2 *>(row + 32 * tb);
    const uint4 r = {a.x, a.y, b.x, b.y};
    return __builtin_bit_cast(bf16x8, r);
}
// B operand of an owner point (lat, w): channels 8 g .. 8 g + 7, gathered from the channel-major tensor
__device__ __forceinline__ bf16x8 gather_point(const bf16raw *slice, size_t plane, size_t at, int g)
{
    bf16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = raw_to_bf16(slice[size_t(8 * g + j) * plane + at]);
    return r;
}
__device__ __forceinline__ bf16x8 pack2(f32x4 a, f32x4 b)
{
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        r[i] = (__bf16)a[i];
        r[4 + i] = (__bf16)b[i];
    }
    return r;
}
// The same in two bf16 terms, hi + lo = x to about 2^-17 relative: dS (and P in the dk/dv kernel) multiply single
// large terms of the gradient sums, where one bf16 rounding (2^-9) of the factor would show in the result.
__device__ __forceinline__ void pack2_split(f32x4 a, f32x4 b, bf16x8 &hi, bf16x8 &lo)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        hi[i] = (__bf16)a[i];
        lo[i] = (__bf16)(a[i] - float(hi[i]));
        hi[4 + i] = (__bf16)b[i];
        lo[4 + i] = (__bf16)(b[i] - float(hi[4 + i]));
    }
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

// One row of the other side as seen from a workgroup whose owners are the columns [W0, W0 + 256) of their latitude:
// arc half-width (or whole circle), first unwrapped column of the first stage and the number of 64-column stages.
// Unwrapped columns are offset by nlon so that they stay non-negative; column X is longitude X mod nlon.
struct RowWindow {
    int hw, full, X0, nst;
    __device__ __forceinline__ void set(int cnt, int nlon, int W0, int nown)
    {
        full = cnt == nlon;
        hw = full ? 0 : (cnt - 1) >> 1;
        if (full) {
            X0 = nlon + W0;
            nst = nlon >> 6;
        } else {
            const int off = (hw & 15) >= 1 && (hw & 15) <= 8 ? 8 : 0;      // tile grid shifted by 8 saves a tile
            const int lo = nlon + W0 - hw;
            X0 = ((lo - off) & ~15) + off;
            nst = (nlon + W0 + nown + hw - X0 + 63) >> 6;
        }
    }
};

// does the 16-column tile at unwrapped column Xt touch the band of the 16 owners at Wo, and does it lie inside it?
__device__ __forceinline__ bool touches(const RowWindow &r, int Xt, int Wo)
{
    return r.full || (Xt + 15 >= Wo - r.hw && Xt <= Wo + 15 + r.hw);
}
__device__ __forceinline__ bool inside(const RowWindow &r, int Xt, int Wo)
{
    const int dlt = Xt > Wo ? Xt - Wo : Wo - Xt;
    return r.full || r.hw >= 15 + dlt;
}

// ---------------------------------------------------------------------------------------------------------------
// Forward.  Block -> (output latitude by work, slice, group of 64 NOW longitudes); NOW = owner tiles per wavefront.
template <int NOW>
__global__ void __launch_bounds__(256, 3)
nattn_fwd_bf16(S2DeviceTables t, int nbh, int first_row, float c2, const bf16raw *__restrict__ q, const bf16raw *__restrict__ k,
               const bf16raw *__restrict__ v, bf16raw *__restrict__ out, float *__restrict__ lse)
{
    __shared__ __attribute__((aligned(16))) char lds[2][kTokBytes + kChanBytes];
    const int nlon = t.nlon_in;
    constexpr int GW = 64 * NOW, WW = 16 * NOW;          // owners per workgroup and per wavefront
    const int ngrp = (nlon + GW - 1) / GW;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int bh = id % nbh;
    const int h = t.row_order[first_row + id / nbh];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int W0 = grp * GW;
    const int nown = nlon - W0 < GW ? nlon - W0 : GW;
    const bool active = W0 + WW * wave < nlon;          // longitude counts are multiples of 64: all or nothing
    const size_t plane = size_t(t.nlat_in) * nlon;      // equal grids
    const bf16raw *qs = q + size_t(bh) * kD * plane, *ks = k + size_t(bh) * kD * plane, *vs = v + size_t(bh) * kD * plane;
    const int Wb = nlon + W0 + WW * wave;               // unwrapped column of the wavefront's first owner

    bf16x8 qreg[NOW];
    f32x4 acc[NOW][2];
    float m[NOW], l[NOW];
#pragma unroll
    for (int o = 0; o < NOW; ++o) {
        if (active) qreg[o] = gather_point(qs, plane, size_t(h) * nlon + (W0 + WW * wave + 16 * o + n), g);
        acc[o][0] = acc[o][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        m[o] = -INFINITY;
        l[o] = 0.f;
    }

    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    RowWindow cur, nxt;
    int b = 0, s = 0, nb_next = 0, s_next = 0;
    cur.set(t.cnt[h * t.band_max], nlon, W0, nown);
    uint4 rk = load_piece(ks, plane, hp0, nlon, cur.X0, tid), rv = load_piece(vs, plane, hp0, nlon, cur.X0, tid);
    store_tok(lds[0], rk, tid);
    store_chan(lds[0] + kTokBytes, rv, tid);
    __syncthreads();
    int buf = 0;
    while (true) {
        // the stage after this one
        nb_next = b;
        s_next = s + 1;
        nxt = cur;
        if (s_next == cur.nst) {
            nb_next = b + 1;
            s_next = 0;
            if (nb_next < nb) nxt.set(t.cnt[h * t.band_max + nb_next], nlon, W0, nown);
        }
        const bool more = nb_next < nb;
        if (more) {
            rk = load_piece(ks, plane, hp0 + nb_next, nlon, nxt.X0 + 64 * s_next, tid);
            rv = load_piece(vs, plane, hp0 + nb_next, nlon, nxt.X0 + 64 * s_next, tid);
        }
        if (active) {
            const char *Kt = lds[buf], *Vc = lds[buf] + kTokBytes;
            const float lw2 = __log2f(t.omega_rel[hp0 + b]);
            const int Xs = cur.X0 + 64 * s;
            bf16x8 ka[4];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) ka[kt] = tok_operand(Kt, kt, lane);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 v0 = chan_operand(Vc, 0, 2 * j, 2 * j + 1, lane), v1 = chan_operand(Vc, 1, 2 * j, 2 * j + 1, lane);
#pragma unroll
                for (int o = 0; o < NOW; ++o) {
                    const int Wo = Wb + 16 * o;
                    f32x4 x[2];
                    bool tch[2];
                    float mx = -INFINITY;
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int Xt = Xs + 16 * (2 * j + u);
                        tch[u] = touches(cur, Xt, Wo);
                        if (!tch[u]) continue;
                        const f32x4 sc = mfma16(ka[2 * j + u], qreg[o], f32x4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
                        for (int r = 0; r < 4; ++r) x[u][r] = fmaf(sc[r], c2, lw2);
                        if (!inside(cur, Xt, Wo)) {
                            const unsigned uu = unsigned(Xt + 4 * g - (Wo + n) + cur.hw), lim = unsigned(2 * cur.hw);
#pragma unroll
                            for (int r = 0; r < 4; ++r) x[u][r] = uu + r <= lim ? x[u][r] : -INFINITY;
                        }
                        mx = fmaxf(mx, fmaxf(fmaxf(x[u][0], x[u][1]), fmaxf(x[u][2], x[u][3])));
                    }
                    if (!tch[0] && !tch[1]) continue;
                    if (__any(mx > m[o] + 8.f)) {
                        mx = group_max(mx);
                        const float m_new = mx > m[o] + 8.f ? mx : m[o];
                        // unchanged reference: factor 1 (also when it is still -inf); first member: 0, nothing summed yet
                        const float corr = m_new == m[o] ? 1.f : __builtin_amdgcn_exp2f(m[o] - m_new);
                        m[o] = m_new;
                        l[o] *= corr;
#pragma unroll
                        for (int r = 0; r < 4; ++r) { acc[o][0][r] *= corr; acc[o][1][r] *= corr; }
                    }
                    const float ms = m[o] == -INFINITY ? 0.f : m[o];        // no member yet: every x is -inf
                    float ps = 0.f;
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        if (tch[u]) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                x[u][r] = __builtin_amdgcn_exp2f(x[u][r] - ms);
                                ps += x[u][r];
                            }
                        } else {
                            x[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                        }
                    }
                    l[o] += ps;
                    const bf16x8 pb = pack2(x[0], x[1]);
                    acc[o][0] = mfma16(v0, pb, acc[o][0]);
                    acc[o][1] = mfma16(v1, pb, acc[o][1]);
                }
            }
        }
        if (!more) break;
        store_tok(lds[buf ^ 1], rk, tid);
        store_chan(lds[buf ^ 1] + kTokBytes, rv, tid);
        __syncthreads();
        buf ^= 1;
        b = nb_next;
        s = s_next;
        cur = nxt;
    }
    if (!active) return;
    const size_t so = plane;
#pragma unroll
    for (int o = 0; o < NOW; ++o) {
        const float lt = group_sum(l[o]);
        const float inv = 1.f / lt;
        const size_t at = size_t(h) * nlon + (W0 + WW * wave + 16 * o + n);
        bf16raw *ob = out + size_t(bh) * kD * so + at;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) ob[size_t(16 * mt + 4 * g + r) * so] = bf16_bits(acc[o][mt][r] * inv);
        if (g == 0) lse[size_t(bh) * so + at] = (m[o] + __log2f(lt)) * 0.6931471805599453f + t.ln_omega_ref;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Backward, query side: D_i = dout_i . out_i (stored for the key side), dS_ij = p_ij (dout_i . v_j - D_i),
// dq_i = scale sum_j dS_ij k_j, with p_ij = omega_j exp(scale q_i.k_j - lse_i) recomputed from the saved logsumexp.
template <int NOW>
__global__ void __launch_bounds__(256, 3)
nattn_bwd_dq_bf16(S2DeviceTables t, int nbh, int first_row, float scale, const bf16raw *__restrict__ q, const bf16raw *__restrict__ k,
                  const bf16raw *__restrict__ v, const bf16raw *__restrict__ o_, const float *__restrict__ lse,
                  const bf16raw *__restrict__ go, bf16raw *__restrict__ dq, float *__restrict__ Dws)
{
    constexpr int kStage = 2 * kTokBytes + kChanBytes;       // K and V token-major, K channel-major
    __shared__ __attribute__((aligned(16))) char lds[2][kStage];
    const int nlon = t.nlon_in;
    constexpr int GW = 64 * NOW, WW = 16 * NOW;          // owners per workgroup and per wavefront
    const int ngrp = (nlon + GW - 1) / GW;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int bh = id % nbh;
    const int h = t.row_order[first_row + id / nbh];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int W0 = grp * GW;
    const int nown = nlon - W0 < GW ? nlon - W0 : GW;
    const bool active = W0 + WW * wave < nlon;
    const size_t plane = size_t(t.nlat_in) * nlon;
    const bf16raw *qs = q + size_t(bh) * kD * plane, *ks = k + size_t(bh) * kD * plane, *vs = v + size_t(bh) * kD * plane;
    const bf16raw *os = o_ + size_t(bh) * kD * plane, *gs = go + size_t(bh) * kD * plane;
    const int Wb = nlon + W0 + WW * wave;
    const float c2 = scale * kLog2e;

    bf16x8 qreg[NOW], greg[NOW];
    f32x4 acc[NOW][2];
    float L2[NOW], Dn[NOW];
#pragma unroll
    for (int o = 0; o < NOW; ++o) {
        acc[o][0] = acc[o][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        L2[o] = 0.f;
        Dn[o] = 0.f;
        if (active) {
            const size_t at = size_t(h) * nlon + (W0 + WW * wave + 16 * o + n);
            qreg[o] = gather_point(qs, plane, at, g);
            greg[o] = gather_point(gs, plane, at, g);
            const bf16x8 oo = gather_point(os, plane, at, g);
            float dsum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) dsum = fmaf(float(greg[o][j]), float(oo[j]), dsum);
            dsum = group_sum(dsum);
            if (g == 0) Dws[size_t(bh) * plane + at] = dsum;
            Dn[o] = -dsum;
            L2[o] = (lse[size_t(bh) * plane + at] - t.ln_omega_ref) * kLog2e;
        }
    }

    const int nb = t.band_n[h], hp0 = t.band_lo[h];
    RowWindow cur, nxt;
    int b = 0, s = 0, nb_next = 0, s_next = 0;
    cur.set(t.cnt[h * t.band_max], nlon, W0, nown);
    uint4 rk = load_piece(ks, plane, hp0, nlon, cur.X0, tid), rv = load_piece(vs, plane, hp0, nlon, cur.X0, tid);
    store_tok(lds[0], rk, tid);
    store_tok(lds[0] + kTokBytes, rv, tid);
    store_chan(lds[0] + 2 * kTokBytes, rk, tid);
    __syncthreads();
    int buf = 0;
    while (true) {
        nb_next = b;
        s_next = s + 1;
        nxt = cur;
        if (s_next == cur.nst) {
            nb_next = b + 1;
            s_next = 0;
            if (nb_next < nb) nxt.set(t.cnt[h * t.band_max + nb_next], nlon, W0, nown);
        }
        const bool more = nb_next < nb;
        if (more) {
            rk = load_piece(ks, plane, hp0 + nb_next, nlon, nxt.X0 + 64 * s_next, tid);
            rv = load_piece(vs, plane, hp0 + nb_next, nlon, nxt.X0 + 64 * s_next, tid);
        }
        if (active) {
            const char *Kt = lds[buf], *Vt = lds[buf] + kTokBytes, *Kc = lds[buf] + 2 * kTokBytes;
            const float lw2 = __log2f(t.omega_rel[hp0 + b]);
            const int Xs = cur.X0 + 64 * s;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 k0 = chan_operand(Kc, 0, 2 * j, 2 * j + 1, lane), k1 = chan_operand(Kc, 1, 2 * j, 2 * j + 1, lane);
#pragma unroll
                for (int o = 0; o < NOW; ++o) {
                    const int Wo = Wb + 16 * o;
                    f32x4 ds[2];
                    bool any_tile = false;
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int Xt = Xs + 16 * (2 * j + u);
                        ds[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                        if (!touches(cur, Xt, Wo)) continue;
                        any_tile = true;
                        const f32x4 sc = mfma16(tok_operand(Kt, 2 * j + u, lane), qreg[o], f32x4{0.f, 0.f, 0.f, 0.f});
                        const f32x4 dp = mfma16(tok_operand(Vt, 2 * j + u, lane), greg[o], f32x4{Dn[o], Dn[o], Dn[o], Dn[o]});   // dout.v - D
                        const float bias = lw2 - L2[o];
                        if (inside(cur, Xt, Wo)) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) ds[u][r] = __builtin_amdgcn_exp2f(fmaf(sc[r], c2, bias)) * dp[r];
                        } else {
                            const unsigned uu = unsigned(Xt + 4 * g - (Wo + n) + cur.hw), lim = unsigned(2 * cur.hw);
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                ds[u][r] = uu + r <= lim ? __builtin_amdgcn_exp2f(fmaf(sc[r], c2, bias)) * dp[r] : 0.f;
                        }
                    }
                    if (!any_tile) continue;
                    bf16x8 dh, dl;
                    pack2_split(ds[0], ds[1], dh, dl);
                    acc[o][0] = mfma16(k0, dl, mfma16(k0, dh, acc[o][0]));
                    acc[o][1] = mfma16(k1, dl, mfma16(k1, dh, acc[o][1]));
                }
            }
        }
        if (!more) break;
        store_tok(lds[buf ^ 1], rk, tid);
        store_tok(lds[buf ^ 1] + kTokBytes, rv, tid);
        store_chan(lds[buf ^ 1] + 2 * kTokBytes, rk, tid);
        __syncthreads();
        buf ^= 1;
        b = nb_next;
        s = s_next;
        cur = nxt;
    }
    if (!active) return;
#pragma unroll
    for (int o = 0; o < NOW; ++o) {
        bf16raw *ob = dq + size_t(bh) * kD * plane + size_t(h) * nlon + (W0 + WW * wave + 16 * o + n);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) ob[size_t(16 * mt + 4 * g + r) * plane] = bf16_bits(acc[o][mt][r] * scale);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Backward, key side: the owners are input points j (lane = (key n, output group g)); the outputs whose disk holds j
// are, on every output latitude of the transposed band, the columns within the same half-width of j.
// dk_j = scale sum_i dS_ij q_i, dv_j = sum_i p_ij dout_i: gathered, no atomics.
template <int NOW>
__global__ void __launch_bounds__(256)
nattn_bwd_dkdv_bf16(S2DeviceTables t, int nbh, int first_row, float scale, const bf16raw *__restrict__ q, const bf16raw *__restrict__ k,
                    const bf16raw *__restrict__ v, const float *__restrict__ lse, const bf16raw *__restrict__ go,
                    const float *__restrict__ Dws, bf16raw *__restrict__ dk, bf16raw *__restrict__ dv)
{
    constexpr int kStage = 2 * kTokBytes + 2 * kChanBytes + 512;     // q, dout token-major; q, dout channel-major; L2, -D
    __shared__ __attribute__((aligned(16))) char lds[2][kStage];
    const int nlon = t.nlon_in;
    constexpr int GW = 64 * NOW, WW = 16 * NOW;          // owners per workgroup and per wavefront
    const int ngrp = (nlon + GW - 1) / GW;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int bh = id % nbh;
    const int hp = t.trow_order[first_row + id / nbh];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int W0 = grp * GW;
    const int nown = nlon - W0 < GW ? nlon - W0 : GW;
    const bool active = W0 + WW * wave < nlon;
    const size_t plane = size_t(t.nlat_in) * nlon;
    const bf16raw *qs = q + size_t(bh) * kD * plane, *ks = k + size_t(bh) * kD * plane, *vs = v + size_t(bh) * kD * plane;
    const bf16raw *gs = go + size_t(bh) * kD * plane;
    const float *ls = lse + size_t(bh) * plane, *Ds = Dws + size_t(bh) * plane;
    const int Wb = nlon + W0 + WW * wave;
    const float c2 = scale * kLog2e;
    const float lw2 = __log2f(t.omega_rel[hp]);     // -inf for a latitude of weight zero: p = 0
    const float lref = t.ln_omega_ref;

    bf16x8 kreg[NOW], vreg[NOW];
    f32x4 adk[NOW][2], adv[NOW][2];
#pragma unroll
    for (int o = 0; o < NOW; ++o) {
        adk[o][0] = adk[o][1] = adv[o][0] = adv[o][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (active) {
            const size_t at = size_t(hp) * nlon + (W0 + WW * wave + 16 * o + n);
            kreg[o] = gather_point(ks, plane, at, g);
            vreg[o] = gather_point(vs, plane, at, g);
        }
    }

    const int nb = t.tband_n[hp], h0 = t.tband_lo[hp];
    RowWindow cur, nxt;
    int b = 0, s = 0, nb_next = 0, s_next = 0;
    cur.set(t.tcnt[hp * t.tband_max], nlon, W0, nown);
    // the float rows (64 values each): threads 0..63 the logsumexp, 64..127 D
    auto load_stat = [&](int lat, int X0) -> float {
        if (tid >= 128) return 0.f;
        const int col = (X0 + (tid & 63)) % nlon;
        return tid < 64 ? (ls[size_t(lat) * nlon + col] - lref) * kLog2e : -Ds[size_t(lat) * nlon + col];
    };
    auto store_stage = [&](char *base, uint4 a, uint4 c, float st) {
        store_tok(base, a, tid);
        store_tok(base + kTokBytes, c, tid);
        store_chan(base + 2 * kTokBytes, a, tid);
        store_chan(base + 2 * kTokBytes + kChanBytes, c, tid);
        if (tid < 128) reinterpret_cast<float *>(base + 2 * kTokBytes + 2 * kChanBytes)[tid] = st;
    };
    uint4 rq = load_piece(qs, plane, h0, nlon, cur.X0, tid), rg = load_piece(gs, plane, h0, nlon, cur.X0, tid);
    float rs = load_stat(h0, cur.X0);
    store_stage(lds[0], rq, rg, rs);
    __syncthreads();
    int buf = 0;
    while (true) {
        nb_next = b;
        s_next = s + 1;
        nxt = cur;
        if (s_next == cur.nst) {
            nb_next = b + 1;
            s_next = 0;
            if (nb_next < nb) nxt.set(t.tcnt[hp * t.tband_max + nb_next], nlon, W0, nown);
        }
        const bool more = nb_next < nb;
        if (more) {
            rq = load_piece(qs, plane, h0 + nb_next, nlon, nxt.X0 + 64 * s_next, tid);
            rg = load_piece(gs, plane, h0 + nb_next, nlon, nxt.X0 + 64 * s_next, tid);
            rs = load_stat(h0 + nb_next, nxt.X0 + 64 * s_next);
        }
        if (active) {
            const char *Qt = lds[buf], *Gt = lds[buf] + kTokBytes, *Qc = lds[buf] + 2 * kTokBytes;
            const char *Gc = Qc + kChanBytes;
            const float *Ls = reinterpret_cast<const float *>(Gc + kChanBytes), *Dn = Ls + 64;
            const int Xs = cur.X0 + 64 * s;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 q0 = chan_operand(Qc, 0, 2 * j, 2 * j + 1, lane), q1 = chan_operand(Qc, 1, 2 * j, 2 * j + 1, lane);
                const bf16x8 g0 = chan_operand(Gc, 0, 2 * j, 2 * j + 1, lane), g1 = chan_operand(Gc, 1, 2 * j, 2 * j + 1, lane);
                bf16x8 qa[2], ga[2];
                f32x4 L[2], Dm[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    qa[u] = tok_operand(Qt, 2 * j + u, lane);
                    ga[u] = tok_operand(Gt, 2 * j + u, lane);
                    L[u] = *reinterpret_cast<const f32x4 *>(Ls + 16 * (2 * j + u) + 4 * g);      // outputs 4 g .. 4 g + 3 of the tile
                    Dm[u] = *reinterpret_cast<const f32x4 *>(Dn + 16 * (2 * j + u) + 4 * g);
                }
#pragma unroll
                for (int o = 0; o < NOW; ++o) {
                    const int Wo = Wb + 16 * o;
                    f32x4 p[2], ds[2];
                    bool any_tile = false;
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int Xt = Xs + 16 * (2 * j + u);
                        p[u] = ds[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                        if (!touches(cur, Xt, Wo)) continue;
                        any_tile = true;
                        const f32x4 sc = mfma16(qa[u], kreg[o], f32x4{0.f, 0.f, 0.f, 0.f});    // rows: outputs, lane: key
                        const f32x4 dp = mfma16(ga[u], vreg[o], Dm[u]);                        // dout.v - D
                        if (inside(cur, Xt, Wo)) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                p[u][r] = __builtin_amdgcn_exp2f(fmaf(sc[r], c2, lw2 - L[u][r]));
                                ds[u][r] = p[u][r] * dp[r];
                            }
                        } else {
                            const unsigned uu = unsigned(Xt + 4 * g - (Wo + n) + cur.hw), lim = unsigned(2 * cur.hw);
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                p[u][r] = uu + r <= lim ? __builtin_amdgcn_exp2f(fmaf(sc[r], c2, lw2 - L[u][r])) : 0.f;
                                ds[u][r] = p[u][r] * dp[r];
                            }
                        }
                    }
                    if (!any_tile) continue;
                    bf16x8 ph, pl, dh, dl;
                    pack2_split(p[0], p[1], ph, pl);
                    pack2_split(ds[0], ds[1], dh, dl);
                    adv[o][0] = mfma16(g0, pl, mfma16(g0, ph, adv[o][0]));
                    adv[o][1] = mfma16(g1, pl, mfma16(g1, ph, adv[o][1]));
                    adk[o][0] = mfma16(q0, dl, mfma16(q0, dh, adk[o][0]));
                    adk[o][1] = mfma16(q1, dl, mfma16(q1, dh, adk[o][1]));
                }
            }
        }
        if (!more) break;
        store_stage(lds[buf ^ 1], rq, rg, rs);
        __syncthreads();
        buf ^= 1;
        b = nb_next;
        s = s_next;
        cur = nxt;
    }
    if (!active) return;
#pragma unroll
    for (int o = 0; o < NOW; ++o) {
        const size_t at = size_t(bh) * kD * plane + size_t(hp) * nlon + (W0 + WW * wave + 16 * o + n);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                dk[at + size_t(16 * mt + 4 * g + r) * plane] = bf16_bits(adk[o][mt][r] * scale);
                dv[at + size_t(16 * mt + 4 * g + r) * plane] = bf16_bits(adv[o][mt][r]);
            }
    }
}

}  // namespace

bool s2_nattn_bf16_supported(const S2DeviceTables &t, int d, int e)
{
    return d == kD && e == kD && t.upscale == 1 && t.pscale == 1 && t.nlon_in == t.nlon_out && t.nlat_in == t.nlat_out &&
           t.nlon_in % 64 == 0 && !s2_debug_flag(S2_DEBUG_NO_MFMA);
}

namespace {

// ===================================================================================================================
// Light latitudes (short arcs: at most 57 offsets on every band row, one contiguous range of latitudes).  With 256
// longitudes of ONE latitude per workgroup a 64-column stage gives a wavefront one or two tiles of work per barrier,
// and the windows of the nine band rows are fetched again for every latitude.  Here a workgroup owns 64 longitudes of
// FOUR consecutive latitudes (one per wavefront): an input row is staged once, as one stage of 128 columns (the
// window of 64 owners for half-widths up to 28), and serves every wavefront whose band holds it; behind each pair of
// barriers lies the arithmetic of a whole band row.  Every 16-owner tile walks its own key tiles from the staged row,
// starting at the first column of its band rounded down to a multiple of four (operand reads stay 8-byte aligned), so
// no tile is computed that the band does not touch.  The staged tiles carry 32 zeroed rows / columns of padding:
// a tile that reaches past the window reads zeros, never stale bits that a matrix instruction could turn into NaN.
constexpr int kLRows = 160;                      // 128 staged columns + 32 of zero padding
constexpr int kLPitchC = 2 * kLRows + 16;        // bytes per channel row
constexpr int kLTok = kLRows * kPitchT + 64;     // rows 64..127 sit 64 bytes further on (see store_tok128)
constexpr int kLChan = kD * kLPitchC;

// piece i of 512: channel i >> 4, the eight columns X0 + 8 (i & 15) .. + 7
__device__ __forceinline__ uint4 load_piece128(const bf16raw *slice, size_t plane, int lat, int nlon, int X0, int i)
{
    int col = X0 + 8 * (i & 15);               // below 3 nlon
    col = col >= nlon ? col - nlon : col;
    col = col >= nlon ? col - nlon : col;
    return *reinterpret_cast<const uint4 *>(slice + size_t(i >> 4) * plane + size_t(lat) * nlon + col);
}
__device__ __forceinline__ void store_chan128(char *tile, uint4 v, int i)
{
    *reinterpret_cast<uint4 *>(tile + (i >> 4) * kLPitchC + 16 * (i & 15)) = v;
}
__device__ __forceinline__ void store_tok128(char *tile, uint4 v, int i)
{
    const int c = i >> 4, p = i & 15;
    // rows r and r + 64 would share their banks (64 * 80 bytes = 20 * 64 words): the second 64 rows are shifted by 16
    // words, into the banks the 16 pieces of a wavefront's scatter leave free
    char *dst = tile + 8 * p * kPitchT + ((p >> 3) << 6) + (((c >> 3) ^ ((p >> 1) & 3)) << 4) + 2 * (c & 7);
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int u = 0; u < 8; ++u)
        *reinterpret_cast<bf16raw *>(dst + u * kPitchT) = bf16raw(w[u >> 1] >> (16 * (u & 1)));
}
// operands of a 16-token tile that starts at row / column R0 (a multiple of 4) of the staged window
__device__ __forceinline__ bf16x8 tok_operand_at(const char *tile, int R0, int lane)
{
    const int row = R0 + (lane & 15), g = lane >> 4;
    return *reinterpret_cast<const bf16x8 *>(tile + row * kPitchT + (((row >> 6) & 1) << 6) + ((g ^ ((row >> 4) & 3)) << 4));
}
__device__ __forceinline__ bf16x8 chan_operand_at(const char *tile, int mt, int Ca, int Cb, int lane)
{
    const int m = lane & 15, g = lane >> 4;
    const char *row = tile + (16 * mt + m) * kLPitchC + 8 * g;
    const uint2 a = *reinterpret_cast<const uint2 *>(row + 2 * Ca);
    const uint2 b = *reinterpret_cast<const uint2 *>(row + 2 * Cb);
    const uint4 r = {a.x, a.y, b.x, b.y};
    return __builtin_bit_cast(bf16x8, r);
}
__device__ __forceinline__ void zero_lds(char *lds, int bytes, int tid)
{
    for (int i = tid; i < bytes / 4; i += 256) reinterpret_cast<unsigned *>(lds)[i] = 0u;
}

// The rows a workgroup of four consecutive latitudes [first, first + 4) ∩ [.., end) has to stage, and per row the
// largest half-width among them (uniform scalar code).
struct LightRows {
    int rmin, rmax;
    __device__ __forceinline__ void set(const int *blo, const int *bn, int first, int end)
    {
        rmin = 1 << 30;
        rmax = -1;
        for (int w = 0; w < 4; ++w) {
            const int hh = first + w;
            if (hh >= end) break;
            rmin = min(rmin, blo[hh]);
            rmax = max(rmax, blo[hh] + bn[hh] - 1);
        }
    }
};
// Row metadata of a workgroup, read from the grid tables ONCE before the row loop and kept in registers (lane i
// holds row rmin + i; the host guarantees at most 64 rows per workgroup): a table read inside the loop is a vector
// load whose wait also waits for the row prefetch in flight, which serialises the loop on memory latency.
//   hwm: largest half-width on that row among the workgroup's latitudes (defines the staged window)
//   hw:  this wavefront's half-width on that row, -1 if the row is not in its band
//   lw2: log2 of the row's relative quadrature weight
struct LightMeta {
    int hwm_v, hw_v;
    float lw2_v;
    __device__ __forceinline__ void load(const int *blo, const int *bn, const int *cnt, int bmax, const float *omega_rel,
                                         int first, int end, int own, bool active, const LightRows &rows, int lane)
    {
        const int r = rows.rmin + lane;
        const bool valid = r <= rows.rmax;
        hwm_v = 0;
        hw_v = -1;
        for (int w = 0; w < 4; ++w) {
            const int hh = first + w;
            if (hh >= end) break;
            const int b = r - blo[hh];
            if (valid && b >= 0 && b < bn[hh]) {
                const int x = (cnt[hh * bmax + b] - 1) >> 1;
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

__global__ void __launch_bounds__(256, 4)
nattn_fwd_bf16_light(S2DeviceTables t, int nbh, float c2, const bf16raw *__restrict__ q, const bf16raw *__restrict__ k,
                     const bf16raw *__restrict__ v, bf16raw *__restrict__ out, float *__restrict__ lse)
{
    __shared__ __attribute__((aligned(16))) char lds[kLTok + kLChan];
    const int nlon = t.nlon_in, ngrp = nlon >> 6, nseg = (t.bl_hi - t.bl_lo + 3) >> 2;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int seg = id % nseg, bh = id / nseg;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int first = t.bl_lo + 4 * seg, h = first + wave;
    const bool active = h < t.bl_hi;
    const int W0 = grp << 6, Wb = nlon + W0;
    const size_t plane = size_t(t.nlat_in) * nlon;
    const bf16raw *qs = q + size_t(bh) * kD * plane, *ks = k + size_t(bh) * kD * plane, *vs = v + size_t(bh) * kD * plane;
    char *Kt = lds, *Vc = lds + kLTok;

    bf16x8 qreg[4];
    f32x4 acc[4][2];
    float m[4], l[4];
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        if (active) qreg[o] = gather_point(qs, plane, size_t(h) * nlon + (W0 + 16 * o + n), g);
        acc[o][0] = acc[o][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        m[o] = -INFINITY;
        l[o] = 0.f;
    }
    LightRows rows;
    rows.set(t.band_lo, t.band_n, first, t.bl_hi);
    LightMeta meta;
    meta.load(t.band_lo, t.band_n, t.cnt, t.band_max, t.omega_rel, first, t.bl_hi, h, active, rows, lane);
    zero_lds(lds, kLTok + kLChan, tid);
    int X0 = (Wb - meta.hwmax(0)) & ~7;
    uint4 rk[2], rv[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        rk[j] = load_piece128(ks, plane, rows.rmin, nlon, X0, tid + 256 * j);
        rv[j] = load_piece128(vs, plane, rows.rmin, nlon, X0, tid + 256 * j);
    }
    for (int r = rows.rmin; r <= rows.rmax; ++r) {
        __syncthreads();                    // everybody is done with the previous row (first pass: with the zero fill)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            store_tok128(Kt, rk[j], tid + 256 * j);
            store_chan128(Vc, rv[j], tid + 256 * j);
        }
        __syncthreads();
        const int Xr = X0;                  // first staged column of this row
        if (r < rows.rmax) {
            X0 = (Wb - meta.hwmax(r + 1 - rows.rmin)) & ~7;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                rk[j] = load_piece128(ks, plane, r + 1, nlon, X0, tid + 256 * j);
                rv[j] = load_piece128(vs, plane, r + 1, nlon, X0, tid + 256 * j);
            }
        }
        const int hw = meta.hw(r - rows.rmin);
        if (hw < 0) continue;
        const float lw2 = meta.lw2(r - rows.rmin);
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            const int Wo = Wb + 16 * o;
            const int Xo = (Wo - hw) & ~3;                       // first key tile of this owner tile
            const int nt = (Wo + 16 + hw - Xo + 15) >> 4;        // key tiles that touch its band (at most 5)
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                if (2 * p >= nt) break;
                const int Xt0 = Xo + 32 * p, R0 = Xt0 - Xr;
                const bool two = 2 * p + 1 < nt;
                f32x4 x[2];
                float mx = -INFINITY;
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (u == 1 && !two) break;
                    const int Xt = Xt0 + 16 * u;
                    const f32x4 sc = mfma16(tok_operand_at(Kt, R0 + 16 * u, lane), qreg[o], f32x4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) x[u][rr] = fmaf(sc[rr], c2, lw2);
                    const int dlt = Xt > Wo ? Xt - Wo : Wo - Xt;
                    if (hw < 15 + dlt) {
                        const unsigned uu = unsigned(Xt + 4 * g - (Wo + n) + hw), lim = unsigned(2 * hw);
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) x[u][rr] = uu + rr <= lim ? x[u][rr] : -INFINITY;
                    }
                    mx = fmaxf(mx, fmaxf(fmaxf(x[u][0], x[u][1]), fmaxf(x[u][2], x[u][3])));
                }
                if (__any(mx > m[o] + 8.f)) {
                    mx = group_max(mx);
                    const float m_new = mx > m[o] + 8.f ? mx : m[o];
                    const float corr = m_new == m[o] ? 1.f : __builtin_amdgcn_exp2f(m[o] - m_new);
                    m[o] = m_new;
                    l[o] *= corr;
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) { acc[o][0][rr] *= corr; acc[o][1][rr] *= corr; }
                }
                const float ms = m[o] == -INFINITY ? 0.f : m[o];
                float ps = 0.f;
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (u == 0 || two) {
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) {
                            x[u][rr] = __builtin_amdgcn_exp2f(x[u][rr] - ms);
                            ps += x[u][rr];
                        }
                    } else {
                        x[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                }
                l[o] += ps;
                const bf16x8 pb = pack2(x[0], x[1]);
                acc[o][0] = mfma16(chan_operand_at(Vc, 0, R0, R0 + 16, lane), pb, acc[o][0]);
                acc[o][1] = mfma16(chan_operand_at(Vc, 1, R0, R0 + 16, lane), pb, acc[o][1]);
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        const float lt = group_sum(l[o]);
        const float inv = 1.f / lt;
        const size_t at = size_t(h) * nlon + (W0 + 16 * o + n);
        bf16raw *ob = out + size_t(bh) * kD * plane + at;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) ob[size_t(16 * mt + 4 * g + rr) * plane] = bf16_bits(acc[o][mt][rr] * inv);
        if (g == 0) lse[size_t(bh) * plane + at] = (m[o] + __log2f(lt)) * 0.6931471805599453f + t.ln_omega_ref;
    }
}

__global__ void __launch_bounds__(256, 2)
nattn_bwd_dq_bf16_light(S2DeviceTables t, int nbh, float scale, const bf16raw *__restrict__ q, const bf16raw *__restrict__ k,
                        const bf16raw *__restrict__ v, const bf16raw *__restrict__ o_, const float *__restrict__ lse,
                        const bf16raw *__restrict__ go, bf16raw *__restrict__ dq, float *__restrict__ Dws)
{
    __shared__ __attribute__((aligned(16))) char lds[2 * kLTok + kLChan];
    const int nlon = t.nlon_in, ngrp = nlon >> 6, nseg = (t.bl_hi - t.bl_lo + 3) >> 2;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int seg = id % nseg, bh = id / nseg;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int first = t.bl_lo + 4 * seg, h = first + wave;
    const bool active = h < t.bl_hi;
    const int W0 = grp << 6, Wb = nlon + W0;
    const size_t plane = size_t(t.nlat_in) * nlon;
    const bf16raw *qs = q + size_t(bh) * kD * plane, *ks = k + size_t(bh) * kD * plane, *vs = v + size_t(bh) * kD * plane;
    const bf16raw *os = o_ + size_t(bh) * kD * plane, *gs = go + size_t(bh) * kD * plane;
    const float c2 = scale * kLog2e;
    char *Kt = lds, *Vt = lds + kLTok, *Kc = lds + 2 * kLTok;

    bf16x8 qreg[4], greg[4];
    f32x4 acc[4][2];
    float L2[4], Dn[4];
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        acc[o][0] = acc[o][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        L2[o] = 0.f;
        Dn[o] = 0.f;
        if (active) {
            const size_t at = size_t(h) * nlon + (W0 + 16 * o + n);
            qreg[o] = gather_point(qs, plane, at, g);
            greg[o] = gather_point(gs, plane, at, g);
            const bf16x8 oo = gather_point(os, plane, at, g);
            float dsum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) dsum = fmaf(float(greg[o][j]), float(oo[j]), dsum);
            dsum = group_sum(dsum);
            if (g == 0) Dws[size_t(bh) * plane + at] = dsum;
            Dn[o] = -dsum;
            L2[o] = (lse[size_t(bh) * plane + at] - t.ln_omega_ref) * kLog2e;
        }
    }
    LightRows rows;
    rows.set(t.band_lo, t.band_n, first, t.bl_hi);
    LightMeta meta;
    meta.load(t.band_lo, t.band_n, t.cnt, t.band_max, t.omega_rel, first, t.bl_hi, h, active, rows, lane);
    zero_lds(lds, 2 * kLTok + kLChan, tid);
    int X0 = (Wb - meta.hwmax(0)) & ~7;
    uint4 rk[2], rv[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        rk[j] = load_piece128(ks, plane, rows.rmin, nlon, X0, tid + 256 * j);
        rv[j] = load_piece128(vs, plane, rows.rmin, nlon, X0, tid + 256 * j);
    }
    for (int r = rows.rmin; r <= rows.rmax; ++r) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            store_tok128(Kt, rk[j], tid + 256 * j);
            store_tok128(Vt, rv[j], tid + 256 * j);
            store_chan128(Kc, rk[j], tid + 256 * j);
        }
        __syncthreads();
        const int Xr = X0;
        if (r < rows.rmax) {
            X0 = (Wb - meta.hwmax(r + 1 - rows.rmin)) & ~7;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                rk[j] = load_piece128(ks, plane, r + 1, nlon, X0, tid + 256 * j);
                rv[j] = load_piece128(vs, plane, r + 1, nlon, X0, tid + 256 * j);
            }
        }
        const int hw = meta.hw(r - rows.rmin);
        if (hw < 0) continue;
        const float lw2 = meta.lw2(r - rows.rmin);
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            const int Wo = Wb + 16 * o;
            const int Xo = (Wo - hw) & ~3;
            const int nt = (Wo + 16 + hw - Xo + 15) >> 4;
            const float bias = lw2 - L2[o];
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                if (2 * p >= nt) break;
                const int Xt0 = Xo + 32 * p, R0 = Xt0 - Xr;
                const bool two = 2 * p + 1 < nt;
                f32x4 ds[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    ds[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (u == 1 && !two) break;
                    const int Xt = Xt0 + 16 * u;
                    const f32x4 sc = mfma16(tok_operand_at(Kt, R0 + 16 * u, lane), qreg[o], f32x4{0.f, 0.f, 0.f, 0.f});
                    const f32x4 dp = mfma16(tok_operand_at(Vt, R0 + 16 * u, lane), greg[o], f32x4{Dn[o], Dn[o], Dn[o], Dn[o]});
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) ds[u][rr] = __builtin_amdgcn_exp2f(fmaf(sc[rr], c2, bias)) * dp[rr];
                    const int dlt = Xt > Wo ? Xt - Wo : Wo - Xt;
                    if (hw < 15 + dlt) {
                        const unsigned uu = unsigned(Xt + 4 * g - (Wo + n) + hw), lim = unsigned(2 * hw);
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) ds[u][rr] = uu + rr <= lim ? ds[u][rr] : 0.f;
                    }
                }
                bf16x8 dh, dl;
                pack2_split(ds[0], ds[1], dh, dl);
                const bf16x8 k0 = chan_operand_at(Kc, 0, R0, R0 + 16, lane), k1 = chan_operand_at(Kc, 1, R0, R0 + 16, lane);
                acc[o][0] = mfma16(k0, dl, mfma16(k0, dh, acc[o][0]));
                acc[o][1] = mfma16(k1, dl, mfma16(k1, dh, acc[o][1]));
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        bf16raw *ob = dq + size_t(bh) * kD * plane + size_t(h) * nlon + (W0 + 16 * o + n);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) ob[size_t(16 * mt + 4 * g + rr) * plane] = bf16_bits(acc[o][mt][rr] * scale);
    }
}

__global__ void __launch_bounds__(256, 3)
nattn_bwd_dkdv_bf16_light(S2DeviceTables t, int nbh, float scale, const bf16raw *__restrict__ q, const bf16raw *__restrict__ k,
                          const bf16raw *__restrict__ v, const float *__restrict__ lse, const bf16raw *__restrict__ go,
                          const float *__restrict__ Dws, bf16raw *__restrict__ dk, bf16raw *__restrict__ dv)
{
    constexpr int kStats = 2 * kLRows * 4;
    __shared__ __attribute__((aligned(16))) char lds[2 * kLTok + 2 * kLChan + kStats];
    const int nlon = t.nlon_in, ngrp = nlon >> 6, nseg = (t.tbl_hi - t.tbl_lo + 3) >> 2;
    int id = blockIdx.x;
    const int grp = id % ngrp; id /= ngrp;
    const int seg = id % nseg, bh = id / nseg;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const int first = t.tbl_lo + 4 * seg, hp = first + wave;
    const bool active = hp < t.tbl_hi;
    const int W0 = grp << 6, Wb = nlon + W0;
    const size_t plane = size_t(t.nlat_in) * nlon;
    const bf16raw *qs = q + size_t(bh) * kD * plane, *ks = k + size_t(bh) * kD * plane, *vs = v + size_t(bh) * kD * plane;
    const bf16raw *gs = go + size_t(bh) * kD * plane;
    const float *ls = lse + size_t(bh) * plane, *Ds = Dws + size_t(bh) * plane;
    const float c2 = scale * kLog2e, lref = t.ln_omega_ref;
    const float lw2 = active ? __log2f(t.omega_rel[hp]) : 0.f;
    char *Qt = lds, *Gt = lds + kLTok, *Qc = lds + 2 * kLTok, *Gc = Qc + kLChan;
    float *Ls = reinterpret_cast<float *>(Gc + kLChan), *Dn = Ls + kLRows;

    bf16x8 kreg[4], vreg[4];
    f32x4 adk[4][2], adv[4][2];
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        adk[o][0] = adk[o][1] = adv[o][0] = adv[o][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (active) {
            const size_t at = size_t(hp) * nlon + (W0 + 16 * o + n);
            kreg[o] = gather_point(ks, plane, at, g);
            vreg[o] = gather_point(vs, plane, at, g);
        }
    }
    LightRows rows;
    rows.set(t.tband_lo, t.tband_n, first, t.tbl_hi);
    LightMeta meta;
    meta.load(t.tband_lo, t.tband_n, t.tcnt, t.tband_max, t.omega_rel, first, t.tbl_hi, hp, active, rows, lane);
    zero_lds(lds, 2 * kLTok + 2 * kLChan + kStats, tid);
    auto load_stat = [&](int lat, int Xs) -> float {      // threads 0..127: logsumexp (base 2, relative), 128..255: -D
        int col = Xs + (tid & 127);
        col = col >= nlon ? col - nlon : col;
        col = col >= nlon ? col - nlon : col;
        return tid < 128 ? (ls[size_t(lat) * nlon + col] - lref) * kLog2e : -Ds[size_t(lat) * nlon + col];
    };
    int X0 = (Wb - meta.hwmax(0)) & ~7;
    uint4 rq[2], rg[2];
    float rs;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        rq[j] = load_piece128(qs, plane, rows.rmin, nlon, X0, tid + 256 * j);
        rg[j] = load_piece128(gs, plane, rows.rmin, nlon, X0, tid + 256 * j);
    }
    rs = load_stat(rows.rmin, X0);
    for (int r = rows.rmin; r <= rows.rmax; ++r) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            store_tok128(Qt, rq[j], tid + 256 * j);
            store_tok128(Gt, rg[j], tid + 256 * j);
            store_chan128(Qc, rq[j], tid + 256 * j);
            store_chan128(Gc, rg[j], tid + 256 * j);
        }
        (tid < 128 ? Ls : Dn)[tid & 127] = rs;
        __syncthreads();
        const int Xr = X0;
        if (r < rows.rmax) {
            X0 = (Wb - meta.hwmax(r + 1 - rows.rmin)) & ~7;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                rq[j] = load_piece128(qs, plane, r + 1, nlon, X0, tid + 256 * j);
                rg[j] = load_piece128(gs, plane, r + 1, nlon, X0, tid + 256 * j);
            }
            rs = load_stat(r + 1, X0);
        }
        const int hw = meta.hw(r - rows.rmin);
        if (hw < 0) continue;
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            const int Wo = Wb + 16 * o;
            const int Xo = (Wo - hw) & ~3;
            const int nt = (Wo + 16 + hw - Xo + 15) >> 4;
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                if (2 * p >= nt) break;
                const int Xt0 = Xo + 32 * p, R0 = Xt0 - Xr;
                const bool two = 2 * p + 1 < nt;
                f32x4 pr[2], ds[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    pr[u] = ds[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (u == 1 && !two) break;
                    const int Xt = Xt0 + 16 * u, Ru = R0 + 16 * u;
                    const f32x4 L = *reinterpret_cast<const f32x4 *>(Ls + Ru + 4 * g);
                    const f32x4 Dm = *reinterpret_cast<const f32x4 *>(Dn + Ru + 4 * g);
                    const f32x4 sc = mfma16(tok_operand_at(Qt, Ru, lane), kreg[o], f32x4{0.f, 0.f, 0.f, 0.f});
                    const f32x4 dp = mfma16(tok_operand_at(Gt, Ru, lane), vreg[o], Dm);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        pr[u][rr] = __builtin_amdgcn_exp2f(fmaf(sc[rr], c2, lw2 - L[rr]));
                        ds[u][rr] = pr[u][rr] * dp[rr];
                    }
                    // both matrix results are consumed above, in the block that issues them: a consumer behind the
                    // uniform branch below is not covered by the compiler's wait-state bookkeeping for matrix results
                    const int dlt = Xt > Wo ? Xt - Wo : Wo - Xt;
                    if (hw < 15 + dlt) {
                        const unsigned uu = unsigned(Xt + 4 * g - (Wo + n) + hw), lim = unsigned(2 * hw);
#pragma unroll
                        for (int rr = 0; rr < 4; ++rr) {
                            const bool in = uu + rr <= lim;
                            pr[u][rr] = in ? pr[u][rr] : 0.f;
                            ds[u][rr] = in ? ds[u][rr] : 0.f;
                        }
                    }
                }
                bf16x8 ph, pl, dh, dl;
                pack2_split(pr[0], pr[1], ph, pl);
                pack2_split(ds[0], ds[1], dh, dl);
                const bf16x8 g0 = chan_operand_at(Gc, 0, R0, R0 + 16, lane), g1 = chan_operand_at(Gc, 1, R0, R0 + 16, lane);
                adv[o][0] = mfma16(g0, pl, mfma16(g0, ph, adv[o][0]));
                adv[o][1] = mfma16(g1, pl, mfma16(g1, ph, adv[o][1]));
                const bf16x8 q0 = chan_operand_at(Qc, 0, R0, R0 + 16, lane), q1 = chan_operand_at(Qc, 1, R0, R0 + 16, lane);
                adk[o][0] = mfma16(q0, dl, mfma16(q0, dh, adk[o][0]));
                adk[o][1] = mfma16(q1, dl, mfma16(q1, dh, adk[o][1]));
            }
        }
    }
    if (!active) return;
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        const size_t at = size_t(bh) * kD * plane + size_t(hp) * nlon + (W0 + 16 * o + n);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                dk[at + size_t(16 * mt + 4 * g + rr) * plane] = bf16_bits(adk[o][mt][rr] * scale);
                dv[at + size_t(16 * mt + 4 * g + rr) * plane] = bf16_bits(adv[o][mt][rr]);
            }
    }
}

}  // namespace

// Two launches per kernel: the latitudes of the three heavy classes (dense neighborhoods near the poles), then the
// light ones; the library's launch trace reports them separately.
// Owner tiles per wavefront of the one-latitude kernels: two (a workgroup owns 128 points).  With four the dense
// latitudes of the 129 x 256 workload are 512 workgroups, two wavefronts per SIMD, and the launches wait half of their
// time; with two: forward 0.145 -> 0.077 ms, dq 0.150 -> 0.087, dk/dv 0.203 -> 0.159 (one tile: the same again).
constexpr int kDenseTiles = 2;

template <class F>
static void launch_by_class(const S2DeviceTables &t, bool fwd_side, int nbh, const char *dense_name, const char *light_name,
                            hipStream_t st, F launch)
{
    const int *cls = fwd_side ? t.fwd_cls : t.bwd_cls;
    const double *pairs = fwd_side ? t.fwd_pairs : t.bwd_pairs;
    const int ngrp = (t.nlon_in + 64 * kDenseTiles - 1) / (64 * kDenseTiles);
    const int ndense = cls[0] + cls[1] + cls[2];
    if (ndense > 0) {
        S2TraceScope tr(dense_name, nbh * (pairs[0] + pairs[1] + pairs[2]), st);
        launch(0, unsigned(long(nbh) * ndense * ngrp));
    }
    if (cls[3] > 0) {
        S2TraceScope tr(light_name, nbh * pairs[3], st);
        const int lo = fwd_side ? t.bl_lo : t.tbl_lo, hi = fwd_side ? t.bl_hi : t.tbl_hi;
        if (hi - lo == cls[3])      // the light latitudes are a contiguous range of short arcs: four latitudes per workgroup
            launch(-1, unsigned(long(nbh) * ((hi - lo + 3) / 4) * (t.nlon_in / 64)));
        else
            launch(ndense, unsigned(long(nbh) * cls[3] * ngrp));
    }
}

int s2_nattn_fwd_bf16(const S2DeviceTables &t, int nbh, int, int, float scale, const void *q, const void *k,
                      const void *v, void *out, float *lse, hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    launch_by_class(t, true, nbh, "nattn_fwd_bf16<dense>", "nattn_fwd_bf16<light>", st, [&](int first, unsigned nblk) {
        if (first < 0) {
            hipLaunchKernelGGL(nattn_fwd_bf16_light, dim3(nblk), dim3(256), 0, st, t, nbh, scale * kLog2e,
                               static_cast<const bf16raw *>(q), static_cast<const bf16raw *>(k),
                               static_cast<const bf16raw *>(v), static_cast<bf16raw *>(out), lse);
            return;
        }
        hipLaunchKernelGGL(nattn_fwd_bf16<kDenseTiles>, dim3(nblk), dim3(256), 0, st, t, nbh, first, scale * kLog2e,
                           static_cast<const bf16raw *>(q), static_cast<const bf16raw *>(k),
                           static_cast<const bf16raw *>(v), static_cast<bf16raw *>(out), lse);
    });
    return 0;
}

int s2_nattn_bwd_dq_bf16(const S2DeviceTables &t, int nbh, int, int, float scale, const void *q, const void *k,
                         const void *v, const void *o, const float *lse, const void *go, void *dq, float *Dws,
                         hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    launch_by_class(t, true, nbh, "nattn_bwd_dq_bf16<dense>", "nattn_bwd_dq_bf16<light>", st, [&](int first, unsigned nblk) {
        if (first < 0) {
            hipLaunchKernelGGL(nattn_bwd_dq_bf16_light, dim3(nblk), dim3(256), 0, st, t, nbh, scale,
                               static_cast<const bf16raw *>(q), static_cast<const bf16raw *>(k),
                               static_cast<const bf16raw *>(v), static_cast<const bf16raw *>(o), lse,
                               static_cast<const bf16raw *>(go), static_cast<bf16raw *>(dq), Dws);
            return;
        }
        hipLaunchKernelGGL(nattn_bwd_dq_bf16<kDenseTiles>, dim3(nblk), dim3(256), 0, st, t, nbh, first, scale,
                           static_cast<const bf16raw *>(q), static_cast<const bf16raw *>(k),
                           static_cast<const bf16raw *>(v), static_cast<const bf16raw *>(o), lse,
                           static_cast<const bf16raw *>(go), static_cast<bf16raw *>(dq), Dws);
    });
    return 0;
}

int s2_nattn_bwd_dkdv_bf16(const S2DeviceTables &t, int nbh, int, int, float scale, const void *q, const void *k,
                           const void *v, const float *lse, const void *go, const float *Dws, void *dk, void *dv,
                           hipStream_t st)
{
    if (s2_debug_flag(S2_DEBUG_FAIL_LAUNCH)) return -1;
    launch_by_class(t, false, nbh, "nattn_bwd_dkdv_bf16<dense>", "nattn_bwd_dkdv_bf16<light>", st, [&](int first, unsigned nblk) {
        if (first < 0) {
            hipLaunchKernelGGL(nattn_bwd_dkdv_bf16_light, dim3(nblk), dim3(256), 0, st, t, nbh, scale,
                               static_cast<const bf16raw *>(q), static_cast<const bf16raw *>(k),
                               static_cast<const bf16raw *>(v), lse, static_cast<const bf16raw *>(go), Dws,
                               static_cast<bf16raw *>(dk), static_cast<bf16raw *>(dv));
            return;
        }
        hipLaunchKernelGGL(nattn_bwd_dkdv_bf16<kDenseTiles>, dim3(nblk), dim3(256), 0, st, t, nbh, first, scale,
                           static_cast<const bf16raw *>(q), static_cast<const bf16raw *>(k),
                           static_cast<const bf16raw *>(v), lse, static_cast<const bf16raw *>(go), Dws,
                           static_cast<bf16raw *>(dk), static_cast<bf16raw *>(dv));
    });
    return 0;
}
