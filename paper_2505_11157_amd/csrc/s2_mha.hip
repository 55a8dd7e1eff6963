// Spherical multi-head attention sub-block (Sec. 3.4 "Spherical attention blocks": pre-norm, residual) around the
// neighborhood attention kernels, float32:
//     xhat = instance norm of x per (batch, channel) over the grid points (plain moments, biased variance)
//     xn   = gamma xhat + beta + pos
//     q, k, v = Wq xn + bq, Wk xn + bk, Wv xn + bv          (1x1 convolutions; head i owns channels i d .. (i+1) d - 1,
//                                                            which is the [batch][heads][d] layout of the kernels)
//     a    = s2_nattn_fwd(q, k, v), scale 1 / sqrt(d)
//     y    = x + Wo a + bo
// and its backward.  The channel matrices run on the fp32 matrix cores (v_mfma_f32_32x32x2_f32).  Up to 128 channels
// (multiples of 32 rows, 64 columns) the weight matrix stays in LDS and every wavefront streams its own 32 grid
// points of the activations straight from memory (mha_gemm_wres); otherwise a workgroup of four wavefronts owns a
// 128 x 128 tile of the output, each wavefront 64 x 64 (2 x 2 matrix tiles), operands staged through LDS in slices
// of 16 along the contraction (mha_gemm).  Weight gradients contract over batch and grid points
// (hundreds of thousands of terms): split over workgroups into partial sums that a second launch adds in a fixed
// order, so every result is bit-reproducible.
#include <algorithm>
#include <initializer_list>

#include "s2_nattn_kernels.h"

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTM = 128, kTN = 128, kTK = 16;
constexpr int kPitch = kTM + 4;      // LDS row pitch of the k-major operand tiles (floats)
constexpr int kPitchW = kTK + 1;     // pitch of the row-major tiles of the weight-gradient kernel

__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// C[b][m][n] (+)= sum_k A(m, k) X[b][k][n] + bias[m] + R[b][m][n]
// A(m, k) = W[m * K + k] (TRANS_A = false, W is M x K) or W[k * M + m] (TRANS_A = true, W is K x M).
// M, K multiples of 16; N a multiple of 4.  grid (ceil(N / 128), ceil(M / 128), batch), 256 threads.
template <bool TRANS_A>
__global__ void __launch_bounds__(256)
mha_gemm(int M, int N, int K, const float *__restrict__ W, const float *__restrict__ X, const float *__restrict__ bias,
         const float *__restrict__ R, float *__restrict__ C, int accumulate)
{
    __shared__ float As[2][kTK * kPitch];      // [k][m]
    __shared__ float Bs[2][kTK * kPitch];      // [k][n]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * kTN, m0 = blockIdx.y * kTM;
    const float *Xb = X + size_t(blockIdx.z) * K * N;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int col = lane & 31, kk = lane >> 5;

    float4 ra[2], rb[2];
    auto load = [&](int k0) {
        if constexpr (TRANS_A) {
            const int kr = tid >> 4, mo = (tid & 15) * 8;      // row k0 + kr of W, columns m0 + mo .. + 7
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int m = m0 + mo + 4 * j;
                ra[j] = m < M ? *reinterpret_cast<const float4 *>(W + size_t(k0 + kr) * M + m) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        } else {
            const int mr = tid >> 1, ko = (tid & 1) * 8;       // row m0 + mr of W, columns k0 + ko .. + 7
#pragma unroll
            for (int j = 0; j < 2; ++j)
                ra[j] = m0 + mr < M ? *reinterpret_cast<const float4 *>(W + size_t(m0 + mr) * K + k0 + ko + 4 * j)
                                    : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        const int kr = tid >> 4, no = (tid & 15) * 8;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + no + 4 * j;
            rb[j] = n < N ? *reinterpret_cast<const float4 *>(Xb + size_t(k0 + kr) * N + n) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto store = [&](int buf) {
        if constexpr (TRANS_A) {
            const int kr = tid >> 4, mo = (tid & 15) * 8;
            *reinterpret_cast<float4 *>(&As[buf][kr * kPitch + mo]) = ra[0];
            *reinterpret_cast<float4 *>(&As[buf][kr * kPitch + mo + 4]) = ra[1];
        } else {
            const int mr = tid >> 1, ko = (tid & 1) * 8;
            const float v[8] = {ra[0].x, ra[0].y, ra[0].z, ra[0].w, ra[1].x, ra[1].y, ra[1].z, ra[1].w};
#pragma unroll
            for (int j = 0; j < 8; ++j) As[buf][(ko + j) * kPitch + mr] = v[j];
        }
        const int kr = tid >> 4, no = (tid & 15) * 8;
        *reinterpret_cast<float4 *>(&Bs[buf][kr * kPitch + no]) = rb[0];
        *reinterpret_cast<float4 *>(&Bs[buf][kr * kPitch + no + 4]) = rb[1];
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    load(0);
    store(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = 0; k0 < K; k0 += kTK) {
        const bool more = k0 + kTK < K;
        if (more) load(k0 + kTK);
#pragma unroll
        for (int s = 0; s < kTK / 2; ++s) {
            const float *ar = &As[buf][(2 * s + kk) * kPitch + wm + col], *br = &Bs[buf][(2 * s + kk) * kPitch + wn + col];
            const float a0 = ar[0], a1 = ar[32], b0 = br[0], b1 = br[32];
            acc[0][0] = mfma32(a0, b0, acc[0][0]);
            acc[0][1] = mfma32(a0, b1, acc[0][1]);
            acc[1][0] = mfma32(a1, b0, acc[1][0]);
            acc[1][1] = mfma32(a1, b1, acc[1][1]);
        }
        if (more) {
            store(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }
    float *Cb = C + size_t(blockIdx.z) * M * N;
    const float *Rb = R ? R + size_t(blockIdx.z) * M * N : nullptr;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn + 32 * j + col;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm + 32 * i + 8 * (e >> 2) + 4 * kk + (e & 3);
                if (m < M && n < N) {
                    float x = acc[i][j][e];
                    if (bias) x += bias[m];
                    if (Rb) x += Rb[size_t(m) * N + n];
                    if (accumulate) x += Cb[size_t(m) * N + n];
                    Cb[size_t(m) * N + n] = x;
                }
            }
        }
}

// The same product for small channel counts (M <= 128 a multiple of 32, K a multiple of 64, the whole weight matrix in
// LDS): no staging of X and no barrier in the loop.  A workgroup of eight wavefronts copies W to LDS once ([k][m],
// pitch = 33 mod 64: the two k rows one matrix instruction reads lie 33 banks apart) and then walks over tiles of 32
// grid points; a wavefront owns a whole tile (all M rows, MT = M / 32 accumulators), reads its operand of X straight
// from memory (lane (column, half) reads X[2 s + half][n0 + column]: each element of X is read once, by one lane, in
// 128-byte row pieces, 16 steps ahead of their use; the first 16 steps of the NEXT tile are requested before the
// results of this one are stored, so they do not queue behind the stores) and its operand of W from LDS.
// The tiles are dealt out in whole rounds; what is left over after the last whole round (fewer tiles than wavefronts)
// is cut into its MT row blocks and dealt out again, so the last round costs 1 / MT of a tile.
struct WresTile {       // where a wavefront's operand of X starts and where its results go
    const char *rp;     // uniform: row 0 of X[b]
    unsigned lane_off;  // bytes: (half * N + column); lanes past the last column read column 0 (a valid address, no
                        // branch around the loads: a branch per load makes the compiler wait for all loads in flight
                        // at every merge) and store nothing
    int b, n;
    bool ok;
};
__device__ __forceinline__ WresTile wres_tile(int t, int tiles_per_batch, int N, int K, const float *X, int col, int kk)
{
    WresTile w;
    w.b = t / tiles_per_batch;
    w.n = (t - w.b * tiles_per_batch) * 32 + col;
    w.ok = w.n < N;
    w.rp = reinterpret_cast<const char *>(X + size_t(w.b) * K * N);
    w.lane_off = unsigned((size_t(kk) * N + (w.ok ? w.n : 0)) * sizeof(float));
    // a uniform running row pointer plus one 32-bit lane offset, kept opaque so that the compiler does not park a
    // 64-bit lane address per load in registers
    asm volatile("" : "+s"(w.rp));
    asm volatile("" : "+v"(w.lane_off));
    return w;
}
__device__ __forceinline__ void wres_fetch(WresTile &w, size_t step_bytes, float (&x)[16])
{
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        // (an explicitly global load: a flat one also counts as an LDS access, and every wait for an operand of W
        // would then wait for all the loads of X in flight)
        x[j] = *(const __attribute__((address_space(1))) float *)(w.rp + w.lane_off);
        w.rp += step_bytes;
    }
    __builtin_amdgcn_sched_barrier(0);      // the requests stay in front of the arithmetic they are meant to overlap
}
// all K steps of one tile for MT row blocks starting at row m0 of W; xa holds the first 16 steps on entry
template <int MT>
__device__ __forceinline__ void wres_contract(WresTile &w, size_t step_bytes, int K, int pitch, const float *wl,
                                              float (&xa)[16], f32x16 (&acc)[MT])
{
    float xb[16];
    for (int s0 = 0; s0 < K / 2; s0 += 32) {       // 32 steps (64 values of k) per pass, in two halves
        wres_fetch(w, step_bytes, xb);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float *wr = wl + 2 * (s0 + j) * pitch;
#pragma unroll
            for (int i = 0; i < MT; ++i) acc[i] = mfma32(wr[32 * i], xa[j], acc[i]);
        }
        if (s0 + 32 < K / 2) wres_fetch(w, step_bytes, xa);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float *wr = wl + 2 * (s0 + 16 + j) * pitch;
#pragma unroll
            for (int i = 0; i < MT; ++i) acc[i] = mfma32(wr[32 * i], xb[j], acc[i]);
        }
    }
}
// results of one tile: per row block all the reads (bias, residual, old value) are issued before the first store, so
// they overlap instead of each waiting for the store in front of it
template <int MT>
__device__ __forceinline__ void wres_store(const f32x16 (&acc)[MT], int M, int N, int m0, int b, int n, int kk,
                                           const float *__restrict__ bias, const float *__restrict__ R,
                                           float *__restrict__ C, int accumulate)
{
    float *Cb = C + size_t(b) * M * N + n;
    const float *Rb = R ? R + size_t(b) * M * N + n : nullptr;
#pragma unroll
    for (int i = 0; i < 2 * MT; ++i) {      // half a row block (eight rows per lane) at a time
        float add[8], res[8], old[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int m = m0 + 16 * i + 8 * (e >> 2) + 4 * kk + (e & 3);
            add[e] = bias ? bias[m] : 0.f;
            res[e] = Rb ? Rb[size_t(m) * N] : 0.f;
            old[e] = accumulate ? Cb[size_t(m) * N] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int m = m0 + 16 * i + 8 * (e >> 2) + 4 * kk + (e & 3);
            Cb[size_t(m) * N] = ((acc[i >> 1][8 * (i & 1) + e] + add[e]) + res[e]) + old[e];
        }
    }
}

template <bool TRANS_A, int MT>
__global__ void __launch_bounds__(512)
mha_gemm_wres(int M, int N, int K, int pitch, int tiles_per_batch, int ntiles, const float *__restrict__ W,
              const float *__restrict__ X, const float *__restrict__ bias, const float *__restrict__ R,
              float *__restrict__ C, int accumulate)
{
    extern __shared__ __attribute__((aligned(16))) float Ws[];      // [K][pitch]
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, kk = lane >> 5;
    const int nwaves = gridDim.x * 8, me = blockIdx.x * 8 + wave;
    const int whole = ntiles / nwaves * nwaves;         // tiles of the whole rounds
    const size_t step_bytes = size_t(2) * N * sizeof(float);
    const float *wl = Ws + kk * pitch + col;

    // the first operands are requested before W is copied
    float xa[16];
    WresTile cur = wres_tile(me < whole ? me : 0, tiles_per_batch, N, K, X, col, kk);
    if (me < whole) wres_fetch(cur, step_bytes, xa);

    for (int i0 = tid; i0 < (M * K) >> 2; i0 += 4 * 512) {      // four 16-byte pieces in flight per thread
        float4 w4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + 512 * u;
            w4[u] = i < (M * K) >> 2 ? *reinterpret_cast<const float4 *>(W + 4 * i) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + 512 * u;
            if (i >= (M * K) >> 2) break;
            const float4 w = w4[u];
            if constexpr (TRANS_A) {      // W is K x M: rows are copied as they are
                const int k = (4 * i) / M, m = 4 * i - k * M;
                float *d = Ws + k * pitch + m;
                d[0] = w.x; d[1] = w.y; d[2] = w.z; d[3] = w.w;
            } else {                      // W is M x K: transposed on the way
                const int m = (4 * i) / K, k = 4 * i - m * K;
                float *d = Ws + k * pitch + m;
                d[0] = w.x; d[pitch] = w.y; d[2 * pitch] = w.z; d[3 * pitch] = w.w;
            }
        }
    }
    __syncthreads();

    for (int t = me; t < whole; t += nwaves) {
        f32x16 acc[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
        wres_contract<MT>(cur, step_bytes, K, pitch, wl, xa, acc);
        const int b = cur.b, n = cur.n;
        const bool ok = cur.ok;
        if (t + nwaves < whole) {
            cur = wres_tile(t + nwaves, tiles_per_batch, N, K, X, col, kk);
            wres_fetch(cur, step_bytes, xa);
        }
        if (ok) wres_store<MT>(acc, M, N, 0, b, n, kk, bias, R, C, accumulate);
    }
    // the tiles of the last, partial round, one row block per wavefront
    for (int u = me; u < (ntiles - whole) * MT; u += nwaves) {
        const int t = whole + u / MT, m0 = 32 * (u % MT);
        WresTile w = wres_tile(t, tiles_per_batch, N, K, X, col, kk);
        wres_fetch(w, step_bytes, xa);
        f32x16 acc[1];
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[0][e] = 0.f;
        wres_contract<1>(w, step_bytes, K, pitch, wl + m0, xa, acc);
        if (w.ok) wres_store<1>(acc, M, N, m0, w.b, w.n, kk, bias, R, C, accumulate);
    }
}

// LDS row pitch of the resident weight matrix: the smallest p >= M with p = 33 mod 64
inline int wres_pitch(int M) { return (M + 30) / 64 * 64 + 33; }
inline int num_compute_units()
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
inline bool wres_ok(int M, int K)
{
    return M % 32 == 0 && M <= 128 && K % 64 == 0 && size_t(K) * wres_pitch(M) * sizeof(float) <= 160 * 1024;
}

// Partial weight gradients: part[split][m][k] = sum over the split's share of (batch, grid point) of
// dY[b][m][n] X[b][k][n].  M, K multiples of 16, N a multiple of 16.  grid (ceil(K / 128), ceil(M / 128), splits).
__global__ void __launch_bounds__(256)
mha_wgrad_partial(int M, int K, int N, int batch, int nsplit, const float *__restrict__ dY, const float *__restrict__ X,
                  float *__restrict__ part)
{
    __shared__ float Ys[2][kTM * kPitchW];     // [m][n']
    __shared__ float Xs[2][kTN * kPitchW];     // [k][n']
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int k0t = blockIdx.x * kTN, m0 = blockIdx.y * kTM, split = blockIdx.z;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int col = lane & 31, kk = lane >> 5;
    const long chunks = long(batch) * (N / kTK);
    const long c_lo = chunks * split / nsplit, c_hi = chunks * (split + 1) / nsplit;
    const int row = tid >> 1, off = (tid & 1) * 8;

    float4 ry[2], rx[2];
    auto load = [&](long c) {
        const int b = int(c / (N / kTK)), nn = int(c % (N / kTK)) * kTK + off;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            ry[j] = m0 + row < M ? *reinterpret_cast<const float4 *>(dY + (size_t(b) * M + m0 + row) * N + nn + 4 * j)
                                 : make_float4(0.f, 0.f, 0.f, 0.f);
            rx[j] = k0t + row < K ? *reinterpret_cast<const float4 *>(X + (size_t(b) * K + k0t + row) * N + nn + 4 * j)
                                  : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto store = [&](int buf) {
        const float y[8] = {ry[0].x, ry[0].y, ry[0].z, ry[0].w, ry[1].x, ry[1].y, ry[1].z, ry[1].w};
        const float x[8] = {rx[0].x, rx[0].y, rx[0].z, rx[0].w, rx[1].x, rx[1].y, rx[1].z, rx[1].w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            Ys[buf][row * kPitchW + off + j] = y[j];
            Xs[buf][row * kPitchW + off + j] = x[j];
        }
    };
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    if (c_lo < c_hi) {
        load(c_lo);
        store(0);
    }
    __syncthreads();
    int buf = 0;
    for (long c = c_lo; c < c_hi; ++c) {
        const bool more = c + 1 < c_hi;
        if (more) load(c + 1);
#pragma unroll
        for (int s = 0; s < kTK / 2; ++s) {
            const float a0 = Ys[buf][(wm + col) * kPitchW + 2 * s + kk], a1 = Ys[buf][(wm + 32 + col) * kPitchW + 2 * s + kk];
            const float b0 = Xs[buf][(wn + col) * kPitchW + 2 * s + kk], b1 = Xs[buf][(wn + 32 + col) * kPitchW + 2 * s + kk];
            acc[0][0] = mfma32(a0, b0, acc[0][0]);
            acc[0][1] = mfma32(a0, b1, acc[0][1]);
            acc[1][0] = mfma32(a1, b0, acc[1][0]);
            acc[1][1] = mfma32(a1, b1, acc[1][1]);
        }
        if (more) {
            store(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }
    float *P = part + size_t(split) * M * K;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int k = k0t + wn + 32 * j + col;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm + 32 * i + 8 * (e >> 2) + 4 * kk + (e & 3);
                if (m < M && k < K) P[size_t(m) * K + k] = acc[i][j][e];
            }
        }
}

// out[i] = sum of the nsplit partial values of element i.  A workgroup owns 64 elements; thread (q, e) adds the
// partials q, q + 4, q + 8, ... of element e (four chains of loads in flight per element), and the four chain sums
// are added in a fixed order: bit-reproducible.
__global__ void __launch_bounds__(256)
mha_sum_partials(int count, int nsplit, const float *__restrict__ part, float *__restrict__ out)
{
    __shared__ float red[4][64];
    const int e = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + e;
    float s = 0.f;
    if (i < count)
        for (int p = q; p < nsplit; p += 4) s += part[size_t(p) * count + i];
    red[q][e] = s;
    __syncthreads();
    if (q == 0 && i < count) out[i] = (red[0][e] + red[1][e]) + (red[2][e] + red[3][e]);
}

// block-wide sum of one value per thread (256 threads), result in every thread; fixed order
__device__ __forceinline__ float block_sum(float x, float *red)
{
    const int tid = threadIdx.x;
    red[tid] = x;
    __syncthreads();
#pragma unroll
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

// Instance normalisation: one workgroup per (batch, channel): mean and 1 / sqrt(var + eps) over the N grid points
// (two passes: the moments are taken about the mean), then xn = gamma xhat + beta + pos.  N is a multiple of 4 and the
// rows are 16-byte aligned: 16-byte accesses, each lane with four running sums (one per component) that are added in a
// fixed order.
__device__ __forceinline__ float sum4(float4 a) { return (a.x + a.y) + (a.z + a.w); }

__global__ void __launch_bounds__(256)
mha_instnorm_fwd(int C, int N, float eps, const float *__restrict__ x, const float *__restrict__ gamma,
                 const float *__restrict__ beta, const float *__restrict__ pos, float *__restrict__ mean,
                 float *__restrict__ rstd, float *__restrict__ xn)
{
    __shared__ float red[256];
    const int bc = blockIdx.x, c = bc % C, tid = threadIdx.x, n4 = N >> 2;
    const float4 *xr = reinterpret_cast<const float4 *>(x + size_t(bc) * N);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int i = tid; i < n4; i += 256) {
        const float4 a = xr[i];
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    }
    const float mu = block_sum(sum4(s), red) / float(N);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int i = tid; i < n4; i += 256) {
        const float4 a = xr[i];
        const float dx = a.x - mu, dy = a.y - mu, dz = a.z - mu, dw = a.w - mu;
        v.x = fmaf(dx, dx, v.x); v.y = fmaf(dy, dy, v.y); v.z = fmaf(dz, dz, v.z); v.w = fmaf(dw, dw, v.w);
    }
    const float rs = 1.f / sqrtf(block_sum(sum4(v), red) / float(N) + eps);
    if (tid == 0) { mean[bc] = mu; rstd[bc] = rs; }
    const float ga = gamma ? gamma[c] : 1.f, be = beta ? beta[c] : 0.f;
    const float4 *pr = pos ? reinterpret_cast<const float4 *>(pos + size_t(c) * N) : nullptr;
    float4 *o = reinterpret_cast<float4 *>(xn + size_t(bc) * N);
#pragma unroll 4
    for (int i = tid; i < n4; i += 256) {
        const float4 a = xr[i], p = pr ? pr[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        o[i] = make_float4(fmaf(ga, (a.x - mu) * rs, be) + p.x, fmaf(ga, (a.y - mu) * rs, be) + p.y,
                           fmaf(ga, (a.z - mu) * rs, be) + p.z, fmaf(ga, (a.w - mu) * rs, be) + p.w);
    }
}

// dx = dy + rstd (dxhat - mean(dxhat) - xhat mean(dxhat xhat)), dxhat = gamma dxn; one workgroup per (batch, channel)
__global__ void __launch_bounds__(256)
mha_instnorm_bwd(int C, int N, const float *__restrict__ x, const float *__restrict__ gamma, const float *__restrict__ mean,
                 const float *__restrict__ rstd, const float *__restrict__ dxn, const float *__restrict__ dy,
                 float *__restrict__ dx)
{
    __shared__ float red[256];
    const int bc = blockIdx.x, c = bc % C, tid = threadIdx.x, n4 = N >> 2;
    const float mu = mean[bc], rs = rstd[bc], ga = gamma ? gamma[c] : 1.f;
    const float4 *xr = reinterpret_cast<const float4 *>(x + size_t(bc) * N);
    const float4 *gr = reinterpret_cast<const float4 *>(dxn + size_t(bc) * N);
    const float4 *yr = reinterpret_cast<const float4 *>(dy + size_t(bc) * N);
    float4 s1 = make_float4(0.f, 0.f, 0.f, 0.f), s2 = s1;
#pragma unroll 2
    for (int i = tid; i < n4; i += 256) {
        const float4 g = gr[i], a = xr[i];
        const float hx = ga * g.x, hy = ga * g.y, hz = ga * g.z, hw = ga * g.w;
        s1.x += hx; s1.y += hy; s1.z += hz; s1.w += hw;
        s2.x = fmaf(hx, (a.x - mu) * rs, s2.x); s2.y = fmaf(hy, (a.y - mu) * rs, s2.y);
        s2.z = fmaf(hz, (a.z - mu) * rs, s2.z); s2.w = fmaf(hw, (a.w - mu) * rs, s2.w);
    }
    const float m1 = block_sum(sum4(s1), red) / float(N), m2 = block_sum(sum4(s2), red) / float(N);
    float4 *o = reinterpret_cast<float4 *>(dx + size_t(bc) * N);
#pragma unroll 2
    for (int i = tid; i < n4; i += 256) {
        const float4 g = gr[i], a = xr[i], y = yr[i];
        o[i] = make_float4(y.x + rs * (ga * g.x - m1 - (a.x - mu) * rs * m2), y.y + rs * (ga * g.y - m1 - (a.y - mu) * rs * m2),
                           y.z + rs * (ga * g.z - m1 - (a.z - mu) * rs * m2), y.w + rs * (ga * g.w - m1 - (a.w - mu) * rs * m2));
    }
}

// out[c] = sum over batch and grid points of u[b][c][n] (* xhat[b][c][n] if x is given); one workgroup per channel.
// 16-byte loads, four independent partial sums per thread (several loads in flight; the order of the additions is
// fixed, so the result is bit-reproducible).
__global__ void __launch_bounds__(256)
mha_channel_sum(int batch, int C, int N, const float *__restrict__ u, const float *__restrict__ x,
                const float *__restrict__ mean, const float *__restrict__ rstd, float *__restrict__ out)
{
    __shared__ float red[256];
    const int c = blockIdx.x, tid = threadIdx.x;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    const int n4 = (N % 4 == 0) ? N / 4 : 0;          // rows that are not 16-byte multiples take the scalar loop
    for (int b = 0; b < batch; ++b) {
        const float *ur = u + (size_t(b) * C + c) * N;
        const float4 *u4 = reinterpret_cast<const float4 *>(ur);
        if (x) {
            const float *xr = x + (size_t(b) * C + c) * N;
            const float4 *x4 = reinterpret_cast<const float4 *>(xr);
            const float mu = mean[b * C + c], rs = rstd[b * C + c];
            for (int i0 = tid; i0 < n4; i0 += 1024) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = i0 + 256 * j;
                    if (i < n4) {
                        const float4 a = u4[i], v = x4[i];
                        s[j] = fmaf(a.x, (v.x - mu) * rs, s[j]);
                        s[j] = fmaf(a.y, (v.y - mu) * rs, s[j]);
                        s[j] = fmaf(a.z, (v.z - mu) * rs, s[j]);
                        s[j] = fmaf(a.w, (v.w - mu) * rs, s[j]);
                    }
                }
            }
            for (int i = 4 * n4 + tid; i < N; i += 256) s[0] = fmaf(ur[i], (xr[i] - mu) * rs, s[0]);
        } else {
            for (int i0 = tid; i0 < n4; i0 += 1024) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = i0 + 256 * j;
                    if (i < n4) {
                        const float4 a = u4[i];
                        s[j] += (a.x + a.y) + (a.z + a.w);
                    }
                }
            }
            for (int i = 4 * n4 + tid; i < N; i += 256) s[0] += ur[i];
        }
    }
    const float r = block_sum((s[0] + s[1]) + (s[2] + s[3]), red);
    if (tid == 0) out[c] = r;
}

// The same sum in two launches for rows that are multiples of 16 bytes: workgroup (c, p) adds piece p % seg of row
// (batch element p / seg, channel c) into part[p][c]; mha_sum_partials adds the pieces in order.  Many more workgroups
// than channels (one workgroup per channel leaves most of the device idle), still a fixed order of additions.
__global__ void __launch_bounds__(256)
mha_channel_sum_pieces(int C, int N, int seg, const float *__restrict__ u, const float *__restrict__ x,
                       const float *__restrict__ mean, const float *__restrict__ rstd, float *__restrict__ part)
{
    __shared__ float red[256];
    const int c = blockIdx.x, p = blockIdx.y, b = p / seg, tid = threadIdx.x;
    const int n4 = N >> 2, len = (n4 + seg - 1) / seg, lo = (p - b * seg) * len, hi = min(n4, lo + len);
    const float4 *u4 = reinterpret_cast<const float4 *>(u + (size_t(b) * C + c) * N);
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    if (x) {
        const float4 *x4 = reinterpret_cast<const float4 *>(x + (size_t(b) * C + c) * N);
        const float mu = mean[b * C + c], rs = rstd[b * C + c];
        for (int i0 = lo + tid; i0 < hi; i0 += 1024) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + 256 * j;
                if (i < hi) {
                    const float4 a = u4[i], v = x4[i];
                    s[j] = fmaf(a.x, (v.x - mu) * rs, s[j]);
                    s[j] = fmaf(a.y, (v.y - mu) * rs, s[j]);
                    s[j] = fmaf(a.z, (v.z - mu) * rs, s[j]);
                    s[j] = fmaf(a.w, (v.w - mu) * rs, s[j]);
                }
            }
        }
    } else {
        for (int i0 = lo + tid; i0 < hi; i0 += 1024) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = i0 + 256 * j;
                if (i < hi) {
                    const float4 a = u4[i];
                    s[j] += (a.x + a.y) + (a.z + a.w);
                }
            }
        }
    }
    const float r = block_sum((s[0] + s[1]) + (s[2] + s[3]), red);
    if (tid == 0) part[size_t(p) * C + c] = r;
}

// dpos[c][n] = sum_b dxn[b][c][n]
__global__ void __launch_bounds__(256)
mha_batch_sum(int batch, size_t CN, const float *__restrict__ u, float *__restrict__ out)
{
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= CN) return;
    float s = 0.f;
    for (int b = 0; b < batch; ++b) s += u[size_t(b) * CN + i];
    out[i] = s;
}

// Split-K weight gradients: enough splits that the launch has about three workgroups per compute unit (at least 64, at
// most 512); the partial sums are added in split order by a second launch, so the result does not depend on timing.
inline int wgrad_splits(int M, int K)
{
    const int tiles = ((M + 127) / 128) * ((K + 127) / 128);
    return std::min(512, std::max(64, 768 / tiles));
}

struct Layout {      // offsets (in floats) into the workspace
    size_t mean, rstd, xn, q, k, v, a, lse, da, dq, dk, dv, dxn, D, part, total;
};
Layout layout(const s2_grid_t *g, int batch, int C, int heads)
{
    const size_t N = size_t(g->nlat_in) * g->nlon_in, T = size_t(batch) * C * N;
    auto up = [](size_t x) { return (x + 63) / 64 * 64; };      // 256-byte pieces
    Layout L{};
    size_t at = 0;
    L.mean = at; at += up(size_t(batch) * C);
    L.rstd = at; at += up(size_t(batch) * C);
    L.xn = at; at += up(T);
    L.q = at; at += up(T);
    L.k = at; at += up(T);
    L.v = at; at += up(T);
    L.a = at; at += up(T);
    L.lse = at; at += up(size_t(batch) * heads * N);
    L.da = at; at += up(T);
    L.dq = at; at += up(T);
    L.dk = at; at += up(T);
    L.dv = at; at += up(T);
    L.dxn = at; at += up(T);
    L.D = at; at += up(size_t(batch) * heads * N);
    L.part = at; at += up(size_t(wgrad_splits(C, C)) * C * C);
    L.total = at;
    return L;
}

// the kernels read tensors and weight matrices in 16-byte pieces (NULL = an optional tensor that is absent)
bool aligned16(std::initializer_list<const void *> ptrs)
{
    for (const void *q : ptrs)
        if (reinterpret_cast<uintptr_t>(q) % 16 != 0) return false;
    return true;
}

int check(const s2_grid_t *g, int batch, int C, int heads, const void *ws, size_t ws_bytes)
{
    if (!g) return s2_fail(S2_ERR_INVALID_ARG, "grid is NULL");
    if (batch < 1 || heads < 1 || C < 1 || C % heads != 0) return s2_fail(S2_ERR_INVALID_ARG, "channels must be a positive multiple of heads");
    if (!g->on_device) return s2_fail(S2_ERR_DEVICE, "grid handle has no device tables (no HIP device at init)");
    if (g->nlat_in != g->nlat_out || g->nlon_in != g->nlon_out)
        return s2_fail(S2_ERR_UNSUPPORTED, "the attention sub-block is self-attention: input and output grid must be equal");
    if (C % 16 != 0 || (size_t(g->nlat_in) * g->nlon_in) % 16 != 0)
        return s2_fail(S2_ERR_UNSUPPORTED, "channels and the number of grid points must be multiples of 16");
    if (C / heads > 128) return s2_fail(S2_ERR_UNSUPPORTED, "head dimensions above 128 are not supported");
    if (!ws || reinterpret_cast<uintptr_t>(ws) % 256 != 0 || ws_bytes < layout(g, batch, C, heads).total * sizeof(float))
        return s2_fail(S2_ERR_WORKSPACE, "workspace missing, not 256-byte aligned or smaller than s2_mha_workspace_bytes()");
    return S2_OK;
}

// out[c] = sum over batch and grid points of u (times xhat if x is given).  With scratch for the pieces (`part`,
// part_floats floats) and rows that are multiples of 16 bytes the sum is cut into about 2048 workgroups.
void channel_sum(int batch, int C, int N, const float *u, const float *x, const float *mean, const float *rstd, float *out,
                 float *part, size_t part_floats, hipStream_t st)
{
    const int seg = std::min(16, std::max(1, (2048 + C * batch - 1) / (C * batch)));
    const size_t pieces = size_t(batch) * seg;
    if (N % 4 != 0 || !part || pieces * C > part_floats || pieces > 65535) {
        hipLaunchKernelGGL(mha_channel_sum, dim3(C), dim3(256), 0, st, batch, C, N, u, x, mean, rstd, out);
        return;
    }
    hipLaunchKernelGGL(mha_channel_sum_pieces, dim3(C, unsigned(pieces)), dim3(256), 0, st, C, N, seg, u, x, mean, rstd, part);
    hipLaunchKernelGGL(mha_sum_partials, dim3((C + 63) / 64), dim3(256), 0, st, C, int(pieces), part, out);
}

void gemm(bool trans, int M, int N, int K, int batch, const float *W, const float *X, const float *bias, const float *R,
          float *C, bool accumulate, hipStream_t st)
{
    if (wres_ok(M, K)) {
        const int pitch = wres_pitch(M), tpb = (N + 31) / 32, ntiles = tpb * batch;
        const size_t lds = size_t(K) * pitch * sizeof(float);
        const int nwg = std::min((ntiles + 7) / 8, num_compute_units());
#define S2_WRES(T, MT)                                                                                                 \
    hipLaunchKernelGGL((mha_gemm_wres<T, MT>), dim3(nwg), dim3(512), lds, st, M, N, K, pitch, tpb, ntiles, W, X, bias, \
                       R, C, int(accumulate))
        switch (M / 32 + (trans ? 4 : 0)) {
        case 1: S2_WRES(false, 1); break;
        case 2: S2_WRES(false, 2); break;
        case 3: S2_WRES(false, 3); break;
        case 4: S2_WRES(false, 4); break;
        case 5: S2_WRES(true, 1); break;
        case 6: S2_WRES(true, 2); break;
        case 7: S2_WRES(true, 3); break;
        default: S2_WRES(true, 4); break;
        }
#undef S2_WRES
        return;
    }
    const dim3 grid((N + kTN - 1) / kTN, (M + kTM - 1) / kTM, batch);
    if (trans)
        hipLaunchKernelGGL(mha_gemm<true>, grid, dim3(256), 0, st, M, N, K, W, X, bias, R, C, int(accumulate));
    else
        hipLaunchKernelGGL(mha_gemm<false>, grid, dim3(256), 0, st, M, N, K, W, X, bias, R, C, int(accumulate));
}

void wgrad(int M, int K, int N, int batch, const float *dY, const float *X, float *part, float *dW, hipStream_t st)
{
    const int nsplit = wgrad_splits(M, K);
    hipLaunchKernelGGL(mha_wgrad_partial, dim3((K + kTN - 1) / kTN, (M + kTM - 1) / kTM, nsplit), dim3(256), 0, st, M, K, N,
                       batch, nsplit, dY, X, part);
    hipLaunchKernelGGL(mha_sum_partials, dim3((M * K + 63) / 64), dim3(256), 0, st, M * K, nsplit, part, dW);
}

}  // namespace

// once per device (from s2_grid_init): the weight-resident channel products keep up to 160 KB of LDS
int s2_mha_configure()
{
    auto raise = [](auto kern) {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   160 * 1024) == hipSuccess;
    };
    return raise(mha_gemm_wres<false, 1>) && raise(mha_gemm_wres<false, 2>) && raise(mha_gemm_wres<false, 3>) &&
                   raise(mha_gemm_wres<false, 4>) && raise(mha_gemm_wres<true, 1>) && raise(mha_gemm_wres<true, 2>) &&
                   raise(mha_gemm_wres<true, 3>) && raise(mha_gemm_wres<true, 4>)
               ? 0
               : -1;
}

void s2_gemm_f32(bool trans_a, int M, int N, int K, int batch, const float *W, const float *X, const float *bias,
                 const float *R, float *C, bool accumulate, hipStream_t st)
{
    gemm(trans_a, M, N, K, batch, W, X, bias, R, C, accumulate, st);
}
size_t s2_wgrad_part_floats(int M, int K) { return size_t(wgrad_splits(M, K)) * M * K; }
void s2_wgrad_f32(int M, int K, int N, int batch, const float *dY, const float *X, float *part, float *dW, hipStream_t st)
{
    wgrad(M, K, N, batch, dY, X, part, dW, st);
}
void s2_channel_sum_f32(int batch, int C, int N, const float *u, float *out, float *part, size_t part_floats,
                        hipStream_t st)
{
    channel_sum(batch, C, N, u, nullptr, nullptr, nullptr, out, part, part_floats, st);
}

extern "C" size_t s2_mha_workspace_bytes(const s2_grid_t *g, int batch, int channels, int heads)
{
    if (!g || batch < 1 || channels < 1 || heads < 1) return 0;
    return layout(g, batch, channels, heads).total * sizeof(float);
}

extern "C" int s2_mha_fwd(const s2_grid_t *g, int batch, int channels, int heads, float eps, const float *x,
                          const s2_mha_params_t *p, float *y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check(g, batch, channels, heads, workspace, workspace_bytes);
    if (rc) return rc;
    if (!x || !p || !y || !p->Wq || !p->Wk || !p->Wv || !p->Wo) return s2_fail(S2_ERR_INVALID_ARG, "NULL tensor or weight pointer");
    if (!aligned16({x, y, p->pos, p->Wq, p->Wk, p->Wv, p->Wo}))
        return s2_fail(S2_ERR_INVALID_ARG, "x, y, pos and the weight matrices must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int C = channels, N = g->nlat_in * g->nlon_in, d = C / heads;
    float *ws = static_cast<float *>(workspace);
    const Layout L = layout(g, batch, C, heads);
    {
        S2TraceScope tr("mha_instnorm_fwd", 0.0, st);
        hipLaunchKernelGGL(mha_instnorm_fwd, dim3(batch * C), dim3(256), 0, st, C, N, eps, x, p->gamma, p->beta, p->pos,
                           ws + L.mean, ws + L.rstd, ws + L.xn);
    }
    {
        S2TraceScope tr("mha_gemm qkv", 0.0, st);
        gemm(false, C, N, C, batch, p->Wq, ws + L.xn, p->bq, nullptr, ws + L.q, false, st);
        gemm(false, C, N, C, batch, p->Wk, ws + L.xn, p->bk, nullptr, ws + L.k, false, st);
        gemm(false, C, N, C, batch, p->Wv, ws + L.xn, p->bv, nullptr, ws + L.v, false, st);
    }
    rc = s2_nattn_fwd(g, batch, heads, d, d, S2_F32, 1.f / sqrtf(float(d)), ws + L.q, ws + L.k, ws + L.v, ws + L.a,
                      ws + L.lse, hip_stream);
    if (rc) return rc;
    {
        S2TraceScope tr("mha_gemm out", 0.0, st);
        gemm(false, C, N, C, batch, p->Wo, ws + L.a, p->bo, x, y, false, st);
    }
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}

extern "C" int s2_mha_bwd(const s2_grid_t *g, int batch, int channels, int heads, float eps, const float *x,
                          const s2_mha_params_t *p, const float *dy, float *dx, const s2_mha_grads_t *grads,
                          void *workspace, size_t workspace_bytes, void *hip_stream)
{
    (void)eps;      // the moments saved by the forward pass are reused
    int rc = check(g, batch, channels, heads, workspace, workspace_bytes);
    if (rc) return rc;
    if (!x || !p || !dy || !dx || !grads || !p->Wq || !p->Wk || !p->Wv || !p->Wo)
        return s2_fail(S2_ERR_INVALID_ARG, "NULL tensor or weight pointer");
    if (!aligned16({x, dy, dx, p->pos, p->Wq, p->Wk, p->Wv, p->Wo}))
        return s2_fail(S2_ERR_INVALID_ARG, "x, dy, dx, pos and the weight matrices must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int C = channels, N = g->nlat_in * g->nlon_in, d = C / heads;
    float *ws = static_cast<float *>(workspace);
    const Layout L = layout(g, batch, C, heads);
    float *gWq = grads->Wq, *gWk = grads->Wk, *gWv = grads->Wv, *gWo = grads->Wo;
    auto chan = [&](const float *u, bool with_xhat, float *dst) {
        if (dst)
            channel_sum(batch, C, N, u, with_xhat ? x : nullptr, ws + L.mean, ws + L.rstd, dst, ws + L.part,
                        L.total - L.part, st);
    };
    {
        // y = x + Wo a + bo
        S2TraceScope tr("mha_bwd out-projection", 0.0, st);
        if (gWo) wgrad(C, C, N, batch, dy, ws + L.a, ws + L.part, gWo, st);
        chan(dy, false, grads->bo);
        gemm(true, C, N, C, batch, p->Wo, dy, nullptr, nullptr, ws + L.da, false, st);
    }
    rc = s2_nattn_bwd(g, batch, heads, d, d, S2_F32, 1.f / sqrtf(float(d)), ws + L.q, ws + L.k, ws + L.v, ws + L.a,
                      ws + L.lse, ws + L.da, ws + L.dq, ws + L.dk, ws + L.dv, ws + L.D,
                      s2_nattn_bwd_workspace_bytes(g, batch, heads, d, d, S2_F32), hip_stream);
    if (rc) return rc;
    {
        S2TraceScope tr("mha_bwd qkv-projections", 0.0, st);
        const float *dts[3] = {ws + L.dq, ws + L.dk, ws + L.dv};
        const float *Ws[3] = {p->Wq, p->Wk, p->Wv};
        float *gWs[3] = {gWq, gWk, gWv};
        float *gbs[3] = {grads->bq, grads->bk, grads->bv};
        for (int i = 0; i < 3; ++i) {
            if (gWs[i]) wgrad(C, C, N, batch, dts[i], ws + L.xn, ws + L.part, gWs[i], st);
            chan(dts[i], false, gbs[i]);
            gemm(true, C, N, C, batch, Ws[i], dts[i], nullptr, nullptr, ws + L.dxn, i > 0, st);
        }
    }
    {
        S2TraceScope tr("mha_bwd instnorm", 0.0, st);
        if (grads->pos)
            hipLaunchKernelGGL(mha_batch_sum, dim3(unsigned((size_t(C) * N + 255) / 256)), dim3(256), 0, st, batch,
                               size_t(C) * N, ws + L.dxn, grads->pos);
        chan(ws + L.dxn, true, grads->gamma);
        chan(ws + L.dxn, false, grads->beta);
        hipLaunchKernelGGL(mha_instnorm_bwd, dim3(batch * C), dim3(256), 0, st, C, N, x, p->gamma, ws + L.mean, ws + L.rstd,
                           ws + L.dxn, dy, dx);
    }
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}
