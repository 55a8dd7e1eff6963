// Global quadrature-weighted attention on gfx950: bf16 MFMA (32x32x16), fp32
// softmax and accumulation, flash-style streaming over key tiles (App. B.1
// first equation; App. B.2: the quadrature weight is an additive column bias
// ln omega_j on the logits).
//
// Orientation.  Scores are produced TRANSPOSED, S^T = K Q^T, so that in the
// MFMA result layout a lane owns one query column and 16 keys.  The softmax
// over keys is then a per-lane loop plus one exchange between lanes l and l^32,
// and the exponentials can be fed straight back as the B operand of the next
// MFMA (O^T += V^T P^T) without moving data between lanes.  Row r of the K
// tile is mapped to key 16*((r>>2)&1) + 4*(r>>3) + (r&3): with that
// permutation the 16 keys a lane holds are contiguous, so bias, V^T and the
// transposed operands of the backward pass are read with 16-byte loads.
//
// The MFMA "A" operand wants its contraction index contiguous in memory.  V
// (forward) and Q, K, dout (backward) are contracted over tokens, so they are
// transposed once per call into the caller's workspace ([b,h][64][Npad] bf16,
// zero padded to a multiple of 32 tokens).
//
// Backward (App. B.4 with every token in every neighborhood): D_i = dout_i.out_i,
// p_ij = exp(s_ij + ln omega_j - lse_i), dS_ij = p_ij (dout_i.v_j - D_i);
// one kernel owns 32 keys and streams query tiles (dk, dv), one owns 32
// queries and streams key tiles (dq): no atomics.
#include "s2_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef unsigned short bf16raw;

constexpr int kD = 64;            // head dimension of the MFMA path
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ bf16x8 ld8(const bf16raw *p)
{
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(p));
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 pack8(const float *x)
{
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (__bf16)x[i];
    return r;
}

// key (or query) index of tile row r under the permutation described above
__device__ __forceinline__ int perm_row(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }

// in [bh][N][64] -> out [bh][64][Npad], zero for tokens >= N
__global__ void __launch_bounds__(256)
transpose_tokens(const bf16raw *__restrict__ in, bf16raw *__restrict__ out, int N, int Npad)
{
    __shared__ bf16raw tile[64][kD + 2];
    const int bh = blockIdx.y, t0 = blockIdx.x * 64;
    for (int i = threadIdx.x; i < 64 * kD; i += 256) {
        const int tok = i / kD, c = i % kD;
        tile[tok][c] = (t0 + tok < N) ? in[(size_t(bh) * N + t0 + tok) * kD + c] : bf16raw(0);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * kD; i += 256) {
        const int c = i / 64, tok = i % 64;
        if (t0 + tok < Npad) out[(size_t(bh) * kD + c) * Npad + t0 + tok] = tile[tok][c];
    }
}

// Per-token backward constants, padded to Npad tokens per slice so that the kernels can read them
// with 16-byte loads: L2[bh][i] = lse_i * log2(e) (+inf on the padding: p = exp2(-inf) = 0) and
// D[bh][i] = dout_i . out_i (0 on the padding).
__global__ void __launch_bounds__(256)
rowstats(const bf16raw *__restrict__ go, const bf16raw *__restrict__ o, const float *__restrict__ lse,
         float *__restrict__ L2, float *__restrict__ D, int N, int Npad)
{
    const int bh = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Npad) return;
    float acc = 0.f, l2 = INFINITY;
    if (i < N) {
        const size_t t = size_t(bh) * N + i;
#pragma unroll
        for (int c = 0; c < kD; c += 8) {
            const bf16x8 x = ld8(go + t * kD + c), y = ld8(o + t * kD + c);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc = fmaf(float(x[j]), float(y[j]), acc);
        }
        l2 = lse[t] * kLog2e;
    }
    L2[size_t(bh) * Npad + i] = l2;
    D[size_t(bh) * Npad + i] = acc;
}

// Forward.  One wavefront = 64 queries (two 32-query MFMA tiles sharing every K, V^T and bias
// operand they load); bias = log2(omega) per token, -inf on the padding.
__global__ void __launch_bounds__(256)
global_fwd(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ vt,
           const float *__restrict__ bias, bf16raw *__restrict__ out, float *__restrict__ lse, int N, int Npad,
           float c2)
{
    constexpr int NQ = 2;
    const int bh = blockIdx.y;
    const int q0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * (32 * NQ);
    if (q0 >= N) return;
    const int lane = threadIdx.x & 63, col = lane & 31, hl = lane >> 5;
    const int prow = perm_row(col);
    bf16x8 qop[NQ][4];
    f32x16 o0[NQ], o1[NQ];
    float m[NQ], l[NQ];
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        const int query = min(q0 + 32 * t + col, N - 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qop[t][ks] = ld8(q + (size_t(bh) * N + query) * kD + 16 * ks + 8 * hl);
#pragma unroll
        for (int i = 0; i < 16; ++i) { o0[t][i] = 0.f; o1[t][i] = 0.f; }
        m[t] = -INFINITY; l[t] = 0.f;
    }
    const bf16raw *kb = k + size_t(bh) * N * kD + 8 * hl;
    const bf16raw *vb0 = vt + (size_t(bh) * kD + col) * Npad + 16 * hl;
    const bf16raw *vb1 = vb0 + size_t(32) * Npad;
    for (int key0 = 0; key0 < Npad; key0 += 32) {
        const int key = min(key0 + prow, N - 1);
        bf16x8 kc[4], va[2], vb[2];
        float4 bc[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kc[ks] = ld8(kb + size_t(key) * kD + 16 * ks);
#pragma unroll
        for (int g = 0; g < 4; ++g) bc[g] = *reinterpret_cast<const float4 *>(bias + key0 + 16 * hl + 4 * g);
#pragma unroll
        for (int j = 0; j < 2; ++j) { va[j] = ld8(vb0 + key0 + 8 * j); vb[j] = ld8(vb1 + key0 + 8 * j); }
#pragma unroll
        for (int t = 0; t < NQ; ++t) {
            f32x16 s = {0};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) s = mfma(kc[ks], qop[t][ks], s);
            float p[16];
            float mloc = -INFINITY;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 b = bc[g];
                p[4 * g + 0] = fmaf(s[4 * g + 0], c2, b.x);
                p[4 * g + 1] = fmaf(s[4 * g + 1], c2, b.y);
                p[4 * g + 2] = fmaf(s[4 * g + 2], c2, b.z);
                p[4 * g + 3] = fmaf(s[4 * g + 3], c2, b.w);
#pragma unroll
                for (int u = 0; u < 4; ++u) mloc = fmaxf(mloc, p[4 * g + u]);
            }
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
            // move the reference maximum only when a logit exceeds it by more than 2^8
            if (__any(mloc > m[t] + 8.f)) {
                const float m_new = mloc > m[t] + 8.f ? mloc : m[t];
                const float corr = __builtin_amdgcn_exp2f(m[t] - m_new);
                m[t] = m_new;
                l[t] *= corr;
#pragma unroll
                for (int i = 0; i < 16; ++i) { o0[t][i] *= corr; o1[t][i] *= corr; }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                p[i] = __builtin_amdgcn_exp2f(p[i] - m[t]);
                l[t] += p[i];
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 pb = pack8(p + 8 * j);
                o0[t] = mfma(va[j], pb, o0[t]);
                o1[t] = mfma(vb[j], pb, o1[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        const float lt = l[t] + __shfl_xor(l[t], 32);
        const int qi = q0 + 32 * t + col;
        if (qi < N) {
            const float inv = 1.f / lt;
            bf16raw *ob = out + (size_t(bh) * N + qi) * kD + 4 * hl;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 a, b;
#pragma unroll
                for (int u = 0; u < 4; ++u) { a[u] = (__bf16)(o0[t][4 * g + u] * inv); b[u] = (__bf16)(o1[t][4 * g + u] * inv); }
                *reinterpret_cast<bf16x4 *>(ob + 8 * g) = a;
                *reinterpret_cast<bf16x4 *>(ob + 32 + 8 * g) = b;
            }
            if (hl == 0) lse[size_t(bh) * N + qi] = (m[t] + log2f(lt)) * 0.6931471805599453f;
        }
    }
}

// Backward, key side: one wavefront = 64 keys (two MFMA tiles sharing the streamed operands),
// streaming 32-query tiles.
//   S = Q K^T and dP = dout V^T land with lane = key, registers = 16 queries;
//   dV^T += dout^T P,  dK^T += Q^T dS  with the transposed operands from the workspace.
__global__ void __launch_bounds__(256)
global_bwd_dkdv(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ v,
                const bf16raw *__restrict__ go, const bf16raw *__restrict__ qt, const bf16raw *__restrict__ got,
                const float *__restrict__ bias, const float *__restrict__ L2, const float *__restrict__ Dv,
                bf16raw *__restrict__ dk, bf16raw *__restrict__ dv, int N, int Npad, float c2, float scale)
{
    constexpr int NK = 2;
    const int bh = blockIdx.y;
    const int k0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * (32 * NK);
    if (k0 >= N) return;
    const int lane = threadIdx.x & 63, col = lane & 31, hl = lane >> 5;
    const int prow = perm_row(col);
    bf16x8 kop[NK][4], vop[NK][4];
    float bk[NK];
    f32x16 dk0[NK], dk1[NK], dv0[NK], dv1[NK];
#pragma unroll
    for (int t = 0; t < NK; ++t) {
        const int key = min(k0 + 32 * t + col, N - 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            kop[t][ks] = ld8(k + (size_t(bh) * N + key) * kD + 16 * ks + 8 * hl);
            vop[t][ks] = ld8(v + (size_t(bh) * N + key) * kD + 16 * ks + 8 * hl);
        }
        bk[t] = bias[min(k0 + 32 * t + col, Npad - 1)];
#pragma unroll
        for (int i = 0; i < 16; ++i) { dk0[t][i] = 0.f; dk1[t][i] = 0.f; dv0[t][i] = 0.f; dv1[t][i] = 0.f; }
    }
    const bf16raw *qb = q + size_t(bh) * N * kD + 8 * hl, *gb = go + size_t(bh) * N * kD + 8 * hl;
    const bf16raw *qt0 = qt + (size_t(bh) * kD + col) * Npad + 16 * hl, *qt1 = qt0 + size_t(32) * Npad;
    const bf16raw *gt0 = got + (size_t(bh) * kD + col) * Npad + 16 * hl, *gt1 = gt0 + size_t(32) * Npad;
    const float *lb = L2 + size_t(bh) * Npad + 16 * hl, *Db = Dv + size_t(bh) * Npad + 16 * hl;
    for (int q0 = 0; q0 < Npad; q0 += 32) {
        const int qrow = min(q0 + prow, N - 1);
        bf16x8 qa[4], ga[4], qta[2], qtb[2], gta[2], gtb[2];
        float l2[16], dd[16];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qa[ks] = ld8(qb + size_t(qrow) * kD + 16 * ks);
            ga[ks] = ld8(gb + size_t(qrow) * kD + 16 * ks);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 x = *reinterpret_cast<const float4 *>(lb + q0 + 4 * g);
            const float4 y = *reinterpret_cast<const float4 *>(Db + q0 + 4 * g);
            l2[4 * g] = x.x; l2[4 * g + 1] = x.y; l2[4 * g + 2] = x.z; l2[4 * g + 3] = x.w;
            dd[4 * g] = y.x; dd[4 * g + 1] = y.y; dd[4 * g + 2] = y.z; dd[4 * g + 3] = y.w;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            qta[j] = ld8(qt0 + q0 + 8 * j); qtb[j] = ld8(qt1 + q0 + 8 * j);
            gta[j] = ld8(gt0 + q0 + 8 * j); gtb[j] = ld8(gt1 + q0 + 8 * j);
        }
#pragma unroll
        for (int t = 0; t < NK; ++t) {
            f32x16 s = {0}, dp = {0};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                s = mfma(qa[ks], kop[t][ks], s);
                dp = mfma(ga[ks], vop[t][ks], dp);
            }
            float p[16], ds[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                p[i] = __builtin_amdgcn_exp2f(fmaf(s[i], c2, bk[t]) - l2[i]);
                ds[i] = p[i] * (dp[i] - dd[i]);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 pb = pack8(p + 8 * j), sb = pack8(ds + 8 * j);
                dv0[t] = mfma(gta[j], pb, dv0[t]);
                dv1[t] = mfma(gtb[j], pb, dv1[t]);
                dk0[t] = mfma(qta[j], sb, dk0[t]);
                dk1[t] = mfma(qtb[j], sb, dk1[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < NK; ++t) {
        const int key = k0 + 32 * t + col;
        if (key >= N) continue;
        bf16raw *dkb = dk + (size_t(bh) * N + key) * kD + 4 * hl, *dvb = dv + (size_t(bh) * N + key) * kD + 4 * hl;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 a, b, c, d;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a[u] = (__bf16)(dk0[t][4 * g + u] * scale); b[u] = (__bf16)(dk1[t][4 * g + u] * scale);
                c[u] = (__bf16)dv0[t][4 * g + u]; d[u] = (__bf16)dv1[t][4 * g + u];
            }
            *reinterpret_cast<bf16x4 *>(dkb + 8 * g) = a;
            *reinterpret_cast<bf16x4 *>(dkb + 32 + 8 * g) = b;
            *reinterpret_cast<bf16x4 *>(dvb + 8 * g) = c;
            *reinterpret_cast<bf16x4 *>(dvb + 32 + 8 * g) = d;
        }
    }
}

// Backward, query side: one wavefront = 64 queries, streaming 32-key tiles.
//   S^T = K Q^T and dP^T = V dout^T land with lane = query, registers = 16 keys;
//   dQ^T += K^T dS^T with K^T from the workspace.
__global__ void __launch_bounds__(256)
global_bwd_dq(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ v,
              const bf16raw *__restrict__ go, const bf16raw *__restrict__ kt, const float *__restrict__ bias,
              const float *__restrict__ L2, const float *__restrict__ Dv, bf16raw *__restrict__ dq, int N, int Npad,
              float c2, float scale)
{
    constexpr int NQ = 2;
    const int bh = blockIdx.y;
    const int q0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * (32 * NQ);
    if (q0 >= N) return;
    const int lane = threadIdx.x & 63, col = lane & 31, hl = lane >> 5;
    const int prow = perm_row(col);
    bf16x8 qop[NQ][4], gop[NQ][4];
    float lse2[NQ], Dq[NQ];
    f32x16 dq0[NQ], dq1[NQ];
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        const int query = min(q0 + 32 * t + col, N - 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qop[t][ks] = ld8(q + (size_t(bh) * N + query) * kD + 16 * ks + 8 * hl);
            gop[t][ks] = ld8(go + (size_t(bh) * N + query) * kD + 16 * ks + 8 * hl);
        }
        lse2[t] = L2[size_t(bh) * Npad + query];
        Dq[t] = Dv[size_t(bh) * Npad + query];
#pragma unroll
        for (int i = 0; i < 16; ++i) { dq0[t][i] = 0.f; dq1[t][i] = 0.f; }
    }
    const bf16raw *kb = k + size_t(bh) * N * kD + 8 * hl, *vb = v + size_t(bh) * N * kD + 8 * hl;
    const bf16raw *kt0 = kt + (size_t(bh) * kD + col) * Npad + 16 * hl, *kt1 = kt0 + size_t(32) * Npad;
    for (int key0 = 0; key0 < Npad; key0 += 32) {
        const int key = min(key0 + prow, N - 1);
        bf16x8 ka[4], va[4], kta[2], ktb[2];
        float bb[16];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            ka[ks] = ld8(kb + size_t(key) * kD + 16 * ks);
            va[ks] = ld8(vb + size_t(key) * kD + 16 * ks);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 b = *reinterpret_cast<const float4 *>(bias + key0 + 16 * hl + 4 * g);
            bb[4 * g] = b.x; bb[4 * g + 1] = b.y; bb[4 * g + 2] = b.z; bb[4 * g + 3] = b.w;
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) { kta[j] = ld8(kt0 + key0 + 8 * j); ktb[j] = ld8(kt1 + key0 + 8 * j); }
#pragma unroll
        for (int t = 0; t < NQ; ++t) {
            f32x16 s = {0}, dp = {0};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                s = mfma(ka[ks], qop[t][ks], s);
                dp = mfma(va[ks], gop[t][ks], dp);
            }
            float ds[16];
#pragma unroll
            for (int i = 0; i < 16; ++i)
                ds[i] = __builtin_amdgcn_exp2f(fmaf(s[i], c2, bb[i]) - lse2[t]) * (dp[i] - Dq[t]);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 sb = pack8(ds + 8 * j);
                dq0[t] = mfma(kta[j], sb, dq0[t]);
                dq1[t] = mfma(ktb[j], sb, dq1[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < NQ; ++t) {
        const int qi = q0 + 32 * t + col;
        if (qi >= N) continue;
        bf16raw *dqb = dq + (size_t(bh) * N + qi) * kD + 4 * hl;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 a, b;
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = (__bf16)(dq0[t][4 * g + u] * scale); b[u] = (__bf16)(dq1[t][4 * g + u] * scale); }
            *reinterpret_cast<bf16x4 *>(dqb + 8 * g) = a;
            *reinterpret_cast<bf16x4 *>(dqb + 32 + 8 * g) = b;
        }
    }
}

int check_global(const s2_grid_t *g, int batch, int heads, int d, int dtype)
{
    if (!g) return s2_fail(S2_ERR_INVALID_ARG, "grid is NULL");
    if (batch < 1 || heads < 1 || d < 1) return s2_fail(S2_ERR_INVALID_ARG, "batch, heads, d must be >= 1");
    if (long(batch) * heads > 65535) return s2_fail(S2_ERR_INVALID_ARG, "batch*heads too large");
    if (g->nlat_in != g->nlat_out || g->nlon_in != g->nlon_out)
        return s2_fail(S2_ERR_INVALID_ARG, "global attention needs identical input and output grids");
    if (dtype != S2_BF16) return s2_fail(S2_ERR_UNSUPPORTED, "global attention supports S2_BF16 only");
    if (d != kD) return s2_fail(S2_ERR_UNSUPPORTED, "global attention supports head dimension 64 only");
    if (!g->on_device) return s2_fail(S2_ERR_DEVICE, "grid handle has no device tables (no HIP device at init)");
    return S2_OK;
}

size_t transposed_bytes(const s2_grid_t *g, int nbh) { return size_t(nbh) * kD * g->npad_tok * sizeof(bf16raw); }

void launch_transpose(const void *in, void *out, int nbh, int N, int Npad, hipStream_t st)
{
    hipLaunchKernelGGL(transpose_tokens, dim3((Npad + 63) / 64, nbh), dim3(256), 0, st,
                       static_cast<const bf16raw *>(in), static_cast<bf16raw *>(out), N, Npad);
}

}  // namespace

extern "C" size_t s2_attn_global_fwd_workspace_bytes(const s2_grid_t *g, int batch, int heads, int d, int dtype)
{
    (void)d; (void)dtype;
    if (!g || batch < 1 || heads < 1) return 0;
    return transposed_bytes(g, batch * heads);
}

extern "C" size_t s2_attn_global_bwd_workspace_bytes(const s2_grid_t *g, int batch, int heads, int d, int dtype)
{
    (void)d; (void)dtype;
    if (!g || batch < 1 || heads < 1) return 0;
    const size_t npad = size_t(batch) * heads * g->npad_tok;
    return 3 * transposed_bytes(g, batch * heads) + 2 * ((npad * sizeof(float) + 255) / 256 * 256);
}

extern "C" int s2_attn_global_fwd(const s2_grid_t *g, int batch, int heads, int d, int dtype, float scale,
                                  const void *q, const void *k, const void *v, void *out, float *lse,
                                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_global(g, batch, heads, d, dtype);
    if (rc) return rc;
    if (!q || !k || !v || !out || !lse) return s2_fail(S2_ERR_INVALID_ARG, "NULL tensor pointer");
    if (!workspace || workspace_bytes < s2_attn_global_fwd_workspace_bytes(g, batch, heads, d, dtype))
        return s2_fail(S2_ERR_WORKSPACE, "workspace missing or smaller than s2_attn_global_fwd_workspace_bytes()");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int nbh = batch * heads, N = g->nlat_in * g->nlon_in, Npad = g->npad_tok;
    launch_transpose(v, workspace, nbh, N, Npad, st);
    S2TraceScope tr("global_fwd", double(nbh) * N * N, st);
    hipLaunchKernelGGL(global_fwd, dim3((N + 255) / 256, nbh), dim3(256), 0, st, static_cast<const bf16raw *>(q),
                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(workspace), g->dev_bias_tok,
                       static_cast<bf16raw *>(out), lse, N, Npad, scale * kLog2e);
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}

extern "C" int s2_attn_global_bwd(const s2_grid_t *g, int batch, int heads, int d, int dtype, float scale,
                                  const void *q, const void *k, const void *v, const void *out, const float *lse,
                                  const void *dout, void *dq, void *dk, void *dv, void *workspace,
                                  size_t workspace_bytes, void *hip_stream)
{
    int rc = check_global(g, batch, heads, d, dtype);
    if (rc) return rc;
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv)
        return s2_fail(S2_ERR_INVALID_ARG, "NULL tensor pointer");
    if (!workspace || workspace_bytes < s2_attn_global_bwd_workspace_bytes(g, batch, heads, d, dtype))
        return s2_fail(S2_ERR_WORKSPACE, "workspace missing or smaller than s2_attn_global_bwd_workspace_bytes()");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int nbh = batch * heads, N = g->nlat_in * g->nlon_in, Npad = g->npad_tok;
    const size_t tb = transposed_bytes(g, nbh);
    const size_t sb = (size_t(nbh) * Npad * sizeof(float) + 255) / 256 * 256;
    char *ws = static_cast<char *>(workspace);
    bf16raw *qt = reinterpret_cast<bf16raw *>(ws), *kt = reinterpret_cast<bf16raw *>(ws + tb),
            *got = reinterpret_cast<bf16raw *>(ws + 2 * tb);
    float *L2 = reinterpret_cast<float *>(ws + 3 * tb), *Dv = reinterpret_cast<float *>(ws + 3 * tb + sb);
    launch_transpose(q, qt, nbh, N, Npad, st);
    launch_transpose(k, kt, nbh, N, Npad, st);
    launch_transpose(dout, got, nbh, N, Npad, st);
    hipLaunchKernelGGL(rowstats, dim3((Npad + 255) / 256, nbh), dim3(256), 0, st, static_cast<const bf16raw *>(dout),
                       static_cast<const bf16raw *>(out), lse, L2, Dv, N, Npad);
    const float c2 = scale * kLog2e;
    {
    S2TraceScope tr("global_bwd_dkdv", double(nbh) * N * N, st);
    hipLaunchKernelGGL(global_bwd_dkdv, dim3((N + 255) / 256, nbh), dim3(256), 0, st, static_cast<const bf16raw *>(q),
                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(v),
                       static_cast<const bf16raw *>(dout), qt, got, g->dev_bias_tok, L2, Dv,
                       static_cast<bf16raw *>(dk), static_cast<bf16raw *>(dv), N, Npad, c2, scale);
    }
    S2TraceScope tr("global_bwd_dq", double(nbh) * N * N, st);
    hipLaunchKernelGGL(global_bwd_dq, dim3((N + 255) / 256, nbh), dim3(256), 0, st, static_cast<const bf16raw *>(q),
                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(v),
                       static_cast<const bf16raw *>(dout), kt, g->dev_bias_tok, L2, Dv, static_cast<bf16raw *>(dq), N,
                       Npad, c2, scale);
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}
