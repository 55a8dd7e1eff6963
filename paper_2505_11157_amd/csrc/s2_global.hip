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

// D[bh][i] = dout_i . out_i
__global__ void __launch_bounds__(256)
rowdot(const bf16raw *__restrict__ a, const bf16raw *__restrict__ b, float *__restrict__ D, size_t ntok)
{
    const size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    if (i >= ntok) return;
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < kD; c += 8) {
        const bf16x8 x = ld8(a + i * kD + c), y = ld8(b + i * kD + c);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc = fmaf(float(x[j]), float(y[j]), acc);
    }
    D[i] = acc;
}

// Forward.  One wavefront = 32 queries; bias = log2(omega) per token, -inf on the padding.
__global__ void __launch_bounds__(256)
global_fwd(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ vt,
           const float *__restrict__ bias, bf16raw *__restrict__ out, float *__restrict__ lse, int N, int Npad,
           float c2)
{
    const int bh = blockIdx.y;
    const int q0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 32;
    if (q0 >= N) return;
    const int lane = threadIdx.x & 63, col = lane & 31, hl = lane >> 5;
    const int query = min(q0 + col, N - 1);
    const int prow = perm_row(col);
    bf16x8 qop[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qop[ks] = ld8(q + (size_t(bh) * N + query) * kD + 16 * ks + 8 * hl);
    f32x16 o0 = {0}, o1 = {0};
    float m = -INFINITY, l = 0.f;
    const bf16raw *kb = k + size_t(bh) * N * kD + 8 * hl;
    const bf16raw *vb0 = vt + (size_t(bh) * kD + col) * Npad + 16 * hl;
    const bf16raw *vb1 = vb0 + size_t(32) * Npad;
    for (int key0 = 0; key0 < Npad; key0 += 32) {
        const int key = min(key0 + prow, N - 1);
        f32x16 s = {0};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) s = mfma(ld8(kb + size_t(key) * kD + 16 * ks), qop[ks], s);
        float p[16];
        float mloc = -INFINITY;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 b = *reinterpret_cast<const float4 *>(bias + key0 + 16 * hl + 4 * g);
            p[4 * g + 0] = fmaf(s[4 * g + 0], c2, b.x);
            p[4 * g + 1] = fmaf(s[4 * g + 1], c2, b.y);
            p[4 * g + 2] = fmaf(s[4 * g + 2], c2, b.z);
            p[4 * g + 3] = fmaf(s[4 * g + 3], c2, b.w);
#pragma unroll
            for (int t = 0; t < 4; ++t) mloc = fmaxf(mloc, p[4 * g + t]);
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        // move the reference maximum only when a logit exceeds it by more than 2^8
        if (__any(mloc > m + 8.f)) {
            const float m_new = mloc > m + 8.f ? mloc : m;
            const float corr = __builtin_amdgcn_exp2f(m - m_new);
            m = m_new;
            l *= corr;
#pragma unroll
            for (int i = 0; i < 16; ++i) { o0[i] *= corr; o1[i] *= corr; }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            p[i] = __builtin_amdgcn_exp2f(p[i] - m);
            l += p[i];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bf16x8 pb = pack8(p + 8 * j);
            o0 = mfma(ld8(vb0 + key0 + 8 * j), pb, o0);
            o1 = mfma(ld8(vb1 + key0 + 8 * j), pb, o1);
        }
    }
    l += __shfl_xor(l, 32);
    if (q0 + col >= N) return;
    const float inv = 1.f / l;
    bf16raw *ob = out + (size_t(bh) * N + query) * kD + 4 * hl;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        bf16x4 a, b;
#pragma unroll
        for (int t = 0; t < 4; ++t) { a[t] = (__bf16)(o0[4 * g + t] * inv); b[t] = (__bf16)(o1[4 * g + t] * inv); }
        *reinterpret_cast<bf16x4 *>(ob + 8 * g) = a;
        *reinterpret_cast<bf16x4 *>(ob + 32 + 8 * g) = b;
    }
    if (hl == 0) lse[size_t(bh) * N + query] = (m + log2f(l)) * 0.6931471805599453f;
}

// Backward, key side: one wavefront = 32 keys, streaming 32-query tiles.
//   S = Q K^T and dP = dout V^T land with lane = key, registers = 16 queries;
//   dV^T += dout^T P,  dK^T += Q^T dS  with the transposed operands from the workspace.
__global__ void __launch_bounds__(256)
global_bwd_dkdv(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ v,
                const bf16raw *__restrict__ go, const bf16raw *__restrict__ qt, const bf16raw *__restrict__ got,
                const float *__restrict__ bias, const float *__restrict__ lse, const float *__restrict__ Dv,
                bf16raw *__restrict__ dk, bf16raw *__restrict__ dv, int N, int Npad, float c2, float scale)
{
    const int bh = blockIdx.y;
    const int k0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 32;
    if (k0 >= N) return;
    const int lane = threadIdx.x & 63, col = lane & 31, hl = lane >> 5;
    const int key = min(k0 + col, N - 1);
    const int prow = perm_row(col);
    bf16x8 kop[4], vop[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        kop[ks] = ld8(k + (size_t(bh) * N + key) * kD + 16 * ks + 8 * hl);
        vop[ks] = ld8(v + (size_t(bh) * N + key) * kD + 16 * ks + 8 * hl);
    }
    const float bk = bias[k0 + col];
    f32x16 dk0 = {0}, dk1 = {0}, dv0 = {0}, dv1 = {0};
    const bf16raw *qb = q + size_t(bh) * N * kD + 8 * hl, *gb = go + size_t(bh) * N * kD + 8 * hl;
    const bf16raw *qt0 = qt + (size_t(bh) * kD + col) * Npad + 16 * hl, *qt1 = qt0 + size_t(32) * Npad;
    const bf16raw *gt0 = got + (size_t(bh) * kD + col) * Npad + 16 * hl, *gt1 = gt0 + size_t(32) * Npad;
    const float *lb = lse + size_t(bh) * N, *Db = Dv + size_t(bh) * N;
    for (int q0 = 0; q0 < Npad; q0 += 32) {
        const int qrow = min(q0 + prow, N - 1);
        f32x16 s = {0}, dp = {0};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            s = mfma(ld8(qb + size_t(qrow) * kD + 16 * ks), kop[ks], s);
            dp = mfma(ld8(gb + size_t(qrow) * kD + 16 * ks), vop[ks], dp);
        }
        float p[16], ds[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int qi = q0 + 16 * hl + i;
            const int qc = min(qi, N - 1);
            const float pi = qi < N ? __builtin_amdgcn_exp2f(fmaf(s[i], c2, bk) - lb[qc] * kLog2e) : 0.f;
            p[i] = pi;
            ds[i] = pi * (dp[i] - Db[qc]);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bf16x8 pb = pack8(p + 8 * j), sb = pack8(ds + 8 * j);
            dv0 = mfma(ld8(gt0 + q0 + 8 * j), pb, dv0);
            dv1 = mfma(ld8(gt1 + q0 + 8 * j), pb, dv1);
            dk0 = mfma(ld8(qt0 + q0 + 8 * j), sb, dk0);
            dk1 = mfma(ld8(qt1 + q0 + 8 * j), sb, dk1);
        }
    }
    if (k0 + col >= N) return;
    bf16raw *dkb = dk + (size_t(bh) * N + key) * kD + 4 * hl, *dvb = dv + (size_t(bh) * N + key) * kD + 4 * hl;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        bf16x4 a, b, c, d;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            a[t] = (__bf16)(dk0[4 * g + t] * scale); b[t] = (__bf16)(dk1[4 * g + t] * scale);
            c[t] = (__bf16)dv0[4 * g + t]; d[t] = (__bf16)dv1[4 * g + t];
        }
        *reinterpret_cast<bf16x4 *>(dkb + 8 * g) = a;
        *reinterpret_cast<bf16x4 *>(dkb + 32 + 8 * g) = b;
        *reinterpret_cast<bf16x4 *>(dvb + 8 * g) = c;
        *reinterpret_cast<bf16x4 *>(dvb + 32 + 8 * g) = d;
    }
}

// Backward, query side: one wavefront = 32 queries, streaming 32-key tiles.
//   S^T = K Q^T and dP^T = V dout^T land with lane = query, registers = 16 keys;
//   dQ^T += K^T dS^T with K^T from the workspace.
__global__ void __launch_bounds__(256)
global_bwd_dq(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ v,
              const bf16raw *__restrict__ go, const bf16raw *__restrict__ kt, const float *__restrict__ bias,
              const float *__restrict__ lse, const float *__restrict__ Dv, bf16raw *__restrict__ dq, int N, int Npad,
              float c2, float scale)
{
    const int bh = blockIdx.y;
    const int q0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 32;
    if (q0 >= N) return;
    const int lane = threadIdx.x & 63, col = lane & 31, hl = lane >> 5;
    const int query = min(q0 + col, N - 1);
    const int prow = perm_row(col);
    bf16x8 qop[4], gop[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        qop[ks] = ld8(q + (size_t(bh) * N + query) * kD + 16 * ks + 8 * hl);
        gop[ks] = ld8(go + (size_t(bh) * N + query) * kD + 16 * ks + 8 * hl);
    }
    const float lse2 = lse[size_t(bh) * N + query] * kLog2e, Dq = Dv[size_t(bh) * N + query];
    f32x16 dq0 = {0}, dq1 = {0};
    const bf16raw *kb = k + size_t(bh) * N * kD + 8 * hl, *vb = v + size_t(bh) * N * kD + 8 * hl;
    const bf16raw *kt0 = kt + (size_t(bh) * kD + col) * Npad + 16 * hl, *kt1 = kt0 + size_t(32) * Npad;
    for (int key0 = 0; key0 < Npad; key0 += 32) {
        const int key = min(key0 + prow, N - 1);
        f32x16 s = {0}, dp = {0};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            s = mfma(ld8(kb + size_t(key) * kD + 16 * ks), qop[ks], s);
            dp = mfma(ld8(vb + size_t(key) * kD + 16 * ks), gop[ks], dp);
        }
        float ds[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 b = *reinterpret_cast<const float4 *>(bias + key0 + 16 * hl + 4 * g);
            const float bb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int i = 4 * g + t;
                ds[i] = __builtin_amdgcn_exp2f(fmaf(s[i], c2, bb[t]) - lse2) * (dp[i] - Dq);
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bf16x8 sb = pack8(ds + 8 * j);
            dq0 = mfma(ld8(kt0 + key0 + 8 * j), sb, dq0);
            dq1 = mfma(ld8(kt1 + key0 + 8 * j), sb, dq1);
        }
    }
    if (q0 + col >= N) return;
    bf16raw *dqb = dq + (size_t(bh) * N + query) * kD + 4 * hl;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        bf16x4 a, b;
#pragma unroll
        for (int t = 0; t < 4; ++t) { a[t] = (__bf16)(dq0[4 * g + t] * scale); b[t] = (__bf16)(dq1[4 * g + t] * scale); }
        *reinterpret_cast<bf16x4 *>(dqb + 8 * g) = a;
        *reinterpret_cast<bf16x4 *>(dqb + 32 + 8 * g) = b;
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
    const size_t ntok = size_t(batch) * heads * g->nlat_in * g->nlon_in;
    return 3 * transposed_bytes(g, batch * heads) + (ntok * sizeof(float) + 255) / 256 * 256;
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
    hipLaunchKernelGGL(global_fwd, dim3((N + 127) / 128, nbh), dim3(256), 0, st, static_cast<const bf16raw *>(q),
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
    const size_t tb = transposed_bytes(g, nbh), ntok = size_t(nbh) * N;
    char *ws = static_cast<char *>(workspace);
    bf16raw *qt = reinterpret_cast<bf16raw *>(ws), *kt = reinterpret_cast<bf16raw *>(ws + tb),
            *got = reinterpret_cast<bf16raw *>(ws + 2 * tb);
    float *Dv = reinterpret_cast<float *>(ws + 3 * tb);
    launch_transpose(q, qt, nbh, N, Npad, st);
    launch_transpose(k, kt, nbh, N, Npad, st);
    launch_transpose(dout, got, nbh, N, Npad, st);
    hipLaunchKernelGGL(rowdot, dim3((unsigned)((ntok + 255) / 256)), dim3(256), 0, st,
                       static_cast<const bf16raw *>(dout), static_cast<const bf16raw *>(out), Dv, ntok);
    const float c2 = scale * kLog2e;
    hipLaunchKernelGGL(global_bwd_dkdv, dim3((N + 127) / 128, nbh), dim3(256), 0, st, static_cast<const bf16raw *>(q),
                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(v),
                       static_cast<const bf16raw *>(dout), qt, got, g->dev_bias_tok, lse, Dv,
                       static_cast<bf16raw *>(dk), static_cast<bf16raw *>(dv), N, Npad, c2, scale);
    hipLaunchKernelGGL(global_bwd_dq, dim3((N + 127) / 128, nbh), dim3(256), 0, st, static_cast<const bf16raw *>(q),
                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(v),
                       static_cast<const bf16raw *>(dout), kt, g->dev_bias_tok, lse, Dv, static_cast<bf16raw *>(dq), N,
                       Npad, c2, scale);
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}
