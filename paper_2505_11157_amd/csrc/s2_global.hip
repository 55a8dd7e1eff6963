// Global quadrature-weighted attention on gfx950: bf16 MFMA (32x32x16), fp32
// softmax and accumulation, flash-style streaming over key tiles (App. B.1
// first equation; App. B.2 writes the quadrature weight as an additive column
// bias ln omega_j on the logits: here it is carried as the equivalent factor
// omega_j / max omega on the exponentials, folded into the transposed operands,
// so that a zero weight needs no special case and the running maximum follows
// the bare logits).
//
// Orientation.  Scores are produced TRANSPOSED, S^T = K Q^T, so that in the
// MFMA result layout a lane owns one query column and 16 keys.  The softmax
// over keys is then a per-lane loop (the two half-wavefronts of a query only
// talk when the running maximum has to move), and the exponentials are fed
// straight back as the B operand of the next MFMA (O^T += V^T P^T) without
// moving data between lanes.  Row r of the K tile is mapped to key
// 16*((r>>2)&1) + 4*(r>>3) + (r&3): with that permutation the 16 keys a lane
// holds are contiguous.
//
// The MFMA "A" operand wants its contraction index contiguous in memory.  V
// (forward) and Q, K, dout (backward) are contracted over tokens, so they are
// transposed once per call into the caller's workspace ([b,h][64][Npad] bf16,
// zero padded to a multiple of 64 tokens).  All streamed operands reach the
// wavefronts through LDS tiles that a workgroup copies once (see below).
//
// Backward (App. B.4 with every token in every neighborhood): D_i = dout_i.out_i,
// p_ij = omega_j exp(s_ij - lse_i), dS_ij = p_ij (dout_i.v_j - D_i);
// one kernel owns 32 keys per wavefront and streams query tiles (dk, dv), one
// owns 32 queries per wavefront and streams key tiles (dq): no atomics.
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

// Preparation pass.  One launch handles up to three operands (blockIdx.z): each is transposed from
// [bh][N][64] to [bh][64][Npad] (zero for tokens >= N), optionally with every token multiplied by its
// weight first (rounded to bf16 once, after the product).  The block that transposes `stat_go` (dout) also
// writes the per-token backward constants, padded to Npad tokens per slice:
// L2[bh][i] = (lse_i - ln max omega) * log2(e) (+inf on the padding: p = exp2(-inf) = 0) and
// D[bh][i] = -(dout_i . out_i) (0 on the padding): the backward kernels start the accumulation of dout.v
// from -D, so that the matrix core delivers dout_i.v_j - D_i directly.
// A block moves 64 tokens: four threads per token read 32 bytes each (coalesced rows), the tile is turned in
// LDS, and four threads per channel write 32 bytes each.
struct PrepOp {
    const bf16raw *in;
    bf16raw *out;
    const float *wtok;      // weights to multiply with, or null
};
struct PrepArgs {
    PrepOp op[3];
    int stat_op;            // index of the operand that is dout (-1: no statistics)
    const bf16raw *o;       // forward output
    const float *lse;
    float *L2, *D;
    float ln_wref;
};

__global__ void __launch_bounds__(256)
prepare_operands(PrepArgs a, int N, int Npad)
{
    constexpr int kP = 72;   // tile pitch in elements: rows start 16-byte aligned, 36 banks apart
    __shared__ __attribute__((aligned(16))) bf16raw tile[kD][kP];
    const PrepOp op = a.op[blockIdx.z];
    const int bh = blockIdx.y, t0 = blockIdx.x * 64;
    const int tid = threadIdx.x, tok = tid >> 2, part = tid & 3;
    const int token = t0 + tok;
    bf16x8 x[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int u = 0; u < 8; ++u) x[j][u] = (__bf16)0.f;
    if (token < N) {
        const bf16raw *src = op.in + (size_t(bh) * N + token) * kD + 16 * part;
        x[0] = ld8(src);
        x[1] = ld8(src + 8);
    }
    if (int(blockIdx.z) == a.stat_op) {
        float acc = 0.f;
        if (token < N) {
            const bf16raw *po = a.o + (size_t(bh) * N + token) * kD + 16 * part;
            const bf16x8 y0 = ld8(po), y1 = ld8(po + 8);
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = fmaf(float(x[0][u]), float(y0[u]), fmaf(float(x[1][u]), float(y1[u]), acc));
        }
        acc += __shfl_xor(acc, 1);
        acc += __shfl_xor(acc, 2);
        if (part == 0 && token < Npad) {
            a.L2[size_t(bh) * Npad + token] = token < N ? (a.lse[size_t(bh) * N + token] - a.ln_wref) * kLog2e : INFINITY;
            a.D[size_t(bh) * Npad + token] = -acc;
        }
    }
    if (op.wtok && token < N) {
        const float w = op.wtok[token];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int u = 0; u < 8; ++u) x[j][u] = (__bf16)(float(x[j][u]) * w);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const __bf16 e = x[j][u];      // (a bit_cast applied to the vector element itself reads element 0)
            tile[16 * part + 8 * j + u][tok] = __builtin_bit_cast(bf16raw, e);
        }
    __syncthreads();
    const int ch = tid >> 2;
    if (t0 + 16 * part < Npad) {       // Npad is a multiple of 64: a block's 64 tokens are all inside or all outside
        bf16raw *dst = op.out + (size_t(bh) * kD + ch) * Npad + t0 + 16 * part;
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(&tile[ch][16 * part]);
        *reinterpret_cast<uint4 *>(dst + 8) = *reinterpret_cast<const uint4 *>(&tile[ch][16 * part + 8]);
    }
}

// ---------------------------------------------------------------------------------------------
// Staging of streamed operands in LDS.  A workgroup of four wavefronts streams 64-token stages; every
// stage is copied from global memory once per workgroup (coalesced 16-byte pieces, no registers in
// between) into one of two LDS buffers while the other one is being used, and read from there by all
// four wavefronts as MFMA operands.  The two buffers are separate arrays and the stage loop is unrolled
// by two, so every access names its array: the compiler then knows that the reads of one buffer need
// not wait for the copies in flight into the other; the barrier at the end of a stage waits for them.  A staged tile is 64 rows of 128 bytes; the 16-byte
// piece c of row r sits at piece c ^ ((r >> 1) & 7), so that the 16 consecutive lanes a 16-byte LDS read
// serves together (16 consecutive rows, same logical piece) fall on 16 different bank groups, and so do
// the writes of a row.  Token-major tiles ("row tiles": 64 tokens x 64 channels) additionally have the
// rows of each 32-token half permuted so that lane `col` finds the token of MFMA row perm_row(col) in
// LDS row `col`.  Channel-major tiles ("column tiles": 64 channels x 64 tokens) come from the
// token-transposed copies in the workspace.
constexpr int kTileBytes = 64 * 128;

__device__ __forceinline__ int swz(int row, int piece) { return row * 128 + ((piece ^ ((row >> 1) & 7)) << 4); }

// LDS row of token t (0..63) of a stage: inverse of perm_row inside each 32-token half
__device__ __forceinline__ int lds_row_of_token(int t)
{
    const int k = t & 31;
    return (t & 32) | (k & 3) | (((k >> 4) & 1) << 2) | (((k >> 2) & 3) << 3);
}

// Copies go straight from global memory into LDS (global_load_lds_dwordx4: lane i of a wavefront
// deposits its 16 bytes at base + 16 i, i.e. one instruction fills eight consecutive rows), so the
// swizzle and the row permutation are applied on the source side: lane i fetches the piece that belongs
// at physical position i.  Wavefront w of the four copies rows 16 w .. 16 w + 15 of every tile.
typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// token-major tile: LDS row r holds token tok0 + (r & 32) + perm_row(r & 31), clamped to N - 1
__device__ __forceinline__ void copy_row_tile(const bf16raw *base, int tok0, int N, char *tile, int wave, int lane)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = 16 * wave + 8 * h + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        const int t = (r & 32) | perm_row(r & 31);
        const char *src = reinterpret_cast<const char *>(base + size_t(min(tok0 + t, N - 1)) * kD) + 16 * c;
        __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(tile + 2048 * wave + 1024 * h), 16, 0, 0);
    }
}
// channel-major tile from a transposed operand [64][Npad] (Npad a multiple of 64: always in bounds)
__device__ __forceinline__ void copy_col_tile(const bf16raw *base, int tok0, int Npad, char *tile, int wave, int lane)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = 16 * wave + 8 * h + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        const char *src = reinterpret_cast<const char *>(base + size_t(r) * Npad + tok0 + 8 * c);
        __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(tile + 2048 * wave + 1024 * h), 16, 0, 0);
    }
}
// 64 consecutive floats (one wavefront, lane = element)
__device__ __forceinline__ void copy_floats(const float *src, char *dst, int lane)
{
    __builtin_amdgcn_global_load_lds((gptr_t)(src + lane), (lptr_t)dst, 4, 0, 0);
}
__device__ __forceinline__ bf16x8 lds8(const char *p)
{
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(p));
}
// MFMA operand reads by lane (col, hl).  Row tile, 32-token half `half`, contraction step ks (channels
// 16 ks + 8 hl ..): piece 2 ks + hl of row 32 half + col.  Column tile, channel half `rt`, tokens
// 32 half + 16 hl + 8 j ..: piece 4 half + 2 hl + j of row 32 rt + col.  (32 does not touch the swizzle bits.)
__device__ __forceinline__ bf16x8 row_operand(const char *tile, int col, int hl, int half, int ks)
{
    return lds8(tile + half * 4096 + swz(col, 2 * ks + hl));
}
__device__ __forceinline__ bf16x8 col_operand(const char *tile, int col, int hl, int rt, int half, int j)
{
    return lds8(tile + rt * 4096 + swz(col, 4 * half + 2 * hl + j));
}

// Workgroups are numbered so that each of the eight XCDs (which take consecutive workgroup ids in turn)
// works through one contiguous piece of the (slice, block) list: the operands of the few slices an XCD
// has in flight then stay in its own L2.  Returns false for the padding ids at the end of the launch.
__device__ __forceinline__ bool xcd_unit(int nunits, int &unit)
{
    const int per = (nunits + 7) >> 3;
    unit = int(blockIdx.x & 7) * per + int(blockIdx.x >> 3);
    return unit < nunits && int(blockIdx.x >> 3) < per;
}

// Forward.  A workgroup owns 128 queries of one slice (one 32-query MFMA tile per wavefront) and streams
// the keys in stages of 64.  omega enters as a factor, not as a bias: V^T arrives premultiplied by
// w_j = omega_j / max omega (prepare_operands does that), the running sum is l_i = sum_j w_j 2^(x_ij - m_i)
// with x = log2(e) scale q.k, and the reference m_i follows the bare logits of the keys of positive weight (it moves
// only when a logit exceeds it by more than 2^8).  lse_i = ln 2 (m_i + log2 l_i) + ln max omega.
// UNIFORM_W: the longitude count is a multiple of 32, so a 32-key tile never straddles two latitudes.
template <bool UNIFORM_W>
__global__ void __launch_bounds__(256, 3)
global_fwd(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ vt,
           const float *__restrict__ wtok, bf16raw *__restrict__ out, float *__restrict__ lse, int N, int Npad,
           int nqb, int nunits, float c2, float ln_wref)
{
    constexpr int kStage = 2 * kTileBytes + 256;     // K row tile, V^T column tile, 64 weights
    __shared__ __attribute__((aligned(16))) char buf0[kStage];
    __shared__ __attribute__((aligned(16))) char buf1[kStage];
    int unit;
    if (!xcd_unit(nunits, unit)) return;
    const int bh = unit / nqb, qb = unit - bh * nqb;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, col = lane & 31, hl = lane >> 5;
    const int qi = qb * 128 + wave * 32 + col;
    bf16x8 qop[4];
    {
        const bf16raw *qp = q + (size_t(bh) * N + min(qi, N - 1)) * kD + 8 * hl;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) qop[ks] = ld8(qp + 16 * ks);
    }
    f32x16 o0 = {0}, o1 = {0};
    float m = 0.f, l = 0.f;
    const bf16raw *kb = k + size_t(bh) * N * kD;
    const bf16raw *vb = vt + size_t(bh) * kD * Npad;
    const int nst = Npad >> 6;
    auto request = [&](char *buf, int st) {
        copy_row_tile(kb, 64 * st, N, buf, wave, lane);
        copy_col_tile(vb, 64 * st, Npad, buf + kTileBytes, wave, lane);
        if (wave == 0) copy_floats(wtok + 64 * st, buf + 2 * kTileBytes, lane);
    };
    bool started = false;      // has a tile with a key of positive weight been seen (wavefront-uniform)
    auto stage = [&](const char *cur, char *nxt, int st) {
        if (st + 1 < nst) request(nxt, st + 1);
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            // Keys of weight zero (the pole row of the grid of App. A.1, the padding behind the last token) have no
            // term in the sums, so they must not enter the reference maximum either: a tile without a live key is
            // skipped, and in a mixed tile (longitude count not a multiple of 32) their logits are set to -inf.
            const float *wp = reinterpret_cast<const float *>(cur + 2 * kTileBytes) + 32 * kt + 16 * hl;
            float wk[16];
            bool live;
            if (UNIFORM_W) {
                live = __builtin_amdgcn_readfirstlane(__float_as_int(wp[0])) != 0;
            } else {
                bool any = false;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 w = *reinterpret_cast<const float4 *>(wp + 4 * g);
                    wk[4 * g + 0] = w.x; wk[4 * g + 1] = w.y; wk[4 * g + 2] = w.z; wk[4 * g + 3] = w.w;
                    any |= w.x > 0.f || w.y > 0.f || w.z > 0.f || w.w > 0.f;
                }
                live = __any(any);
            }
            if (!live) continue;
            f32x16 s = {0};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) s = mfma(row_operand(cur, col, hl, kt, ks), qop[ks], s);
            float x[16], e[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                x[i] = fmaf(s[i], c2, -m);
                if (!UNIFORM_W) x[i] = wk[i] > 0.f ? x[i] : -INFINITY;
            }
            // Fast path: exponentials relative to the current reference; a logit more than 2^8 above it shows in the
            // tile sum (all terms are positive), so the sum is the overflow test and no per-element maximum is taken.
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                e[i] = __builtin_amdgcn_exp2f(x[i]);
                psum += UNIFORM_W ? e[i] : e[i] * wk[i];
            }
            const bool first = !started;
            started = true;
            // the two half-wavefronts of a query exchange their maxima only when the reference has to move
            if (first || __any(!(psum <= 256.f))) {
                float mx = -INFINITY;
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, x[i]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float delta = first ? mx : (mx > 8.f ? mx : 0.f);
                const float corr = first ? 1.f : __builtin_amdgcn_exp2f(-delta);
                m += delta;
                l *= corr;
                psum = 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    o0[i] *= corr;
                    o1[i] *= corr;
                    e[i] = __builtin_amdgcn_exp2f(x[i] - delta);
                    psum += UNIFORM_W ? e[i] : e[i] * wk[i];
                }
            }
            l = UNIFORM_W ? fmaf(psum, wp[0], l) : l + psum;
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = e[i];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 pb = pack8(x + 8 * j);
                o0 = mfma(col_operand(cur + kTileBytes, col, hl, 0, kt, j), pb, o0);
                o1 = mfma(col_operand(cur + kTileBytes, col, hl, 1, kt, j), pb, o1);
            }
        }
        __syncthreads();   // everybody is done with `cur`, and the copies into `nxt` have landed
    };
    request(buf0, 0);
    __syncthreads();
    for (int st = 0; st < nst; st += 2) {
        stage(buf0, buf1, st);
        if (st + 1 < nst) stage(buf1, buf0, st + 1);
    }
    const float lt = l + __shfl_xor(l, 32);
    if (qi < N) {
        const float inv = 1.f / lt;
        bf16raw *ob = out + (size_t(bh) * N + qi) * kD + 4 * hl;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 a, b;
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = (__bf16)(o0[4 * g + u] * inv); b[u] = (__bf16)(o1[4 * g + u] * inv); }
            *reinterpret_cast<bf16x4 *>(ob + 8 * g) = a;
            *reinterpret_cast<bf16x4 *>(ob + 32 + 8 * g) = b;
        }
        if (hl == 0) lse[size_t(bh) * N + qi] = (m + log2f(lt)) * 0.6931471805599453f + ln_wref;
    }
}

// Backward (App. B.4 with every token in every neighborhood).  With w_j = omega_j / max omega and
// L_i = log2(e) (lse_i - ln max omega):  p_ij = w_j pt_ij,  pt_ij = 2^(log2(e) scale q_i.k_j - L_i),
// dS_ij = p_ij (dout_i.v_j - D_i).  The factor w_j never enters the inner loops: the key-side kernel
// multiplies its finished sums by w_j (the lane's own key), the query-side kernel contracts with
// K^T premultiplied by w_j (prepare_operands).
//
// Key side: a workgroup owns 128 keys (one 32-key tile per wavefront) and streams the queries in stages
// of 64: Q and dout token-major (for S = Q K^T and dP = dout V^T, which land with lane = key,
// registers = 16 queries), Q^T and dout^T channel-major (dV^T += dout^T Pt, dK^T += Q^T dSt), L and D.
__global__ void __launch_bounds__(256, 2)
global_bwd_dkdv(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ v,
                const bf16raw *__restrict__ go, const bf16raw *__restrict__ qt, const bf16raw *__restrict__ got,
                const float *__restrict__ wtok, const float *__restrict__ L2, const float *__restrict__ Dv,
                bf16raw *__restrict__ dk, bf16raw *__restrict__ dv, int N, int Npad, int nkb, int nunits, float c2,
                float scale)
{
    constexpr int kStage = 4 * kTileBytes + 512;     // Q, dout row tiles; Q^T, dout^T column tiles; L, D
    __shared__ __attribute__((aligned(16))) char buf0[kStage];
    __shared__ __attribute__((aligned(16))) char buf1[kStage];
    int unit;
    if (!xcd_unit(nunits, unit)) return;
    const int bh = unit / nkb, kb = unit - bh * nkb;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, col = lane & 31, hl = lane >> 5;
    const int ki = kb * 128 + wave * 32 + col;
    bf16x8 kop[4], vop[4];
    {
        const size_t row = (size_t(bh) * N + min(ki, N - 1)) * kD + 8 * hl;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) { kop[ks] = ld8(k + row + 16 * ks); vop[ks] = ld8(v + row + 16 * ks); }
    }
    f32x16 dk0 = {0}, dk1 = {0}, dv0 = {0}, dv1 = {0};
    const bf16raw *qb = q + size_t(bh) * N * kD, *gb = go + size_t(bh) * N * kD;
    const bf16raw *qtb = qt + size_t(bh) * kD * Npad, *gtb = got + size_t(bh) * kD * Npad;
    const float *Lb = L2 + size_t(bh) * Npad, *Db = Dv + size_t(bh) * Npad;
    const int nst = Npad >> 6;
    auto request = [&](char *buf, int st) {
        const int t0 = 64 * st;
        copy_row_tile(qb, t0, N, buf, wave, lane);
        copy_row_tile(gb, t0, N, buf + kTileBytes, wave, lane);
        copy_col_tile(qtb, t0, Npad, buf + 2 * kTileBytes, wave, lane);
        copy_col_tile(gtb, t0, Npad, buf + 3 * kTileBytes, wave, lane);
        if (wave == 0) copy_floats(Lb + t0, buf + 4 * kTileBytes, lane);
        if (wave == 1) copy_floats(Db + t0, buf + 4 * kTileBytes + 256, lane);
    };
    auto stage = [&](const char *cur, char *nxt, int st) {
        if (st + 1 < nst) request(nxt, st + 1);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float *Lp = reinterpret_cast<const float *>(cur + 4 * kTileBytes) + 32 * h + 16 * hl;
            // dP starts from -D_i (the 16 queries this lane's registers stand for)
            f32x16 s = {0}, dp;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 Dr = *reinterpret_cast<const float4 *>(Lp + 64 + 4 * g);
                dp[4 * g + 0] = Dr.x; dp[4 * g + 1] = Dr.y; dp[4 * g + 2] = Dr.z; dp[4 * g + 3] = Dr.w;
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                s = mfma(row_operand(cur, col, hl, h, ks), kop[ks], s);
                dp = mfma(row_operand(cur + kTileBytes, col, hl, h, ks), vop[ks], dp);
            }
            float p[16], ds[16];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 Lr = *reinterpret_cast<const float4 *>(Lp + 4 * g);
                p[4 * g + 0] = __builtin_amdgcn_exp2f(fmaf(s[4 * g + 0], c2, -Lr.x));
                p[4 * g + 1] = __builtin_amdgcn_exp2f(fmaf(s[4 * g + 1], c2, -Lr.y));
                p[4 * g + 2] = __builtin_amdgcn_exp2f(fmaf(s[4 * g + 2], c2, -Lr.z));
                p[4 * g + 3] = __builtin_amdgcn_exp2f(fmaf(s[4 * g + 3], c2, -Lr.w));
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) ds[i] = p[i] * dp[i];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 pb = pack8(p + 8 * j), sb = pack8(ds + 8 * j);
                dv0 = mfma(col_operand(cur + 3 * kTileBytes, col, hl, 0, h, j), pb, dv0);
                dv1 = mfma(col_operand(cur + 3 * kTileBytes, col, hl, 1, h, j), pb, dv1);
                dk0 = mfma(col_operand(cur + 2 * kTileBytes, col, hl, 0, h, j), sb, dk0);
                dk1 = mfma(col_operand(cur + 2 * kTileBytes, col, hl, 1, h, j), sb, dk1);
            }
        }
        __syncthreads();   // everybody is done with `cur`, and the copies into `nxt` have landed
    };
    request(buf0, 0);
    __syncthreads();
    for (int st = 0; st < nst; st += 2) {
        stage(buf0, buf1, st);
        if (st + 1 < nst) stage(buf1, buf0, st + 1);
    }
    if (ki < N) {
        const float wk = wtok[ki], wks = wk * scale;
        const bool live = wk > 0.f;
        bf16raw *dkb = dk + (size_t(bh) * N + ki) * kD + 4 * hl, *dvb = dv + (size_t(bh) * N + ki) * kD + 4 * hl;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 a, b, c, d;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                // a key of weight zero gets exactly zero (its unweighted sums may have overflowed: its logits are not
                // bounded by any logsumexp)
                a[u] = (__bf16)(live ? dk0[4 * g + u] * wks : 0.f); b[u] = (__bf16)(live ? dk1[4 * g + u] * wks : 0.f);
                c[u] = (__bf16)(live ? dv0[4 * g + u] * wk : 0.f); d[u] = (__bf16)(live ? dv1[4 * g + u] * wk : 0.f);
            }
            *reinterpret_cast<bf16x4 *>(dkb + 8 * g) = a;
            *reinterpret_cast<bf16x4 *>(dkb + 32 + 8 * g) = b;
            *reinterpret_cast<bf16x4 *>(dvb + 8 * g) = c;
            *reinterpret_cast<bf16x4 *>(dvb + 32 + 8 * g) = d;
        }
    }
}

// Query side: a workgroup owns 128 queries and streams the keys in stages of 64: K and V token-major
// (S^T = K Q^T and dP^T = V dout^T land with lane = query, registers = 16 keys) and w K^T channel-major
// (dQ^T += (w K)^T dSt^T).
// DEAD: some keys have weight zero (a pole row of weight zero, padding behind the last token).  Their logits are not
// bounded by the logsumexp, so 2^(x - L) may overflow and inf * (w k = 0) would poison dq: the exponent is capped at
// 100 there (a key of positive weight stays below log2(max omega / omega_j), a few tens at most), which keeps the
// factor finite and the product with the zero row exactly zero.
template <bool DEAD>
__global__ void __launch_bounds__(256, 3)
global_bwd_dq(const bf16raw *__restrict__ q, const bf16raw *__restrict__ k, const bf16raw *__restrict__ v,
              const bf16raw *__restrict__ go, const bf16raw *__restrict__ ktw, const float *__restrict__ L2,
              const float *__restrict__ Dv, bf16raw *__restrict__ dq, int N, int Npad, int nqb, int nunits, float c2,
              float scale)
{
    constexpr int kStage = 3 * kTileBytes;           // K, V row tiles; (w K)^T column tile
    __shared__ __attribute__((aligned(16))) char buf0[kStage];
    __shared__ __attribute__((aligned(16))) char buf1[kStage];
    int unit;
    if (!xcd_unit(nunits, unit)) return;
    const int bh = unit / nqb, qb = unit - bh * nqb;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, col = lane & 31, hl = lane >> 5;
    const int qi = qb * 128 + wave * 32 + col;
    bf16x8 qop[4], gop[4];
    {
        const size_t row = (size_t(bh) * N + min(qi, N - 1)) * kD + 8 * hl;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) { qop[ks] = ld8(q + row + 16 * ks); gop[ks] = ld8(go + row + 16 * ks); }
    }
    const float Lq = L2[size_t(bh) * Npad + min(qi, N - 1)], Dq = Dv[size_t(bh) * Npad + min(qi, N - 1)];
    f32x16 dq0 = {0}, dq1 = {0}, nd;     // nd: -D_q in every register, the start value of dout.v
#pragma unroll
    for (int i = 0; i < 16; ++i) nd[i] = Dq;
    const bf16raw *kb = k + size_t(bh) * N * kD, *vb = v + size_t(bh) * N * kD;
    const bf16raw *ktb = ktw + size_t(bh) * kD * Npad;
    const int nst = Npad >> 6;
    auto request = [&](char *buf, int st) {
        const int t0 = 64 * st;
        copy_row_tile(kb, t0, N, buf, wave, lane);
        copy_row_tile(vb, t0, N, buf + kTileBytes, wave, lane);
        copy_col_tile(ktb, t0, Npad, buf + 2 * kTileBytes, wave, lane);
    };
    auto stage = [&](const char *cur, char *nxt, int st) {
        if (st + 1 < nst) request(nxt, st + 1);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            f32x16 s = {0}, dp = nd;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                s = mfma(row_operand(cur, col, hl, h, ks), qop[ks], s);
                dp = mfma(row_operand(cur + kTileBytes, col, hl, h, ks), gop[ks], dp);
            }
            float ds[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float a = fmaf(s[i], c2, -Lq);
                ds[i] = __builtin_amdgcn_exp2f(DEAD ? fminf(a, 100.f) : a) * dp[i];
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x8 sb = pack8(ds + 8 * j);
                dq0 = mfma(col_operand(cur + 2 * kTileBytes, col, hl, 0, h, j), sb, dq0);
                dq1 = mfma(col_operand(cur + 2 * kTileBytes, col, hl, 1, h, j), sb, dq1);
            }
        }
        __syncthreads();   // everybody is done with `cur`, and the copies into `nxt` have landed
    };
    request(buf0, 0);
    __syncthreads();
    for (int st = 0; st < nst; st += 2) {
        stage(buf0, buf1, st);
        if (st + 1 < nst) stage(buf1, buf0, st + 1);
    }
    if (qi < N) {
        bf16raw *dqb = dq + (size_t(bh) * N + qi) * kD + 4 * hl;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            bf16x4 a, b;
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = (__bf16)(dq0[4 * g + u] * scale); b[u] = (__bf16)(dq1[4 * g + u] * scale); }
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
    // one workgroup per (slice, block of 128 tokens): the launch grid must fit 31 bits
    const long nunits = long(batch) * heads * ((long(g->nlat_in) * g->nlon_in + 127) / 128);
    if (nunits > (1l << 30)) return s2_fail(S2_ERR_INVALID_ARG, "batch*heads*tokens too large for one launch");
    return S2_OK;
}

// the kernels move 16-byte pieces (LDS-direct copies, vector loads and stores)
bool misaligned(const void *p, size_t a = 16) { return reinterpret_cast<uintptr_t>(p) % a != 0; }

size_t transposed_bytes(const s2_grid_t *g, int nbh) { return size_t(nbh) * kD * g->npad_tok * sizeof(bf16raw); }

void launch_prepare(const PrepArgs &a, int nops, int nbh, int N, int Npad, hipStream_t st)
{
    hipLaunchKernelGGL(prepare_operands, dim3(Npad / 64, nbh, nops), dim3(256), 0, st, a, N, Npad);
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
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out))
        return s2_fail(S2_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (!workspace || workspace_bytes < s2_attn_global_fwd_workspace_bytes(g, batch, heads, d, dtype))
        return s2_fail(S2_ERR_WORKSPACE, "workspace missing or smaller than s2_attn_global_fwd_workspace_bytes()");
    if (misaligned(workspace, 256)) return s2_fail(S2_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int nbh = batch * heads, N = g->nlat_in * g->nlon_in, Npad = g->npad_tok;
    PrepArgs pa{};
    pa.op[0] = {static_cast<const bf16raw *>(v), static_cast<bf16raw *>(workspace), g->dev_w_tok};
    pa.stat_op = -1;
    launch_prepare(pa, 1, nbh, N, Npad, st);
    S2TraceScope tr("global_fwd", double(nbh) * N * N, st);
    const int nqb = (N + 127) / 128, nunits = nbh * nqb;
    auto kern = g->nlon_in % 32 == 0 ? global_fwd<true> : global_fwd<false>;
    hipLaunchKernelGGL(kern, dim3(8 * ((nunits + 7) / 8)), dim3(256), 0, st, static_cast<const bf16raw *>(q),
                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(workspace), g->dev_w_tok,
                       static_cast<bf16raw *>(out), lse, N, Npad, nqb, nunits, scale * kLog2e, g->dt.ln_omega_ref);
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
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(dout) || misaligned(dq) ||
        misaligned(dk) || misaligned(dv))
        return s2_fail(S2_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (!workspace || workspace_bytes < s2_attn_global_bwd_workspace_bytes(g, batch, heads, d, dtype))
        return s2_fail(S2_ERR_WORKSPACE, "workspace missing or smaller than s2_attn_global_bwd_workspace_bytes()");
    if (misaligned(workspace, 256)) return s2_fail(S2_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int nbh = batch * heads, N = g->nlat_in * g->nlon_in, Npad = g->npad_tok;
    const size_t tb = transposed_bytes(g, nbh);
    const size_t sb = (size_t(nbh) * Npad * sizeof(float) + 255) / 256 * 256;
    char *ws = static_cast<char *>(workspace);
    bf16raw *qt = reinterpret_cast<bf16raw *>(ws), *kt = reinterpret_cast<bf16raw *>(ws + tb),
            *got = reinterpret_cast<bf16raw *>(ws + 2 * tb);
    float *L2 = reinterpret_cast<float *>(ws + 3 * tb), *Dv = reinterpret_cast<float *>(ws + 3 * tb + sb);
    PrepArgs pa{};
    pa.op[0] = {static_cast<const bf16raw *>(q), qt, nullptr};
    pa.op[1] = {static_cast<const bf16raw *>(k), kt, g->dev_w_tok};
    pa.op[2] = {static_cast<const bf16raw *>(dout), got, nullptr};
    pa.stat_op = 2;
    pa.o = static_cast<const bf16raw *>(out);
    pa.lse = lse;
    pa.L2 = L2;
    pa.D = Dv;
    pa.ln_wref = g->dt.ln_omega_ref;
    launch_prepare(pa, 3, nbh, N, Npad, st);
    const float c2 = scale * kLog2e;
    const int nblk = (N + 127) / 128, nunits = nbh * nblk;
    const dim3 grid(8 * ((nunits + 7) / 8));
    {
    S2TraceScope tr("global_bwd_dkdv", double(nbh) * N * N, st);
    hipLaunchKernelGGL(global_bwd_dkdv, grid, dim3(256), 0, st, static_cast<const bf16raw *>(q),
                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(v),
                       static_cast<const bf16raw *>(dout), qt, got, g->dev_w_tok, L2, Dv,
                       static_cast<bf16raw *>(dk), static_cast<bf16raw *>(dv), N, Npad, nblk, nunits, c2, scale);
    }
    S2TraceScope tr("global_bwd_dq", double(nbh) * N * N, st);
    const bool dead = Npad != N || !g->zero_lat.empty();      // keys of weight zero exist
    auto dq_kernel = dead ? global_bwd_dq<true> : global_bwd_dq<false>;
    hipLaunchKernelGGL(dq_kernel, grid, dim3(256), 0, st, static_cast<const bf16raw *>(q),
                       static_cast<const bf16raw *>(k), static_cast<const bf16raw *>(v),
                       static_cast<const bf16raw *>(dout), kt, L2, Dv, static_cast<bf16raw *>(dq), N, Npad, nblk,
                       nunits, c2, scale);
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}
