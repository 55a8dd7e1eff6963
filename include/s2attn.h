/*
 * s2attn.h -- C ABI of the MI355X (gfx950) spherical attention library.
 *
 * Quadrature-weighted attention on latitude-longitude grids of the sphere
 * ("Attention on the Sphere"): the neighborhood variant restricted to a
 * geodesic disk and the global variant, forward and backward.
 *
 * Conventions
 *   - Every tensor pointer is DEVICE memory owned by the caller; the library
 *     reads inputs, writes outputs and never keeps a pointer after the call.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*; NULL
 *     is the default stream) and return without synchronising.
 *   - The only allocations happen in s2_grid_init (host tables plus one small
 *     device upload).  Scratch memory for the backward passes is passed in as
 *     `workspace`; its size comes from the *_workspace_bytes queries.
 *   - Return value: S2_OK or a negative S2_ERR_* code; s2_last_error() gives
 *     a thread-local message for the last failure on the calling thread.
 *   - Batch and heads are independent problems; tensors carry them as the two
 *     leading axes [batch][heads]... contiguous (App. B.3: B x C x H x W with
 *     C = heads * d).
 */
#ifndef S2ATTN_H
#define S2ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct s2_grid s2_grid_t; /* opaque; immutable after init; usable from any stream */

/* Grid types (Sec. 3.3: equiangular and Gaussian grids). */
enum {
    S2_GRID_EQUIANGULAR = 0,   /* colat_h = pi*h/(nlat-1), both poles, Clenshaw-Curtis weights */
    S2_GRID_LEGENDRE_GAUSS = 1, /* Gauss-Legendre nodes in cos(colat), north first */
    S2_GRID_LEGENDRE_GAUSS_LOBATTO = 3, /* Gauss-Lobatto nodes in cos(colat): both poles plus the zeros of P'_{nlat-1} */
    S2_GRID_EQUIANGULAR_TRAPEZOID = 2 /* the grid as printed in App. A.1: colat_i = pi*i/nlat, i < nlat (north pole
                                         only), weights 2 pi^2 / (nlat nlon) sin(colat_i): zero at the pole, whose
                                         points then never contribute; sums to 4 pi only approximately */
};

enum { S2_F32 = 0, S2_BF16 = 1 };

enum {
    S2_OK = 0,
    S2_ERR_INVALID_ARG = -1,
    S2_ERR_UNSUPPORTED = -2,
    S2_ERR_EMPTY_NEIGHBORHOOD = -3,
    S2_ERR_ALLOC = -4,
    S2_ERR_DEVICE = -5,
    S2_ERR_WORKSPACE = -6,
    S2_ERR_AMBIGUOUS_CUTOFF = -7
};

/*
 * Host precompute (App. A.1 quadrature; Sec. 3.2 eq. (5) disk; App. B.3
 * shift-invariant indicator 1[h,h',w']).
 *
 * Builds, in float64 on the host: colatitudes and quadrature weights
 * omega[h'] = latitude weight * 2*pi/nlon_in of the INPUT grid, and for every
 * output latitude h the input points (h', w') whose great-circle distance to
 * the output point (h, longitude 0) is <= theta_cutoff + 1e-9 rad.  The lists
 * are reused for every output longitude w by the shift w' -> w' + w*pscale,
 * pscale = nlon_in / nlon_out (equal grids and downsampling).  Upsampling
 * (nlon_out = r * nlon_in): output longitude w = r*m + s lies between input
 * meridians unless s = 0, so every latitude gets r lists (one per s), each
 * reused for every m by the shift w' -> w' + m.  Both grids have the same
 * grid_type.
 *
 * If a HIP device is present the compact tables are uploaded to the current
 * device; without a device the handle is host-only (the introspection calls
 * work, the attention calls return S2_ERR_DEVICE).  The first call on a
 * device also raises the LDS limits of the library's kernels there (guarded
 * by a mutex), so that the attention calls only enqueue launches and can be
 * captured into a HIP graph from their first call on.  A handle must be used
 * with the device that was current when it was created.
 *
 * Errors: S2_ERR_INVALID_ARG (nlat < 2, nlon < 1, theta outside (0, pi], NULL
 * out_grid, unknown grid_type); S2_ERR_UNSUPPORTED (neither longitude count
 * is a multiple of the other); S2_ERR_EMPTY_NEIGHBORHOOD (some output point sees no input point);
 * S2_ERR_AMBIGUOUS_CUTOFF (a point lies within 1e-12 rad of the inclusion
 * threshold, so membership would depend on rounding: perturb theta_cutoff);
 * S2_ERR_ALLOC / S2_ERR_DEVICE.
 * Ownership: *out_grid is owned by the library; release with s2_grid_destroy.
 */
int s2_grid_init(int grid_type, int nlat_in, int nlon_in, int nlat_out, int nlon_out,
                 double theta_cutoff, s2_grid_t **out_grid);
void s2_grid_destroy(s2_grid_t *g);

/* Introspection (host buffers; any pointer may be NULL to skip it).
 * colat_in, omega_in: nlat_in doubles (omega includes 2*pi/nlon_in). */
int s2_grid_get_weights(const s2_grid_t *g, double *colat_in, double *omega_in);
/* Number of entries of the canonical neighbor list (sum over output latitudes). */
int64_t s2_grid_num_neighbors(const s2_grid_t *g);
/* Canonical CSR of 1[h,h',w']: row_ptr has nlat_out+1 entries; col holds
 * h'*nlon_in + w' with w' in [0, nlon_in), ascending within each output
 * latitude; col needs s2_grid_num_neighbors(g) entries. */
int s2_grid_get_neighbors(const s2_grid_t *g, int64_t *row_ptr, int32_t *col);
/* Neighbor list of one output point (h, w), eq. (5): absolute input indices h'*nlon_in + w_in,
 * ascending; *count receives their number, col (if not NULL) needs that many entries.  On
 * upsampling grids (nlon_out a multiple of nlon_in) the lists of the output longitudes between two
 * input meridians differ from the one s2_grid_get_neighbors reports for longitude 0.
 * S2_ERR_INVALID_ARG for a point outside the output grid. */
int s2_grid_get_neighbors_at(const s2_grid_t *g, int h, int w, int32_t *col, int *count);

/* Bytes of device scratch s2_nattn_bwd needs (0 for the forward pass). */
size_t s2_nattn_bwd_workspace_bytes(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype);

/*
 * Neighborhood attention forward (App. B.1 second equation; index form of
 * App. B.3):
 *   out[b,hd,c,h,w] = sum_{(h',w') in list(h)} p * v[b,hd,c,h',(w*pscale+w') mod nlon_in]
 *   p = exp(scale * q[b,hd,:,h,w].k[b,hd,:,h',...] + ln omega[h'] - lse[b,hd,h,w])
 *   lse = ln sum exp(scale*q.k + ln omega)        (natural log, omega included)
 * Layouts (contiguous): q, out [batch][heads][d][nlat_out][nlon_out] (out has
 * d_v channels); k [batch][heads][d_qk][nlat_in][nlon_in]; v likewise with d_v;
 * lse float32 [batch][heads][nlat_out][nlon_out].
 * dtype: S2_F32 (float32 tensors, float32 arithmetic throughout) or S2_BF16 (q, k, v, out bf16; products on the
 * bf16 matrix cores where the shape allows - equal grids, d_qk = d_v = 32, longitude count a multiple of 64 - with
 * float32 accumulation and softmax, otherwise float32 arithmetic on bf16 loads; lse float32 either way).
 * d_qk, d_v in [1, 128].
 * Errors: S2_ERR_INVALID_ARG (NULL or not 16-byte aligned pointers, sizes < 1),
 * S2_ERR_UNSUPPORTED (dtype, head dims), S2_ERR_DEVICE (host-only handle or
 * launch failure).
 */
int s2_nattn_fwd(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype, float scale,
                 const void *q, const void *k, const void *v, void *out, float *lse,
                 void *hip_stream);

/*
 * Neighborhood attention backward (App. B.4, with the derivation's typos
 * fixed): given dout = dL/dout and the forward's out and lse,
 *   p_ij = exp(scale*q_i.k_j + ln omega_j - lse_i),  D_i = dout_i.out_i,
 *   dS_ij = p_ij (dout_i.v_j - D_i),
 *   dq_i = scale * sum_{j in N(i)} dS_ij k_j,
 *   dk_j = scale * sum_{i: j in N(i)} dS_ij q_i,   dv_j = sum_{i: j in N(i)} p_ij dout_i.
 * dk and dv are gathered through the transposed neighborhood (input point ->
 * output points): no atomics, bit-reproducible.  omega carries no gradient.
 * dq like q, dk like k, dv like v (bf16 for S2_BF16; D_i and lse stay float32).  workspace: device scratch of at least
 * s2_nattn_bwd_workspace_bytes(...) bytes (S2_ERR_WORKSPACE if smaller).
 */
int s2_nattn_bwd(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype, float scale,
                 const void *q, const void *k, const void *v, const void *out, const float *lse,
                 const void *dout, void *dq, void *dk, void *dv,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * s2_nattn_bwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * s2_nattn_bwd without `workspace`: the per-point scratch lives in a fixed array of S2_STATIC_SCRATCH_BYTES in
 * device memory that each GPU the library runs on holds until the process ends (its address is looked up once per
 * device in s2_grid_init).  The call allocates nothing and calls no allocating routine (keep s2_trace_enable off:
 * tracing creates events).  Limit: batch*heads*nlat_out*nlon_out <= s2_nattn_bwd_static_max_points() (2 097 152;
 * workload 3 needs 1 056 768), otherwise S2_ERR_WORKSPACE; S2_ERR_DEVICE if the handle's device is not the current
 * device.  All calls on one GPU share the array: calls that overlap on one GPU (different streams or threads)
 * race; calls on one stream are ordered and each call overwrites what it later reads, so nothing needs clearing.
 */
#define S2_STATIC_SCRATCH_BYTES (8u << 20)
size_t s2_nattn_bwd_static_max_points(void);
int s2_nattn_bwd_static(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype, float scale,
                        const void *q, const void *k, const void *v, const void *out, const float *lse,
                        const void *dout, void *dq, void *dk, void *dv, void *hip_stream);

/* Bytes of device scratch s2_attn_global_fwd / s2_attn_global_bwd need (token-transposed
 * copies of the operands that are contracted over tokens, and per-token constants of the
 * backward pass). */
size_t s2_attn_global_fwd_workspace_bytes(const s2_grid_t *g, int batch, int heads, int d, int dtype);
size_t s2_attn_global_bwd_workspace_bytes(const s2_grid_t *g, int batch, int heads, int d, int dtype);

/*
 * Global quadrature-weighted attention forward (App. B.1 first equation;
 * App. B.2: softmax with the additive column bias ln omega_j):
 *   out_i = sum_j softmax_j(scale*q_i.k_j + ln omega_j) v_j over all N tokens.
 * The handle must have identical input and output grids; token j = h*nlon + w,
 * N = nlat*nlon.  Layouts (contiguous, token-major): q, k, v, out
 * [batch][heads][N][d]; lse float32 [batch][heads][N].
 * dtype: S2_BF16 (bf16 tensors, MFMA with float32 accumulation, float32
 * softmax and lse); d = 64.  Other dtypes or head dimensions: S2_ERR_UNSUPPORTED.
 * workspace: device scratch of at least s2_attn_global_fwd_workspace_bytes(...)
 * bytes, 256-byte aligned (S2_ERR_WORKSPACE otherwise); its contents are undefined
 * afterwards.  Tensor pointers must be 16-byte aligned (S2_ERR_INVALID_ARG).
 */
int s2_attn_global_fwd(const s2_grid_t *g, int batch, int heads, int d, int dtype, float scale,
                       const void *q, const void *k, const void *v, void *out, float *lse,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Global attention backward: the formulas of s2_nattn_bwd with every token a
 * member of every neighborhood.  dq, dk, dv in the tensors' dtype.
 */
int s2_attn_global_bwd(const s2_grid_t *g, int batch, int heads, int d, int dtype, float scale,
                       const void *q, const void *k, const void *v, const void *out, const float *lse,
                       const void *dout, void *dq, void *dk, void *dv,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Spherical multi-head attention sub-block (Sec. 3.4, "Spherical attention blocks": instance normalisation, position
 * embedding, multi-head neighborhood attention, residual), float32, self-attention on one grid (the handle's input
 * and output grids must be equal):
 *   xhat = (x - mean) / sqrt(var + eps) per (batch, channel) over the grid points (plain moments, biased variance)
 *   xn = gamma xhat + beta + pos;  q, k, v = Wq xn + bq, Wk xn + bk, Wv xn + bv   (1x1 convolutions)
 *   a = neighborhood attention per head, head i = channels i*d .. (i+1)*d - 1, d = channels / heads, scale 1/sqrt(d)
 *   y = x + Wo a + bo
 * x, y, dy, dx: [batch][channels][nlat][nlon] contiguous.  Parameters (device pointers): gamma, beta, bq, bk, bv, bo
 * [channels] and pos [channels][nlat][nlon] may be NULL (1, 0, no bias, no embedding); Wq, Wk, Wv, Wo
 * [channels out][channels in] row-major are required.  s2_mha_bwd writes the gradients of sum(dy * y) to dx and to
 * every non-NULL pointer of `grads` (same shapes as the parameters).
 * workspace: device scratch of s2_mha_workspace_bytes(...) bytes, 256-byte aligned; it carries the activations the
 * backward needs, so s2_mha_bwd must get the workspace of the matching s2_mha_fwd call, untouched.
 * channels and nlat*nlon must be multiples of 16 (else S2_ERR_UNSUPPORTED); x, y, dy, dx, pos and the weight
 * matrices must be 16-byte aligned (else S2_ERR_INVALID_ARG).  Every step runs in the library's own
 * kernels (channel matrices on the fp32 matrix cores); results are bit-reproducible.
 */
typedef struct {
    const float *gamma, *beta, *pos;
    const float *Wq, *bq, *Wk, *bk, *Wv, *bv, *Wo, *bo;
} s2_mha_params_t;
typedef struct {
    float *gamma, *beta, *pos;
    float *Wq, *bq, *Wk, *bk, *Wv, *bv, *Wo, *bo;
} s2_mha_grads_t;
size_t s2_mha_workspace_bytes(const s2_grid_t *g, int batch, int channels, int heads);
int s2_mha_fwd(const s2_grid_t *g, int batch, int channels, int heads, float eps, const float *x,
               const s2_mha_params_t *params, float *y, void *workspace, size_t workspace_bytes, void *hip_stream);
int s2_mha_bwd(const s2_grid_t *g, int batch, int channels, int heads, float eps, const float *x,
               const s2_mha_params_t *params, const float *dy, float *dx, const s2_mha_grads_t *grads,
               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Discrete-continuous (DISCO) convolution on the disk tables of a grid handle (App. B.3, first equation):
 *   z[b,c,k,h,w] = sum_{(h',w') in list(h)} psi_k[h,h',w'] x[b,c,h',(w' + w*pscale) mod nlon_in]
 *   y[b,o,h,w]   = sum_{c,k} weight[o,c,k] z[b,c,k,h,w] + bias[o]
 * with psi_k = hat_k(r) * omega[h'], r the geodesic distance of the input point from the output point and
 * hat_k(r) = max(0, 1 - |r * nbasis / theta_cutoff - k|), k = 0 .. nbasis-1 (piecewise-linear, isotropic; the paper
 * leaves the basis open).  s2_disco_init tabulates psi in float64 on the host for the handle's grids (equal grids or
 * downsampling; upsampling handles: S2_ERR_UNSUPPORTED); nbasis in [1, 16].  The disco handle refers to the grid
 * handle, which must outlive it; release with s2_disco_destroy.
 * Layouts (contiguous float32, device): x [batch][cin][nlat_in][nlon_in], y, dy [batch][cout][nlat_out][nlon_out],
 * weight [cout][cin][nbasis], bias [cout] (may be NULL).  s2_disco_bwd writes dx and, where the pointers are not
 * NULL, dweight and dbias; it needs the workspace of the matching s2_disco_fwd call, untouched (z is kept there).
 * cin*nbasis, cout and nlat_out*nlon_out must be multiples of 16 (else S2_ERR_UNSUPPORTED); batch*cin <= 65535.
 * x, y, dy, dx and weight must be 16-byte aligned (else S2_ERR_INVALID_ARG).
 * workspace: s2_disco_workspace_bytes(...) bytes, 256-byte aligned.  No atomics: results are bit-reproducible.
 */
typedef struct s2_disco s2_disco_t;
int s2_disco_init(const s2_grid_t *g, int nbasis, s2_disco_t **out);
void s2_disco_destroy(s2_disco_t *dc);
size_t s2_disco_workspace_bytes(const s2_disco_t *dc, int batch, int cin, int cout);
int s2_disco_fwd(const s2_disco_t *dc, int batch, int cin, int cout, const float *x, const float *weight,
                 const float *bias, float *y, void *workspace, size_t workspace_bytes, void *hip_stream);
int s2_disco_bwd(const s2_disco_t *dc, int batch, int cin, int cout, const float *x, const float *weight,
                 const float *dy, float *dx, float *dweight, float *dbias, void *workspace, size_t workspace_bytes,
                 void *hip_stream);

/*
 * Per-launch timing for benchmarks (not part of the method).  While enabled, every kernel launch
 * of the attention calls is bracketed by HIP events on the launch stream.  s2_trace_get waits for
 * entry `index` and returns the kernel's name, its duration in ms and the number of (output, input)
 * pairs it covered (batch and heads included); s2_trace_reset drops all entries.  Creates events,
 * so do not enable it under graph capture.  Not thread safe.
 */
int s2_trace_enable(int on);   /* returns the previous setting */
int s2_trace_count(void);
int s2_trace_get(int index, const char **name, float *ms, double *pairs);
void s2_trace_reset(void);

/*
 * Measured ceilings of the current device, for the roofline figures of the benchmark (not part of the method).
 * Runs a plain kernel of the named kind (allocating and freeing its own buffers, on the default stream,
 * synchronising) and stores the rate in *value (host pointer):
 *   S2_PEAK_COPY       streaming copy of 1 GiB, GB/s counting bytes read plus bytes written
 *   S2_PEAK_FMA_F32    independent v_fma_f32 chains, TFLOP/s
 *   S2_PEAK_MFMA_F32   v_mfma_f32_32x32x2_f32 chains, TFLOP/s
 *   S2_PEAK_MFMA_BF16  v_mfma_f32_32x32x16_bf16 chains, TFLOP/s
 *   S2_PEAK_LDS_READ   conflict-free 16-byte LDS reads, TB/s over the whole device
 * Errors: S2_ERR_INVALID_ARG, S2_ERR_ALLOC, S2_ERR_DEVICE.
 */
enum { S2_PEAK_COPY = 0, S2_PEAK_FMA_F32 = 1, S2_PEAK_MFMA_F32 = 2, S2_PEAK_MFMA_BF16 = 3, S2_PEAK_LDS_READ = 4 };
int s2_peak_measure(int kind, double *value);

/* Device-side health of a grid handle (Sec. 3.2 / App. B.3 kernels that synchronise wavefronts through counters
 * in LDS bound every wait; a wait that ran out - which would be a defect of the library, the results of that call
 * are then wrong - sets a sticky flag in device memory).  Synchronises the device, copies the flag word to *flags
 * (0 = healthy) and clears it.  Host pointer; S2_ERR_INVALID_ARG for NULL arguments, S2_ERR_DEVICE if the handle
 * has no device tables or the copy fails. */
int s2_grid_device_flags(const s2_grid_t *g, unsigned *flags);

/*
 * Test-only dispatch switches (not part of the method; nothing else steers the dispatch: the library reads no
 * environment variables).  Sets the bits of set_bits, clears those of clear_bits, returns the new word; process
 * wide, takes effect on the next attention call.
 *   S2_DEBUG_NO_MFMA        dense polar latitudes go to the split vector kernels instead of the matrix cores
 *   S2_DEBUG_NO_STREAM      light latitudes go to the one-wavefront kernels instead of the streaming kernels
 *   S2_DEBUG_NO_ROW_GROUPS  matrix-core kernels never start a second set of wavefronts per workgroup
 *   S2_DEBUG_FAIL_LAUNCH    the launchers of the tuned neighborhood kernels report failure before launching
 *                           anything: s2_nattn_fwd / s2_nattn_bwd then return S2_ERR_DEVICE
 *   S2_DEBUG_FORCE_BAND     float32 tensors with d = e = 32 always run on the band-tile matrix-core kernels that
 *                           serve d = e = 16 and 64 (by default only where the streaming kernels do not apply)
 *   S2_DEBUG_NO_BAND        the band-tile matrix-core kernels are never used (d = 16, 64: shape-agnostic kernels)
 */
enum { S2_DEBUG_NO_MFMA = 1, S2_DEBUG_NO_STREAM = 2, S2_DEBUG_NO_ROW_GROUPS = 4, S2_DEBUG_FAIL_LAUNCH = 8, S2_DEBUG_FORCE_BAND = 16, S2_DEBUG_NO_BAND = 32 };
unsigned s2_debug_control(unsigned set_bits, unsigned clear_bits);

/* Message for the last error on the calling thread ("" if none). */
const char *s2_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* S2ATTN_H */
