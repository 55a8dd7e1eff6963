// Internal definitions shared by the translation units of libs2attn.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "s2attn.h"

// Device-resident compact form of the indicator 1[h,h',w'] (App. B.3).
// For output latitude h the disk meets the input latitudes
// band_lo[h] .. band_lo[h]+band_n[h]-1; on input latitude h' it covers `cnt`
// consecutive longitude offsets centred on w' = 0 (cnt odd), or the whole
// circle (cnt == nlon_in).  tband_*/tcnt hold the same numbers indexed by the
// input latitude (input point -> output latitudes), used by the dk/dv gather.
struct S2DeviceTables {
    const float *omega_rel;   // [nlat_in]   omega[h'] / max omega
    const int *band_lo;       // [nlat_out]
    const int *band_n;        // [nlat_out]
    const int *cnt;           // [nlat_out][band_max]
    const int *tband_lo;      // [nlat_in]
    const int *tband_n;       // [nlat_in]
    const int *tcnt;          // [nlat_in][tband_max]
    const int *row_order;     // [nlat_out]  output latitudes, heaviest first
    const int *trow_order;    // [nlat_in]   input latitudes, heaviest first
    int band_max, tband_max;
    int fwd_cls[4];           // output latitudes (in row_order) whose run list is split 8, 4, 2, 1 ways
    int bwd_cls[4];           // same for input latitudes (trow_order)
    double fwd_pairs[4];      // (output, input) pairs per slice handled by each class of output latitudes
    double bwd_pairs[4];      // the same pairs counted per class of input latitudes
    // the same four tables with all class thresholds divided by four: used when there are too few
    // (batch, head) slices for the coarse split to fill the machine
    int fwd_cls_fine[4], bwd_cls_fine[4];
    double fwd_pairs_fine[4], bwd_pairs_fine[4];
    int nlat_in, nlon_in, nlat_out, nlon_out, pscale;
    // streaming kernels for the light latitudes (the last class): contiguous range [st_lo, st_hi) of output
    // latitudes and the number of wavefronts st_nw such that the band of latitude h + st_nw starts no earlier
    // than the last row of the band of h; st_nw = 0 if the light latitudes do not have that structure.
    // tst_*: the same for input latitudes and the transposed bands.
    int st_lo, st_hi, st_nw;
    int tst_lo, tst_hi, tst_nw;
    // bf16 band-tile kernels, light variant: contiguous range [bl_lo, bl_hi) of output latitudes of the last class whose
    // arcs are all odd and at most 57 offsets long (0, 0 if the light latitudes do not have that structure);
    // tbl_*: the same for input latitudes and the transposed bands.
    int bl_lo, bl_hi, tbl_lo, tbl_hi;
    // fp32 band-tile kernels: on both sides the bands of any four consecutive latitudes 4 s .. 4 s + 3 together span
    // at most 64 rows (a workgroup keeps one row per lane)
    int band_rows_ok;
    unsigned *dev_flags;      // one word in device memory: bit 0 = a bounded wait inside a kernel ran out
    const int *st_cum;        // [st_hi - st_lo + 1]   running cost of the light latitudes (for equal-work segments)
    const int *tst_cum;       // [tst_hi - tst_lo + 1]
    float ln_omega_ref;       // ln(max omega): the stored logsumexp is relative to the true omega
    float omega_ref;          // max omega
    // upsampling (nlon_out = upscale * nlon_in, upscale > 1; pscale is 1 then): output longitude w = upscale*m + s
    // lies between input meridians, so the arc on input latitude band_lo[h] + b depends on the class s:
    // input columns m + ulo .. m + ulo + ucnt - 1 (ucnt may be 0), tables indexed [(h*upscale + s)*band_max + b]
    int upscale;
    const int *ucnt;
    const int *ulo;
};

struct s2_grid {
    int grid_type;
    int nlat_in, nlon_in, nlat_out, nlon_out, pscale;
    double theta;
    std::vector<double> colat_in, omega_in, colat_out;
    // host copies of the compact tables
    std::vector<int> band_lo, band_n, cnt, tband_lo, tband_n, tcnt, row_order, trow_order, st_cum, tst_cum;
    int upscale = 1;
    std::vector<int> ucnt, ulo;      // upsampling only (see S2DeviceTables)
    int band_max = 0, tband_max = 0;
    // the band and arc tables exactly as eq. (5) gives them (introspection); the tables above, which the kernels
    // use, leave out input latitudes of weight zero (listed in zero_lat)
    std::vector<int> c_band_lo, c_band_n, c_cnt, c_ucnt, c_ulo, zero_lat;
    int c_band_max = 0;
    // canonical CSR
    std::vector<int64_t> row_ptr;
    std::vector<int32_t> col;
    // device side
    bool on_device = false;
    int device = -1;
    void *dev_blob = nullptr;
    // global attention: omega / max omega per input token, 0 on the padding up to npad_tok (a multiple of 64)
    int npad_tok = 0;
    const float *dev_w_tok = nullptr;
    S2DeviceTables dt{};
};

// Class table for the split vector kernels.  `dense_taken`: another kernel has taken the latitudes above the
// coarse threshold (classes 0-2 of the coarse table = class 0 of the fine one).  If the coarse split would start
// so few wavefronts that most SIMDs hold fewer than eight, the copy `t` is switched to the fine split.
inline void s2_pick_split(S2DeviceTables &t, bool fwd, int nbh, int nseg, bool dense_taken)
{
    int *c = fwd ? t.fwd_cls : t.bwd_cls;
    double *p = fwd ? t.fwd_pairs : t.bwd_pairs;
    if (dense_taken) {
        c[0] = c[1] = c[2] = 0;
        p[0] = p[1] = p[2] = 0.0;
    }
    const long waves = long(nbh) * nseg * (8 * c[0] + 4 * c[1] + 2 * c[2] + c[3]);
    if (waves >= 8192) return;
    const int *cf = fwd ? t.fwd_cls_fine : t.bwd_cls_fine;
    const double *pf = fwd ? t.fwd_pairs_fine : t.bwd_pairs_fine;
    for (int i = 0; i < 4; ++i) {
        c[i] = dense_taken && i == 0 ? 0 : cf[i];
        p[i] = dense_taken && i == 0 ? 0.0 : pf[i];
    }
}

// Optional per-launch timing (s2_trace_* in the C ABI): when enabled, a scope records a HIP event
// before and after the launches it encloses, on the stream they go to.
void s2_trace_begin(const char *name, double pairs, hipStream_t st);
void s2_trace_end(hipStream_t st);
struct S2TraceScope {
    hipStream_t st;
    S2TraceScope(const char *name, double pairs, hipStream_t s) : st(s) { s2_trace_begin(name, pairs, s); }
    ~S2TraceScope() { s2_trace_end(st); }
};

// Test-only switches (bits of s2_debug_control): which kernel families the dispatch may pick, and a forced
// launcher failure.
bool s2_debug_flag(unsigned bit);

// One-time set-up of the kernels of each translation unit on the current device: raises the dynamic LDS limit of
// every kernel that needs more than the default.  Called from s2_grid_init (once per device), so that the attention
// calls themselves only enqueue launches.  0 on success.
int s2_nattn_tiled_configure();
int s2_nattn_bwd_tiled_configure();
int s2_nattn_stream_configure();
int s2_nattn_mfma_configure();
int s2_nattn_band_configure();
int s2_mha_configure();

// great-circle angle between two points given by their colatitudes and their difference in longitude (float64)
double s2_great_circle(double colat_a, double colat_b, double dphi);

// Channel matrices on the fp32 matrix cores (s2_mha.hip), all tensors [batch][channels][N] contiguous:
//   s2_gemm_f32:  C[b][m][n] (+)= sum_k A(m, k) X[b][k][n] + bias[m] + R[b][m][n],  A = W (M x K) or W^T (W is K x M)
//   s2_wgrad_f32: dW[m][k] = sum_{b, n} dY[b][m][n] X[b][k][n]  (partial sums in `part`, s2_wgrad_part_floats(M, K)
//                 floats, added in a fixed order)
//   s2_channel_sum_f32: out[c] = sum_{b, n} u[b][c][n]  (`part`: scratch of part_floats floats for partial sums, may be
//                       NULL: then one workgroup per channel does the whole sum)
// M, K multiples of 16 and N a multiple of 16.
void s2_gemm_f32(bool trans_a, int M, int N, int K, int batch, const float *W, const float *X, const float *bias,
                 const float *R, float *C, bool accumulate, hipStream_t st);
size_t s2_wgrad_part_floats(int M, int K);
void s2_wgrad_f32(int M, int K, int N, int batch, const float *dY, const float *X, float *part, float *dW, hipStream_t st);
void s2_channel_sum_f32(int batch, int C, int N, const float *u, float *out, float *part, size_t part_floats,
                        hipStream_t st);

void s2_set_error(const std::string &msg);
int s2_fail(int code, const std::string &msg);

#define S2_HIP_CHECK(expr)                                                                   \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return s2_fail(S2_ERR_DEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)
