// C entry points of the neighborhood attention: argument checks and dispatch.
#include "s2_nattn_kernels.h"

namespace {

int check_common(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype)
{
    if (!g) return s2_fail(S2_ERR_INVALID_ARG, "grid is NULL");
    if (batch < 1 || heads < 1 || d_qk < 1 || d_v < 1) return s2_fail(S2_ERR_INVALID_ARG, "batch, heads, d must be >= 1");
    if (dtype != S2_F32 && dtype != S2_BF16) return s2_fail(S2_ERR_UNSUPPORTED, "unknown dtype");
    if (d_qk > 128 || d_v > 128) return s2_fail(S2_ERR_UNSUPPORTED, "head dimensions above 128 are not supported");
    if (long(batch) * heads > (1l << 20)) return s2_fail(S2_ERR_INVALID_ARG, "batch*heads too large");
    if (!g->on_device) return s2_fail(S2_ERR_DEVICE, "grid handle has no device tables (no HIP device at init)");
    return S2_OK;
}

// the tuned kernels move 16-byte pieces (vector loads and stores, LDS-direct copies)
bool misaligned(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 != 0; }

}  // namespace

extern "C" size_t s2_nattn_bwd_workspace_bytes(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype)
{
    (void)d_qk; (void)d_v; (void)dtype;
    if (!g || batch < 1 || heads < 1) return 0;
    // D_i = dout_i . out_i, one float per output point and (batch, head)
    return size_t(batch) * heads * g->nlat_out * g->nlon_out * sizeof(float);
}

// The fp32 band-tile kernels take the head dimensions the hand-tuned d = 32 kernels do not cover, and d = 32 itself on
// grids whose light latitudes do not have the structure the streaming kernels need (bands of more than nine rows,
// e.g. the 64 x 128 Gauss grid: measured 0.41 against 0.71 ms per step there, but 2.9 against 2.5 ms on the
// 129 x 256 grid, where the streaming kernels run).
static bool use_band(const S2DeviceTables &t, int d, int e)
{
    if (!s2_nattn_band_supported(t, d, e) || s2_debug_flag(S2_DEBUG_NO_BAND)) return false;
    if (d != 32 || s2_debug_flag(S2_DEBUG_FORCE_BAND)) return true;
    return !(s2_nattn_stream_supported(t, d, e) && s2_nattn_stream_dq_supported(t, d, e) &&
             s2_nattn_stream_dkdv_supported(t, d, e));
}

// bf16 tensors: what the bf16 matrix-core kernels (d = 32, longitude count a multiple of 64) do not cover goes to the
// fp32 band tiles with bf16 loads and stores where those apply.
static bool band_bf16(const S2DeviceTables &t, int d, int e)
{
    return s2_nattn_band_supported(t, d, e) && !s2_debug_flag(S2_DEBUG_NO_BAND);
}

extern "C" int s2_nattn_fwd(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype, float scale,
                            const void *q, const void *k, const void *v, void *out, float *lse, void *hip_stream)
{
    int rc = check_common(g, batch, heads, d_qk, d_v, dtype);
    if (rc) return rc;
    if (!q || !k || !v || !out || !lse) return s2_fail(S2_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(lse))
        return s2_fail(S2_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (dtype == S2_BF16) {
        auto *fwd16 = s2_nattn_bf16_supported(g->dt, d_qk, d_v) ? s2_nattn_fwd_bf16
                      : band_bf16(g->dt, d_qk, d_v)             ? s2_nattn_fwd_band_bf16
                                                                : s2_nattn_fwd_generic_bf16;
        if (fwd16(g->dt, batch * heads, d_qk, d_v, scale, q, k, v, out, lse, st))
            return s2_fail(S2_ERR_DEVICE, "forward launch configuration failed");
        S2_HIP_CHECK(hipGetLastError());
        return S2_OK;
    }
    auto *fwd = use_band(g->dt, d_qk, d_v)                       ? s2_nattn_fwd_band
                : s2_nattn_fwd_tiled_supported(g->dt, d_qk, d_v) ? s2_nattn_fwd_tiled
                                                                 : s2_nattn_fwd_generic;
    if (fwd(g->dt, batch * heads, d_qk, d_v, scale, static_cast<const float *>(q), static_cast<const float *>(k),
            static_cast<const float *>(v), static_cast<float *>(out), lse, st))
        return s2_fail(S2_ERR_DEVICE, "forward launch configuration failed");
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}

// Argument checks and dispatch shared by s2_nattn_bwd and s2_nattn_bwd_static; Dws: device scratch for D_i.
int s2_nattn_bwd_run(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype, float scale,
                     const void *q, const void *k, const void *v, const void *out, const float *lse, const void *dout,
                     void *dq, void *dk, void *dv, float *Dws, hipStream_t st)
{
    int rc = check_common(g, batch, heads, d_qk, d_v, dtype);
    if (rc) return rc;
    if (!q || !k || !v || !out || !lse || !dout || !dq || !dk || !dv)
        return s2_fail(S2_ERR_INVALID_ARG, "NULL tensor pointer");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(lse) || misaligned(dout) ||
        misaligned(dq) || misaligned(dk) || misaligned(dv))
        return s2_fail(S2_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
    if (dtype == S2_BF16) {
        const bool fast = s2_nattn_bf16_supported(g->dt, d_qk, d_v), band = !fast && band_bf16(g->dt, d_qk, d_v);
        auto *dq16 = fast ? s2_nattn_bwd_dq_bf16 : band ? s2_nattn_bwd_dq_band_bf16 : s2_nattn_bwd_dq_generic_bf16;
        auto *kv16 = fast ? s2_nattn_bwd_dkdv_bf16 : band ? s2_nattn_bwd_dkdv_band_bf16 : s2_nattn_bwd_dkdv_generic_bf16;
        if (dq16(g->dt, batch * heads, d_qk, d_v, scale, q, k, v, out, lse, dout, dq, Dws, st) ||
            kv16(g->dt, batch * heads, d_qk, d_v, scale, q, k, v, lse, dout, Dws, dk, dv, st))
            return s2_fail(S2_ERR_DEVICE, "backward launch configuration failed");
    } else {
        auto *bwd = use_band(g->dt, d_qk, d_v)                       ? s2_nattn_bwd_band
                    : s2_nattn_bwd_tiled_supported(g->dt, d_qk, d_v) ? s2_nattn_bwd_tiled
                                                                     : s2_nattn_bwd_generic;
        if (bwd(g->dt, batch * heads, d_qk, d_v, scale, static_cast<const float *>(q), static_cast<const float *>(k),
                static_cast<const float *>(v), static_cast<const float *>(out), lse, static_cast<const float *>(dout),
                static_cast<float *>(dq), static_cast<float *>(dk), static_cast<float *>(dv), Dws, st))
            return s2_fail(S2_ERR_DEVICE, "backward launch configuration failed");
    }
    // input latitudes of weight zero (the pole row of the grid of App. A.1): dk = dv = 0 exactly
    for (int lat : g->zero_lat) {
        s2_nattn_zero_latitude(g->dt, lat, batch * heads * d_qk, dk, dtype == S2_BF16, st);
        s2_nattn_zero_latitude(g->dt, lat, batch * heads * d_v, dv, dtype == S2_BF16, st);
    }
    S2_HIP_CHECK(hipGetLastError());
    return S2_OK;
}

extern "C" int s2_nattn_bwd(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype, float scale,
                            const void *q, const void *k, const void *v, const void *out, const float *lse,
                            const void *dout, void *dq, void *dk, void *dv, void *workspace, size_t workspace_bytes,
                            void *hip_stream)
{
    if (!g) return s2_fail(S2_ERR_INVALID_ARG, "grid is NULL");
    if (!workspace || workspace_bytes < s2_nattn_bwd_workspace_bytes(g, batch, heads, d_qk, d_v, dtype))
        return s2_fail(S2_ERR_WORKSPACE, "workspace missing or smaller than s2_nattn_bwd_workspace_bytes()");
    if (misaligned(workspace)) return s2_fail(S2_ERR_WORKSPACE, "workspace must be 16-byte aligned");
    return s2_nattn_bwd_run(g, batch, heads, d_qk, d_v, dtype, scale, q, k, v, out, lse, dout, dq, dk, dv,
                            static_cast<float *>(workspace), static_cast<hipStream_t>(hip_stream));
}
