// s2_nattn_bwd_static: the neighborhood-attention backward for callers that cannot allocate or hand over device
// scratch.  The per-point constants D_i = dout_i . out_i, which s2_nattn_bwd keeps in the caller's workspace, live
// here in a fixed array in device memory that every GPU the library runs on holds until the process ends.
#include <mutex>

#include "s2_nattn_kernels.h"

namespace {

constexpr size_t kScratchFloats = S2_STATIC_SCRATCH_BYTES / sizeof(float);
constexpr int kMaxDevices = 64;

// The array's name is a host-side stand-in for the symbol: host code never passes it anywhere.  Each device has
// its own copy at its own address, looked up once (with that device current) and kept in g_scratch_ptr.
static __device__ __align__(256) float scratch[kScratchFloats];

float *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

}  // namespace

int s2_static_scratch_setup(int device)
{
    if (device < 0 || device >= kMaxDevices) return -1;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[device]) return 0;
    float *ptr = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return -1;
    }
    g_scratch_ptr[device] = ptr;
    return 0;
}

extern "C" size_t s2_nattn_bwd_static_max_points(void) { return kScratchFloats; }

extern "C" int s2_nattn_bwd_static(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype, float scale,
                                   const void *q, const void *k, const void *v, const void *out, const float *lse,
                                   const void *dout, void *dq, void *dk, void *dv, void *hip_stream)
{
    if (!g) return s2_fail(S2_ERR_INVALID_ARG, "grid is NULL");
    if (batch < 1 || heads < 1) return s2_fail(S2_ERR_INVALID_ARG, "batch, heads, d must be >= 1");
    if (!g->on_device) return s2_fail(S2_ERR_DEVICE, "grid handle has no device tables (no HIP device at init)");
    const size_t need = size_t(batch) * heads * g->nlat_out * g->nlon_out;
    if (need > kScratchFloats)
        return s2_fail(S2_ERR_WORKSPACE, "batch*heads*nlat_out*nlon_out = " + std::to_string(need) +
                                             " exceeds the static scratch of " + std::to_string(kScratchFloats) +
                                             " points; use s2_nattn_bwd with a workspace");
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess || cur != g->device)
        return s2_fail(S2_ERR_DEVICE, "the device the grid handle was created on is not the current device");
    float *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        ptr = g_scratch_ptr[g->device];
    }
    if (!ptr) return s2_fail(S2_ERR_DEVICE, "static scratch was not set up on this device");
    // nothing in the array has to start at zero: the dq launches store D_i for every output point of the call
    // before the dk/dv launches (same stream) read it
    return s2_nattn_bwd_run(g, batch, heads, d_qk, d_v, dtype, scale, q, k, v, out, lse, dout, dq, dk, dv, ptr,
                            static_cast<hipStream_t>(hip_stream));
}
