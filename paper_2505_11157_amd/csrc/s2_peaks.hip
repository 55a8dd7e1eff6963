// Measured device ceilings for the roofline figures of the benchmark (not part of the method): plain kernels that do
// one thing each - a streaming copy, independent v_fma_f32 chains, fp32 and bf16 matrix-core chains, conflict-free
// 16-byte LDS reads - timed with HIP events.  s2_peak_measure allocates and frees its own buffers.
#include "s2_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__global__ void __launch_bounds__(256) peak_copy(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n)
{
    const size_t stride = size_t(gridDim.x) * 256;
    for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// 16 independent fused multiply-add chains per lane
__global__ void __launch_bounds__(256) peak_fma(float *out, int iters, float a, float b)
{
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = float(threadIdx.x + i);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) x[u] = fmaf(x[u], a, b);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += x[i];
    out[size_t(blockIdx.x) * 256 + threadIdx.x] = s;
}

// four independent accumulator tiles per wavefront, v_mfma_f32_32x32x2_f32
__global__ void __launch_bounds__(256) peak_mfma_f32(float *out, int iters, float a, float b)
{
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    const float av = a + threadIdx.x, bv = b - threadIdx.x;
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    out[size_t(blockIdx.x) * 256 + threadIdx.x] = s;
}

// the same with v_mfma_f32_32x32x16_bf16
__global__ void __launch_bounds__(256) peak_mfma_bf16(float *out, int iters, float a, float b)
{
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    bf16x8 av, bv;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        av[i] = (__bf16)(a + float(threadIdx.x & 7) + i);
        bv[i] = (__bf16)(b - float(threadIdx.x & 3) - i);
    }
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    out[size_t(blockIdx.x) * 256 + threadIdx.x] = s;
}

// conflict-free ds_read_b128: consecutive lanes read consecutive 16-byte pieces of a 64 KB array
__global__ void __launch_bounds__(256) peak_lds(float *out, int iters)
{
    __shared__ float4 buf[4096];
    for (int i = threadIdx.x; i < 4096; i += 256) buf[i] = make_float4(float(i), 1.f, 2.f, 3.f);
    __syncthreads();
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    int idx = threadIdx.x;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const float4 x = buf[(idx + u * 256) & 4095];
            acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
        }
        idx = (idx + 64) & 4095;
    }
    out[size_t(blockIdx.x) * 256 + threadIdx.x] = acc.x + acc.y + acc.z + acc.w;
}

template <class F>
int timed(F launch, int reps, float *ms)
{
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -1;
    launch();                                   // warm-up
    (void)hipEventRecord(a, nullptr);
    for (int r = 0; r < reps; ++r) launch();
    (void)hipEventRecord(b, nullptr);
    int rc = hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(ms, a, b) == hipSuccess ? 0 : -1;
    *ms /= reps;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return rc;
}

}  // namespace

extern "C" int s2_peak_measure(int kind, double *value)
{
    if (!value) return s2_fail(S2_ERR_INVALID_ARG, "value is NULL");
    int dev = 0, ncu = 0;
    S2_HIP_CHECK(hipGetDevice(&dev));
    S2_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int nblk = ncu * 8;                   // two wavefronts per SIMD
    float ms = 0.f;
    if (kind == S2_PEAK_COPY) {
        const size_t bytes = size_t(1) << 30;
        void *src = nullptr, *dst = nullptr;
        if (hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&dst, bytes) != hipSuccess) {
            (void)hipFree(src);
            (void)hipGetLastError();
            return s2_fail(S2_ERR_ALLOC, "hipMalloc for the copy measurement failed");
        }
        (void)hipMemset(src, 1, bytes);
        const int rc = timed([&] {
            hipLaunchKernelGGL(peak_copy, dim3(ncu * 16), dim3(256), 0, nullptr, static_cast<const float4 *>(src),
                               static_cast<float4 *>(dst), bytes / 16);
        }, 5, &ms);
        (void)hipFree(src);
        (void)hipFree(dst);
        if (rc) return s2_fail(S2_ERR_DEVICE, "timing the copy failed");
        *value = 2.0 * double(bytes) / (ms * 1e-3) / 1e9;          // GB/s, read + write
        return S2_OK;
    }
    float *out = nullptr;
    if (hipMalloc(&out, size_t(nblk) * 256 * sizeof(float)) != hipSuccess) {
        (void)hipGetLastError();
        return s2_fail(S2_ERR_ALLOC, "hipMalloc for the peak measurement failed");
    }
    const int iters = 4096;
    int rc = 0;
    double work = 0.0;       // flop (or bytes) per launch
    switch (kind) {
    case S2_PEAK_FMA_F32:
        rc = timed([&] { hipLaunchKernelGGL(peak_fma, dim3(nblk), dim3(256), 0, nullptr, out, iters, 0.999f, 0.5f); }, 5, &ms);
        work = double(nblk) * 256 * 16 * iters * 2;
        break;
    case S2_PEAK_MFMA_F32:
        rc = timed([&] { hipLaunchKernelGGL(peak_mfma_f32, dim3(nblk), dim3(256), 0, nullptr, out, iters, 1e-3f, 2e-3f); }, 5, &ms);
        work = double(nblk) * 4 * 4 * iters * (32.0 * 32 * 2 * 2);
        break;
    case S2_PEAK_MFMA_BF16:
        rc = timed([&] { hipLaunchKernelGGL(peak_mfma_bf16, dim3(nblk), dim3(256), 0, nullptr, out, iters, 1e-3f, 2e-3f); }, 5, &ms);
        work = double(nblk) * 4 * 4 * iters * (32.0 * 32 * 16 * 2);
        break;
    case S2_PEAK_LDS_READ:
        rc = timed([&] { hipLaunchKernelGGL(peak_lds, dim3(nblk), dim3(256), 0, nullptr, out, iters); }, 5, &ms);
        work = double(nblk) * 256 * 16 * iters * 16;
        break;
    default:
        (void)hipFree(out);
        return s2_fail(S2_ERR_INVALID_ARG, "unknown kind of peak");
    }
    (void)hipFree(out);
    if (rc || hipGetLastError() != hipSuccess) return s2_fail(S2_ERR_DEVICE, "timing the peak kernel failed");
    *value = work / (ms * 1e-3) / 1e12;          // TFLOP/s (TB/s for the LDS reads)
    return S2_OK;
}
