// Launchers of the neighborhood-attention kernels (internal).
#pragma once
#include "s2_internal.h"

// Shape-agnostic float32 path: 1 <= d, e <= 128.
int s2_nattn_fwd_generic(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q,
                         const float *k, const float *v, float *out, float *lse, hipStream_t st);
int s2_nattn_bwd_generic(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q,
                         const float *k, const float *v, const float *o, const float *lse, const float *go,
                         float *dq, float *dk, float *dv, float *Dws, hipStream_t st);

// dk, dv of an input latitude of weight zero are zero: x is [rows][nlat_in][nlon_in], rows = slices * channels,
// float32 or bf16 elements.
void s2_nattn_zero_latitude(const S2DeviceTables &t, int lat, int rows, void *x, bool bf16, hipStream_t st);

// Shape-agnostic path on bf16 tensors (float32 arithmetic, float32 lse and D).
int s2_nattn_fwd_generic_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q, const void *k,
                              const void *v, void *out, float *lse, hipStream_t st);
int s2_nattn_bwd_dq_generic_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q,
                                 const void *k, const void *v, const void *o, const float *lse, const void *go, void *dq,
                                 float *Dws, hipStream_t st);
int s2_nattn_bwd_dkdv_generic_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q,
                                   const void *k, const void *v, const float *lse, const void *go, const float *Dws,
                                   void *dk, void *dv, hipStream_t st);

// Tuned float32 forward for d = e = 32, nlon_in / nlon_out in {1, 2}, longitudes a multiple of 4.
bool s2_nattn_fwd_tiled_supported(const S2DeviceTables &t, int d, int e);
int s2_nattn_fwd_tiled(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q, const float *k,
                       const float *v, float *out, float *lse, hipStream_t st);

// dk/dv part of the shape-agnostic backward alone (D_i must already be in Dws).
int s2_nattn_bwd_dkdv_generic(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q,
                              const float *k, const float *v, const float *lse, const float *go, const float *Dws,
                              float *dk, float *dv, hipStream_t st);
// Tuned float32 backward for d = e = 32 (dq for nlon_in / nlon_out in {1, 2}; dk/dv tuned on equal grids).
bool s2_nattn_bwd_tiled_supported(const S2DeviceTables &t, int d, int e);
int s2_nattn_bwd_tiled(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q, const float *k,
                       const float *v, const float *o, const float *lse, const float *go, float *dq, float *dk,
                       float *dv, float *Dws, hipStream_t st);

// Forward on the fp32 matrix cores for the heaviest output latitudes (dense neighborhoods near the
// poles): number of leading latitudes of row_order it takes (0 if the shape does not qualify), and the launch.
int s2_nattn_fwd_mfma_rows(const S2DeviceTables &t, int d, int e);
int s2_nattn_fwd_mfma(const S2DeviceTables &t, int nbh, int nrows, float scale, const float *q, const float *k,
                      const float *v, float *out, float *lse, hipStream_t st);
int s2_nattn_bwd_dq_mfma(const S2DeviceTables &t, int nbh, int nrows, float scale, const float *q, const float *k,
                         const float *v, const float *o, const float *lse, const float *go, float *dq, float *Dws,
                         hipStream_t st);
int s2_nattn_bwd_dkdv_mfma_rows(const S2DeviceTables &t, int d, int e);
int s2_nattn_bwd_dkdv_mfma(const S2DeviceTables &t, int nbh, int nrows, float scale, const float *q, const float *k,
                           const float *v, const float *lse, const float *go, const float *Dws, float *dk, float *dv,
                           hipStream_t st);

// Streaming kernels for the light latitudes (last class) on equal grids: each input latitude is staged in LDS once
// per workgroup and shared by the wavefronts that walk down consecutive output latitudes.
bool s2_nattn_stream_supported(const S2DeviceTables &t, int d, int e);
int s2_nattn_fwd_stream(const S2DeviceTables &t, int nbh, float qscale, const float *q, const float *k,
                        const float *v, float *out, float *lse, hipStream_t st);
bool s2_nattn_stream_dq_supported(const S2DeviceTables &t, int d, int e);
bool s2_nattn_stream_dkdv_supported(const S2DeviceTables &t, int d, int e);
int s2_nattn_bwd_dq_stream(const S2DeviceTables &t, int nbh, float scale, const float *q, const float *k,
                           const float *v, const float *o, const float *lse, const float *go, float *dq, float *Dws,
                           hipStream_t st);
int s2_nattn_bwd_dkdv_stream(const S2DeviceTables &t, int nbh, float scale, const float *q, const float *k,
                             const float *v, const float *lse, const float *go, const float *Dws, float *dk, float *dv,
                             hipStream_t st);

// bf16 tensors on the bf16 matrix cores (band tiles of 16 keys x 16 outputs, float32 softmax and accumulation): equal
// grids, d = e = 32, longitude count a multiple of 64.
bool s2_nattn_bf16_supported(const S2DeviceTables &t, int d, int e);
int s2_nattn_fwd_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q, const void *k,
                      const void *v, void *out, float *lse, hipStream_t st);
int s2_nattn_bwd_dq_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q, const void *k,
                         const void *v, const void *o, const float *lse, const void *go, void *dq, float *Dws,
                         hipStream_t st);
int s2_nattn_bwd_dkdv_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q, const void *k,
                           const void *v, const float *lse, const void *go, const float *Dws, void *dk, void *dv,
                           hipStream_t st);

// float32 tensors on the fp32 matrix cores (band tiles of 16 keys x 16 outputs) for head dimensions the hand-tuned
// kernels do not cover: equal grids, d = e in {16, 32, 64}, longitude count a multiple of 16 (at least 64).
bool s2_nattn_band_supported(const S2DeviceTables &t, int d, int e);
int s2_nattn_fwd_band(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q, const float *k,
                      const float *v, float *out, float *lse, hipStream_t st);
int s2_nattn_bwd_band(const S2DeviceTables &t, int nbh, int d, int e, float scale, const float *q, const float *k,
                      const float *v, const float *o, const float *lse, const float *go, float *dq, float *dk, float *dv,
                      float *Dws, hipStream_t st);

// The same kernels on bf16 tensors (float32 arithmetic on the fp32 matrix cores, bf16 loads and stores): the head
// dimensions and longitude counts the bf16 matrix-core kernels do not cover.
int s2_nattn_fwd_band_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q, const void *k,
                           const void *v, void *out, float *lse, hipStream_t st);
int s2_nattn_bwd_dq_band_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q, const void *k,
                              const void *v, const void *o, const float *lse, const void *go, void *dq, float *Dws,
                              hipStream_t st);
int s2_nattn_bwd_dkdv_band_bf16(const S2DeviceTables &t, int nbh, int d, int e, float scale, const void *q, const void *k,
                                const void *v, const float *lse, const void *go, const float *Dws, void *dk, void *dv,
                                hipStream_t st);

// Backward with the scratch for D_i given as a device pointer (checks and dispatch behind both C entry points).
int s2_nattn_bwd_run(const s2_grid_t *g, int batch, int heads, int d_qk, int d_v, int dtype, float scale,
                     const void *q, const void *k, const void *v, const void *out, const float *lse, const void *dout,
                     void *dq, void *dk, void *dv, float *Dws, hipStream_t st);

// Per-device set-up of the static scratch array behind s2_nattn_bwd_static (the device must be current).
int s2_static_scratch_setup(int device);
