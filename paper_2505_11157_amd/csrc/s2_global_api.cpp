// C entry points of the global attention (placeholder until the MFMA kernels land).
#include "s2_internal.h"

extern "C" size_t s2_attn_global_bwd_workspace_bytes(const s2_grid_t *g, int batch, int heads, int d, int dtype)
{
    (void)g; (void)batch; (void)heads; (void)d; (void)dtype;
    return 0;
}

extern "C" int s2_attn_global_fwd(const s2_grid_t *, int, int, int, int, float, const void *, const void *,
                                  const void *, void *, float *, void *)
{
    return s2_fail(S2_ERR_UNSUPPORTED, "global attention is not built yet");
}

extern "C" int s2_attn_global_bwd(const s2_grid_t *, int, int, int, int, float, const void *, const void *,
                                  const void *, const void *, const float *, const void *, void *, void *, void *,
                                  void *, size_t, void *)
{
    return s2_fail(S2_ERR_UNSUPPORTED, "global attention is not built yet");
}
