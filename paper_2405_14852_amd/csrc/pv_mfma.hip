// Matrix-core nearest-codeword search (placeholder until the filter lands).
#include "pv_internal.h"

bool pv_mfma_supported(const pv_layout *) { return false; }

pv_status pv_launch_mfma_search(pv_ctx *ctx, const pv_layout *, const float *, const float *,
                                const float *, const int32_t *, int64_t, uint16_t *, int64_t *)
{
    return pv_fail(ctx, PV_ERR_UNSUPPORTED, "matrix-core search not built");
}
