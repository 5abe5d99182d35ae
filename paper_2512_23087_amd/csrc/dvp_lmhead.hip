// Fused LM-head variant (placeholder until the MFMA kernels land).
#include "dvp_internal.h"

extern "C" {

size_t dvp_fused_lmhead_workspace_bytes(const dvp_lmhead_params *) { return 0; }

dvp_status dvp_fused_lmhead(const dvp_lmhead_params *, const void *, const void *, const void *,
                            const int64_t *, const float *, const dvp_side_out *,
                            const dvp_side_out *, uint8_t *, float *, float *, void *, size_t, void *)
{
    return DVP_ERR_UNSUPPORTED;
}

}
