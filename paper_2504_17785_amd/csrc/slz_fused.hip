// placeholder until the fused kernel lands
#include "slz_internal.h"
int slz_fused_supported(const slz_params *) { return 0; }
int slz_fused_init(slz_ctx *) { return SLZ_E_UNSUPPORTED; }
void slz_fused_destroy(slz_ctx *) {}
int slz_fused_blind_rotate(slz_ctx *, const uint64_t *, const uint64_t *, const uint32_t *, const double *, uint32_t, uint64_t *,
                           uint64_t *, uint32_t, hipStream_t) { return SLZ_E_UNSUPPORTED; }
