// es_rollout, register-resident MFMA variant (placeholder until the kernel lands).
#include "es_internal.hpp"

namespace es {

int mfma_variant_for(const es_config&) { return -1; }
const char* mfma_variant_name(int) { return "none"; }
int launch_rollout_mfma(es_ctx* ctx, uint32_t, const float*, const void*, const float*, const float*, float*,
                        int32_t*, float*, void*, hipStream_t) {
  return fail(ctx, ES_EUNSUPPORTED, "es_rollout: MFMA variant not built");
}

}  // namespace es
