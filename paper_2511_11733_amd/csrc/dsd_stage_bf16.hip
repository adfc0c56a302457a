// bf16 MFMA path of the verification pass (placeholder until the kernels land).
#include "dsd_internal.h"

int mfma_supported(const dsd_model_desc*) { return 0; }
int mfma_weights_tile(dsd_ctx*, dsd_weights*, const void* const*) { DSD_FAIL(DSD_EUNSUPPORTED, "bf16 MFMA path not built"); }
int mfma_stage_verify(dsd_ctx*, const dsd_weights*, dsd_kv*, const void*, const int32_t*, const uint64_t*,
                      const int32_t*, int, int, void*, float*, int64_t) {
    DSD_FAIL(DSD_EUNSUPPORTED, "bf16 MFMA path not built");
}
