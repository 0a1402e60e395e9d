// Prefill-chunk path (placeholder until the MFMA tile kernel lands).
#include "cs_common.h"
namespace cs {
int launch_prefill(const cs_kv_pool&, int32_t, const cs_batch&, const void*, void*, int32_t, float, hipStream_t) {
    return CS_ERR_UNSUPPORTED;
}
}
