// cs_paged_attention_mixed_static: the attention call for callers that cannot allocate device
// memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
// The workspace of cs_paged_attention_mixed -- the decode work-item list and the fp32 partial
// results of cut decode sequences and of prefill tiles cut into key ranges -- comes from one
// file-scope device array instead of the caller.  Each device the library runs on holds its own
// copy of the array, at its own address, until the process ends.
#include <atomic>
#include "cs_common.h"

// In host code this name is only a handle for hipGetSymbolAddress: it is NOT a device address.
// Kernels, memsets and copies take the per-device pointer that call returns.
static __device__ __align__(256) unsigned char scratch[CS_STATIC_SCRATCH_BYTES];

namespace cs {

constexpr int kScratchDevices = 64;
static std::atomic<void*> g_scratch_ptr[kScratchDevices];

// Device address of `scratch` on the CURRENT device, looked up on the first call there.
static int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_failed(e, "hipGetDevice");
    if (dev < 0 || dev >= kScratchDevices) return CS_ERR_UNSUPPORTED;
    void* p = g_scratch_ptr[dev].load();
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_failed(e, "hipGetSymbolAddress(scratch)");
        if (!p) return CS_ERR_HIP;
        g_scratch_ptr[dev].store(p);
    }
    *out = p;
    return CS_OK;
}

}  // namespace cs

extern "C" {

size_t cs_static_scratch_bytes(void) { return CS_STATIC_SCRATCH_BYTES; }

int cs_paged_attention_mixed_static(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                                    const void* q, void* out, int32_t num_q_heads, float softmax_scale,
                                    void* stream)
{
    // The size check comes first: a batch whose plan does not fit is refused before anything else
    // happens.  (A zero from the query also covers bad arguments; the call below reports those.)
    size_t need = 0;
    if (pool && batch)
        need = cs_paged_attention_workspace_bytes(batch, num_q_heads, pool->num_kv_heads, pool->head_dim);
    if (need > (size_t)CS_STATIC_SCRATCH_BYTES) return CS_ERR_STATIC_SCRATCH_TOO_SMALL;
    void* ws = nullptr;
    if (need > 0) {
        const int rc = cs::static_scratch(&ws);
        if (rc) return rc;
    }
    // Nothing in the scratch has to start at zero: every word a kernel of this call reads (item
    // list, partial maxima, sums and outputs) is written earlier in the same call, on the same
    // stream.  So there is no clearing, and what the previous call left is simply overwritten.
    return cs_paged_attention_mixed(pool, layer, batch, q, out, num_q_heads, softmax_scale,
                                    ws, need > 0 ? (size_t)CS_STATIC_SCRATCH_BYTES : 0, stream);
}

}  // extern "C"
