// Internal declarations shared by the translation units of libconserve_kv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "conserve_kv.h"

namespace cs {

constexpr int kPage = CS_PAGE_SIZE;          // tokens per page
constexpr int kMaxGroup = 16;                // query heads per kv head that fit one MFMA tile

// Records a failed HIP call for cs_last_hip_error(); returns CS_ERR_HIP.
int hip_failed(hipError_t e, const char* what);

inline int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? CS_OK : hip_failed(e, what);
}

// Host-side checks common to every entry point.  Return CS_OK or the error.
int validate_pool(const cs_kv_pool* pool);
int validate_batch(const cs_kv_pool* pool, const cs_batch* batch);

// Plan of the decode path, a pure function of the host lengths (used by both the
// workspace query and the launch).
struct DecodePlan {
    int32_t num_decode;        // sequences with exactly one new token
    int32_t num_prefill;       // sequences with more than one new token
    int32_t max_decode_keys;   // max over decode sequences of ctx + 1
    int32_t split_tokens;      // keys per split (multiple of 16)
    int32_t max_splits;        // ceil(max_decode_keys / split_tokens)
    int64_t decode_keys;       // total keys read by decode sequences
};
DecodePlan plan_decode(const cs_batch* batch, int32_t num_kv_heads);
size_t decode_workspace_bytes(const DecodePlan& p, int32_t num_seqs, int32_t num_q_heads, int32_t head_dim);

// Kernel launchers (defined next to their kernels).
int launch_append(const cs_kv_pool& pool, int32_t layer, const cs_batch& b,
                  const void* k_new, const void* v_new, hipStream_t st);
int launch_page_copy(const cs_kv_pool& pool, int32_t layer_begin, int32_t layer_end,
                     const int32_t* ids, int32_t n, void* staging, bool to_staging, hipStream_t st);
int launch_plain_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
int launch_decode(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& plan,
                  const void* q, void* out, int32_t Hq, float scale, void* workspace, hipStream_t st);
int launch_prefill(const cs_kv_pool& pool, int32_t layer, const cs_batch& b,
                   const void* q, void* out, int32_t Hq, float scale, hipStream_t st);

}  // namespace cs
