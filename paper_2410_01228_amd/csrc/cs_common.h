// Internal declarations shared by the translation units of libconserve_kv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "conserve_kv.h"

namespace cs {

constexpr int kPage = CS_PAGE_SIZE;          // keys per step of the decode path; also the default page size
// Pages hold 16 tokens (the paper's granularity, Sec. 5) or 8; the attention kernels are
// instantiated for each and walk the keys 16 (decode) or 32 (prefill) at a time either way.
inline bool page_size_supported(int32_t ps) { return ps == 16 || ps == 8; }
inline size_t pool_page_bytes(const cs_kv_pool& p) { return (size_t)2 * p.num_kv_heads * p.page_size * p.head_dim * 2; }
constexpr int kMaxGroup = 16;                // query heads per kv head that fit one MFMA tile

// Records a failed HIP call for cs_last_hip_error(); returns CS_ERR_HIP.
int hip_failed(hipError_t e, const char* what);

inline int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? CS_OK : hip_failed(e, what);
}

// Compute units of the current device (memoised per device; 256 where no device answers, and
// whatever cs_debug_set_cu_count forces).  The launch plans size their grids by it.
int32_t device_cus();

// Host-side checks common to every entry point.  Return CS_OK or the error.
int validate_pool(const cs_kv_pool* pool);
int validate_batch(const cs_kv_pool* pool, const cs_batch* batch);

// Split arithmetic of the decode path, shared by the host plan and the kernels.  A decode
// sequence with n keys is cut into round(n / split) pieces (at least one) of equal,
// page-aligned length, so no piece is a sliver.
__host__ __device__ inline int32_t decode_num_splits(int32_t n_keys, int32_t split) {
    const int32_t k = (n_keys + split / 2) / split;
    return k < 1 ? 1 : k;
}
__host__ __device__ inline int32_t decode_chunk_keys(int32_t n_keys, int32_t n_splits) {
    const int32_t c = (n_keys + n_splits - 1) / n_splits;
    return (c + kPage - 1) & ~(kPage - 1);
}

// Tile arithmetic of the prefill path, shared by the host plan and the kernels.
constexpr int kPrefillWaves = 4;
constexpr int kPrefillThreads = kPrefillWaves * 64;
constexpr int kNCT = 2;                       // column tiles (16 query rows) per wavefront
constexpr int kKeysPerStep = 32;              // keys a workgroup walks per step: two pages of 16
constexpr int kTileCols = kPrefillWaves * kNCT;   // column tiles per workgroup

// Workgroup slots.  A sequence with q new tokens has ceil(q/16) * G column tiles, numbered
// token-block major (ct = token_block * G + head), and needs ceil(that / kTileCols)
// workgroups.  Slots are dealt without a prefix sum over tile counts: sequence s starts at
//   start(s) = floor((cu_q_lens[s] + 16 s) * G / (16 * kTileCols)) + s,
// which is strictly increasing and leaves every sequence at least as many slots as it needs.
__host__ __device__ inline int64_t prefill_slot_start(int32_t cu_q, int32_t s, int32_t G) {
    return ((int64_t)cu_q + 16ll * s) * G / (16 * kTileCols) + s;
}

// Small batches carry their work-item list inside the kernel arguments: the host already has
// the lengths, so it lists the items itself, longest first, and no planning kernel and no
// host-to-device copy is needed.  One word per item: sequence (bits 0-15), piece (16-23),
// pieces of that sequence (24-31).  One word per cut sequence for the merge: sequence (bits
// 0-15), its first item (16-31).  The list must fit the 4 KiB argument block of a launch.
constexpr int kMaxArgItems = 880;
struct ItemsInArgs { uint32_t e[kMaxArgItems]; };

// Plan of the decode path, a pure function of the host lengths (used by both the
// workspace query and the launch).
struct DecodePlan {
    int32_t num_decode;        // sequences with exactly one new token
    int32_t num_prefill;       // sequences with more than one new token
    int32_t split_tokens;      // target keys per work item (multiple of 16)
    int32_t total_items;       // sum over decode sequences of their split count
    int32_t num_multi;         // decode sequences cut into more than one item
    int64_t decode_keys;       // total keys read by decode sequences
    int32_t pages_ahead;       // pages a wavefront of the decode kernel prefetches (1 or 2)
    bool    in_args;           // the item list below is valid and replaces the planning kernel
    ItemsInArgs arg_items;     // total_items words
    ItemsInArgs arg_multi;     // num_multi words
};
DecodePlan plan_decode(const cs_batch* batch, int32_t num_kv_heads, int32_t head_dim);
// Workspace layout (all 16-byte aligned): work items | per-sequence item offsets |
// multi-item sequence list | partial (max, sum) | partial outputs.
struct DecodeWorkspace {
    size_t items, cu_items, multi, part_ml, part_o, total;
};
DecodeWorkspace decode_workspace(const DecodePlan& p, int32_t num_seqs, int32_t num_q_heads, int32_t head_dim);

// Kernel launchers (defined next to their kernels).
int launch_append(const cs_kv_pool& pool, int32_t layer, const cs_batch& b,
                  const void* k_new, const void* v_new, hipStream_t st);
int launch_page_copy(const cs_kv_pool& pool, int32_t layer_begin, int32_t layer_end,
                     const int32_t* ids, int32_t n, void* staging, bool to_staging, hipStream_t st,
                     bool page_major = false);
int launch_token_copy(const cs_kv_pool& pool, int32_t layer_begin, int32_t layer_end,
                      const int32_t* token_slots, int32_t n, void* staging, bool to_staging, hipStream_t st);
int launch_plain_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
// f16: the pool, q and out hold IEEE half instead of bf16.
// merge_only: the items' work has been done already (by the fused kernel below); only the
// partials of the cut sequences remain to be merged.  Valid when plan.in_args.
int launch_decode(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& plan,
                  const void* q, void* out, int32_t Hq, float scale, void* workspace, hipStream_t st, bool f16,
                  bool merge_only = false);
// Key-range split of the prefill path (pure function of the host lengths).
// Slot each grid position takes when the host reorders the tiles (see plan_prefill).
constexpr int kMaxSlotOrder = 512;
struct SlotOrder { uint16_t slot[kMaxSlotOrder]; };
struct PrefillPlan {
    int32_t n_ordered;         // > 0: the grid has n_ordered slot positions, position p takes slot order.slot[p]
    SlotOrder order;
    bool    backwards;         // where no table is used: grid position p takes slot (slots - 1 - p)
    int32_t range_steps;       // 32-key steps per key range (>= the longest tile: no split)
    int32_t max_ranges;        // grid depth: ranges of the longest tile
    int32_t cut_first_pos;     // launch positions from this one on are cut (the fused grid's tail; 0: every tile longer than range_steps)
    int32_t base_slot;         // first workgroup slot that can belong to a prefill sequence (set whenever there is a chunk)
    int32_t num_slots;         // slots from base_slot on: the grid's extent; partials are indexed by slot - base_slot
    size_t  bytes;             // workspace for the partials (0 when nothing is cut)
};
PrefillPlan plan_prefill(const cs_batch* batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim);
int launch_prefill(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const PrefillPlan& plan,
                   const void* q, void* out, int32_t Hq, float scale, void* workspace, hipStream_t st, bool f16);
// The merge of the key-range partials alone (what launch_prefill ends with when tiles are cut).
int launch_prefill_merge(const cs_kv_pool& pool, const cs_batch& b, const PrefillPlan& plan, void* out, int32_t Hq,
                         void* workspace, hipStream_t st, bool f16);
// One launch for a batch that holds both chunks and decode tokens.  persistent_wgs == 0: the
// prefill workgroups first, one workgroup per decode (item, kv head) pair behind them, so that
// decode work fills the slots the uneven prefill tiles leave empty instead of waiting for the
// last of them.  persistent_wgs > 0: that many decode workgroups first (the host passes the CU
// count: one per CU), each walking several pairs, the tiles beside them.  Needs the item list
// in the kernel arguments (dplan.in_args).  Tiles cut into key ranges bring one workgroup per
// range; the caller merges their partials (launch_prefill_merge) and the cut decode sequences
// (launch_decode with merge_only) afterwards.  tile_priority: 0, or the higher of the two issue
// priorities the tile wavefronts alternate between (1 or 2; decode wavefronts stay at 0).
int launch_mixed(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& dplan,
                 const PrefillPlan& pplan, const void* q, void* out, int32_t Hq, float scale,
                 void* decode_workspace_base, void* prefill_workspace, hipStream_t st, bool f16,
                 int32_t tile_priority, int32_t persistent_wgs);

}  // namespace cs
