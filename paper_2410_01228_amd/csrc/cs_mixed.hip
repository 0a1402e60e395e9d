// Fused kernel for a mixed batch (paper Sec. 4.2: online decode tokens and offline prefill
// chunks share an iteration).  The prefill workgroups and the decode work items are one grid:
// the prefill tiles, bound by the matrix cores and of uneven length, come first; the decode
// items, bound by HBM and sorted longest first, follow and move into every slot a finished or
// missing prefill tile leaves free -- two kernels in a row would leave those slots idle until
// the longest tile is done.  Both kinds of workgroup have 4 wavefronts and share one LDS
// allocation (a union of the two layouts), so two of them fit a CU in any combination; the
// decode items take the deeper page prefetch, whose registers cost nothing here.  kPhasePriority
// (see prefill_tile) is set by the host when the decode side is the small one.
#include "cs_prefill_impl.h"
#include "cs_decode_impl.h"

namespace cs {

static_assert(kPrefillThreads == kDecodeThreads, "one block size for both kinds of workgroup");

template <int D>
union MixedLds {
    PrefillLds<D> prefill;
    DecodeLds<D> decode;
};

template <int D, class E, bool kPhasePriority, int PS>
__global__ __launch_bounds__(kPrefillThreads, 2) void mixed_kernel(
    const uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t G, int32_t S,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float scale_log2e,
    int32_t range_steps, int32_t base_slot, int32_t max_ranges, float* __restrict__ prefill_part,
    uint32_t wgs_per_range, uint32_t num_prefill_wgs, int32_t backwards, const ItemsInArgs items,
    float* __restrict__ part_o, float* __restrict__ part_ml)
{
    __shared__ MixedLds<D> lds;
    if (blockIdx.x < num_prefill_wgs) {
        // range-major, like the prefill kernel's own grid: all tiles of key range 0, then range 1, ...
        const uint32_t range = blockIdx.x / wgs_per_range, rem = blockIdx.x - range * wgs_per_range;
        const int32_t pos = rem / Hkv;
        const int32_t g = rem - pos * Hkv;
        const int32_t b = backwards ? (int32_t)(wgs_per_range / Hkv) - 1 - pos : pos;   // longest tiles first
        prefill_tile<D, E, kPhasePriority, PS, true>(lds.prefill, layer_base, page_stride, num_pages, Hkv, G, S, block_tables, max_blocks,
                           ctx_lens, cu_q_lens, q, out, scale_log2e, range_steps, base_slot, prefill_part, g, b,
                           (int32_t)range, max_ranges);
    } else {
        const uint32_t w = blockIdx.x - num_prefill_wgs;
        const int32_t item = w / Hkv, g = w - item * Hkv;
        decode_item<D, ItemsInArgs, E, 2, PS>(lds.decode, layer_base, page_stride, num_pages, Hkv, G, block_tables, max_blocks,
                                       items, ctx_lens, cu_q_lens, q, out, scale_log2e, part_o, part_ml, item, g);
    }
}

template <class E>
static int launch_mixed_as(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& dplan,
                           const PrefillPlan& pplan, const void* q, void* out, int32_t Hq, float scale,
                           void* decode_ws, void* prefill_ws, hipStream_t st, bool prio)
{
    const int32_t Hkv = pool.num_kv_heads, D = pool.head_dim, G = Hq / Hkv;
    const uint16_t* layer_base = (const uint16_t*)pool.base + (int64_t)layer * pool.layer_stride;
    const float scale_log2e = scale * 1.4426950408889634f;
    const int64_t slots = prefill_slot_start(b.num_tokens, b.num_seqs, G);
    const int64_t per_range = slots * Hkv;
    const int64_t n_prefill = per_range * pplan.max_ranges, n_decode = (int64_t)dplan.total_items * Hkv;
    if (n_prefill + n_decode > 2147483647ll) return CS_ERR_UNSUPPORTED;
    const DecodeWorkspace w = decode_workspace(dplan, b.num_seqs, Hq, D);
    float* part_ml = (float*)((char*)decode_ws + w.part_ml);
    float* part_o = (float*)((char*)decode_ws + w.part_o);
    dim3 grid((uint32_t)(n_prefill + n_decode));
#define CS_LAUNCH_MIXED_P(DD, PRIO, PS)                                                                      \
    hipLaunchKernelGGL((mixed_kernel<DD, E, PRIO, PS>), grid, dim3(kPrefillThreads), 0, st, layer_base, pool.page_stride, \
                       pool.num_pages, Hkv, G, b.num_seqs, b.block_tables, b.max_blocks_per_seq, b.ctx_lens,    \
                       b.cu_q_lens, (const uint16_t*)q, (uint16_t*)out, scale_log2e, pplan.range_steps,         \
                       pplan.base_slot, pplan.max_ranges, (float*)prefill_ws, (uint32_t)per_range,              \
                       (uint32_t)n_prefill, (int32_t)pplan.backwards, dplan.arg_items, part_o, part_ml);
#define CS_LAUNCH_MIXED(DD, PRIO)                                                                            \
    if (pool.page_size == 16) { CS_LAUNCH_MIXED_P(DD, PRIO, 16) } else { CS_LAUNCH_MIXED_P(DD, PRIO, 8) }
    if (D == 128) { if (prio) { CS_LAUNCH_MIXED(128, true) } else { CS_LAUNCH_MIXED(128, false) } }
    else          { if (prio) { CS_LAUNCH_MIXED(64, true) } else { CS_LAUNCH_MIXED(64, false) } }
#undef CS_LAUNCH_MIXED
#undef CS_LAUNCH_MIXED_P
    return check_launch("mixed kernel");
}

int launch_mixed(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& dplan,
                 const PrefillPlan& pplan, const void* q, void* out, int32_t Hq, float scale,
                 void* decode_ws, void* prefill_ws, hipStream_t st, bool f16, bool prio)
{
    return f16 ? launch_mixed_as<F16>(pool, layer, b, dplan, pplan, q, out, Hq, scale, decode_ws, prefill_ws, st, prio)
               : launch_mixed_as<Bf16>(pool, layer, b, dplan, pplan, q, out, Hq, scale, decode_ws, prefill_ws, st, prio);
}

}  // namespace cs
