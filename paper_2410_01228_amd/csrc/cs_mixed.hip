// Fused kernel for a mixed batch (paper Sec. 4.2: online decode tokens and offline prefill
// chunks share an iteration).  The prefill tile-workgroups (bound by the matrix cores, of uneven
// length) and the decode work (bound by HBM) are one grid, in one of two arrangements the host
// picks from the batch's lengths:
//  - decode beside the tiles: min(CUs, pairs) decode workgroups come FIRST in the grid, one per
//    CU, and each walks several (work item, kv head) pairs in a row; the tiles take the other
//    workgroup slot of every CU and, once the decode workgroups retire, both.  The matrix pipe
//    and HBM are then busy at the same time for as long as the decode side lasts;
//  - decode behind the tiles: one workgroup per pair after the last tile; the pairs move into
//    every slot a finished or missing tile leaves free (two kernels in a row would leave those
//    slots idle until the longest tile is done).  Better when the decode side is small: it does
//    not hold a slot per CU while the tiles need both.
// Both kinds of workgroup have 4 wavefronts and share one LDS allocation (a union of the two
// layouts), so two of them fit a CU in any combination.  kPriority (see prefill_tile) is
// chosen by the host: 1 or 2 beside the tiles, 1 behind them when the decode side is the small one.
#include "cs_prefill_impl.h"
#include "cs_decode_impl.h"

namespace cs {

static_assert(kPrefillThreads == kDecodeThreads, "one block size for both kinds of workgroup");

template <int D>
union MixedLds {
    PrefillLds<D> prefill;
    DecodeLds<D> decode;
};

// Workgroups [dec_first, dec_first + dec_wgs) are decode workgroups, the others tiles (numbered
// without the gap).  Tiles, in launch positions from tile slot base_slot on: first the whole
// tiles of positions 0 .. cut_first_pos-1, then, range-major like the prefill kernel's own grid,
// the key ranges of the positions behind them (cut_first_pos == 0: every tile longer than
// range_steps is cut; == num_slots with max_ranges == 1: none is).  Decode workgroup j takes the pairs j, 2*dec_wgs-1-j, 2*dec_wgs+j, ... of the
// n_decode (item, kv head) pairs: the items are sorted longest first, so walking the rounds back
// and forth evens the sums; with dec_wgs == n_decode that is one pair each.
template <int D, class E, int kPriority, int PS>
__global__ __launch_bounds__(kPrefillThreads, 2) void mixed_kernel(
    const uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t G, int32_t S,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float scale_log2e,
    int32_t range_steps, int32_t base_slot, int32_t num_slots, int32_t cut_first_pos, int32_t max_ranges,
    float* __restrict__ prefill_part, uint32_t dec_first, uint32_t dec_wgs, uint32_t n_decode, int32_t backwards,
    const ItemsInArgs items, float* __restrict__ part_o, float* __restrict__ part_ml)
{
    __shared__ MixedLds<D> lds;
    if (blockIdx.x < dec_first || blockIdx.x >= dec_first + dec_wgs) {
        const uint32_t ti = blockIdx.x < dec_first ? blockIdx.x : blockIdx.x - dec_wgs;
        const uint32_t wgs_whole = (uint32_t)cut_first_pos * Hkv, wgs_per_range = (uint32_t)(num_slots - cut_first_pos) * Hkv;
        // a whole tile: one range longer than any tile (and small enough to add a tile's steps to)
        int32_t pos, g, range = 0, steps_per_range = 1 << 30;
        float* part_tile = nullptr;
        if (ti < wgs_whole) {
            pos = ti / Hkv;
            g = ti - pos * Hkv;
        } else {
            const uint32_t u = ti - wgs_whole;
            range = u / wgs_per_range;
            const uint32_t rem = u - range * wgs_per_range;
            pos = cut_first_pos + rem / Hkv;
            g = rem - (rem / Hkv) * Hkv;
            steps_per_range = range_steps;
            part_tile = partials_of<D>(prefill_part, pos - cut_first_pos, Hkv, g, max_ranges);
        }
        const int32_t b = base_slot + (backwards ? num_slots - 1 - pos : pos);   // backwards: longest tiles first
        prefill_tile<D, E, kPriority, PS, true>(lds.prefill, layer_base, page_stride, num_pages, Hkv, G, S, block_tables, max_blocks,
                           ctx_lens, cu_q_lens, q, out, scale_log2e, steps_per_range, part_tile, g, b, range);
    } else {
        const uint32_t j = blockIdx.x - dec_first;
        for (uint32_t base = 0, round = 0; base < n_decode; base += dec_wgs, ++round) {
            const uint32_t w = base + ((round & 1) ? dec_wgs - 1 - j : j);
            if (w >= n_decode) continue;
            const int32_t item = w / Hkv, g = w - item * Hkv;
            // one page ahead, with loads the compiler can count (a workgroup that shares its CU
            // with a tile must stream by itself); a deeper queue only delays the tile's own
            // copies, which share the CU's memory pipeline
            decode_item<D, ItemsInArgs, E, 1, PS, true>(lds.decode, layer_base, page_stride, num_pages, Hkv, G, block_tables, max_blocks,
                                           items, ctx_lens, cu_q_lens, q, out, scale_log2e, part_o, part_ml, item, g);
            __syncthreads();     // the next pair reuses the merge buffers
        }
    }
}

template <class E>
static int launch_mixed_as(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& dplan,
                           const PrefillPlan& pplan, const void* q, void* out, int32_t Hq, float scale,
                           void* decode_ws, void* prefill_ws, hipStream_t st, int32_t prio, int32_t persistent_wgs)
{
    const int32_t Hkv = pool.num_kv_heads, D = pool.head_dim, G = Hq / Hkv;
    const uint16_t* layer_base = (const uint16_t*)pool.base + (int64_t)layer * pool.layer_stride;
    const float scale_log2e = scale * 1.4426950408889634f;
    const int64_t n_prefill = ((int64_t)pplan.cut_first_pos + (int64_t)(pplan.num_slots - pplan.cut_first_pos) * pplan.max_ranges) * Hkv;
    const int64_t n_decode = (int64_t)dplan.total_items * Hkv;
    // decode beside the tiles: a few workgroups first; behind the tiles: one per pair, last
    const int64_t dec_wgs = persistent_wgs > 0 ? std::min<int64_t>(persistent_wgs, n_decode) : n_decode;
    const int64_t dec_first = persistent_wgs > 0 ? 0 : n_prefill;
    if (n_prefill + dec_wgs > 2147483647ll) return CS_ERR_UNSUPPORTED;
    const DecodeWorkspace w = decode_workspace(dplan, b.num_seqs, Hq, D);
    float* part_ml = (float*)((char*)decode_ws + w.part_ml);
    float* part_o = (float*)((char*)decode_ws + w.part_o);
    dim3 grid((uint32_t)(n_prefill + dec_wgs));
#define CS_LAUNCH_MIXED_P(DD, PRIO, PS)                                                                      \
    hipLaunchKernelGGL((mixed_kernel<DD, E, PRIO, PS>), grid, dim3(kPrefillThreads), 0, st, layer_base, pool.page_stride, \
                       pool.num_pages, Hkv, G, b.num_seqs, b.block_tables, b.max_blocks_per_seq, b.ctx_lens,    \
                       b.cu_q_lens, (const uint16_t*)q, (uint16_t*)out, scale_log2e, pplan.range_steps,         \
                       pplan.base_slot, pplan.num_slots, pplan.cut_first_pos, pplan.max_ranges,                 \
                       (float*)prefill_ws, (uint32_t)dec_first, (uint32_t)dec_wgs, (uint32_t)n_decode, (int32_t)pplan.backwards,    \
                       dplan.arg_items, part_o, part_ml);
#define CS_LAUNCH_MIXED(DD, PRIO)                                                                            \
    if (pool.page_size == 16) { CS_LAUNCH_MIXED_P(DD, PRIO, 16) } else { CS_LAUNCH_MIXED_P(DD, PRIO, 8) }
    if (D == 128) { if (prio == 2) { CS_LAUNCH_MIXED(128, 2) } else if (prio == 1) { CS_LAUNCH_MIXED(128, 1) } else { CS_LAUNCH_MIXED(128, 0) } }
    else          { if (prio == 2) { CS_LAUNCH_MIXED(64, 2) } else if (prio == 1) { CS_LAUNCH_MIXED(64, 1) } else { CS_LAUNCH_MIXED(64, 0) } }
#undef CS_LAUNCH_MIXED
#undef CS_LAUNCH_MIXED_P
    return check_launch("mixed kernel");
}

int launch_mixed(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& dplan,
                 const PrefillPlan& pplan, const void* q, void* out, int32_t Hq, float scale,
                 void* decode_ws, void* prefill_ws, hipStream_t st, bool f16, int32_t prio, int32_t persistent_wgs)
{
    return f16 ? launch_mixed_as<F16>(pool, layer, b, dplan, pplan, q, out, Hq, scale, decode_ws, prefill_ws, st, prio, persistent_wgs)
               : launch_mixed_as<Bf16>(pool, layer, b, dplan, pplan, q, out, Hq, scale, decode_ws, prefill_ws, st, prio, persistent_wgs);
}

}  // namespace cs
