// Kernels, launch plan and launcher of the prefill-chunk path (the workgroup's work itself is
// in cs_prefill_impl.h, shared with the fused mixed-batch kernel).
#include "cs_prefill_impl.h"

namespace cs {

// grid.x = slots * Hkv, kv head fastest (the slots from base_slot on: no sequence before it has a
// chunk); grid.y = key ranges
template <int D, class E, int PS>
__global__ __launch_bounds__(kPrefillThreads, 2) void prefill_kernel(
    const uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t G, int32_t S,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float scale_log2e,
    int32_t range_steps, int32_t base_slot, float* __restrict__ part, int32_t n_ordered, const SlotOrder order,
    int32_t backwards)
{
    __shared__ PrefillLds<D> lds;
    const int32_t pos = blockIdx.x / Hkv;
    const int32_t g = blockIdx.x - pos * Hkv;
    const int32_t b = n_ordered > 0 ? (int32_t)order.slot[pos]
                                    : base_slot + (backwards ? (int32_t)(gridDim.x / Hkv) - 1 - pos : pos);
    // (with key ranges the grid has no order table: cut position = slot position)
    prefill_tile<D, E, 1, PS, false>(lds, layer_base, page_stride, num_pages, Hkv, G, S, block_tables, max_blocks, ctx_lens, cu_q_lens,
                       q, out, scale_log2e, range_steps, partials_of<D>(part, b - base_slot, Hkv, g, gridDim.y), g, b,
                       blockIdx.y);
}

// Merge of the key-range partials of the tiles that were cut: grid.x = Hkv * cut tiles (launch
// positions cut_first_pos .. num_slots-1, the same numbering as the kernel that wrote them),
// grid.y = kMergeParts row groups of a tile; one lane per (query row, 4 features), so a
// wavefront reads whole 512-byte runs of a partial's rows.
constexpr int kMergeParts = 4;
template <int D, class E>
__global__ __launch_bounds__(kPrefillThreads) void prefill_merge_kernel(
    int32_t Hkv, int32_t G, int32_t S, const int32_t* __restrict__ ctx_lens,
    const int32_t* __restrict__ cu_q_lens, uint16_t* __restrict__ out,
    int32_t range_steps, int32_t max_ranges, int32_t base_slot, int32_t num_slots, int32_t cut_first_pos,
    int32_t backwards, const float* __restrict__ part)
{
    constexpr int kPartRow = D + 4;
    constexpr int kQuads = D / 4;                                  // lanes per query row
    constexpr int kRows = kTileCols * 16 / kMergeParts;            // rows of this workgroup
    const int32_t g = blockIdx.x % Hkv, cut_pos = blockIdx.x / Hkv, pos = cut_first_pos + cut_pos;
    const int32_t b = base_slot + (backwards ? num_slots - 1 - pos : pos);
    int32_t lo = 0, hi = S;
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (prefill_slot_start(cu_q_lens[mid], mid, G) <= b) lo = mid; else hi = mid;
    }
    const int32_t s = lo;
    const int32_t t_seq = cu_q_lens[s];
    const int32_t q_len = cu_q_lens[s + 1] - t_seq;
    if (q_len <= 1) return;
    const int32_t n_ct = ((q_len + 15) >> 4) * G;
    const int32_t ct0 = (int32_t)(b - prefill_slot_start(t_seq, s, G)) * kTileCols;
    if (ct0 >= n_ct) return;
    const int32_t tb_max = (min(ct0 + kTileCols, n_ct) - 1) / G;
    const int32_t n_keys = ctx_lens[s] + min(q_len, (tb_max + 1) * 16);
    const int32_t n_steps = (n_keys + kKeysPerStep - 1) / kKeysPerStep;
    const int32_t n_ranges = (n_steps + range_steps - 1) / range_steps;
    if (n_ranges <= 1) return;                               // written directly by the tile kernel
    const float* tile = partials_of<D>(const_cast<float*>(part), cut_pos, Hkv, g, max_ranges);
    const int64_t rstride = (int64_t)kTileCols * 16 * kPartRow;
    const int32_t Hq = Hkv * G;
    for (int32_t idx = threadIdx.x; idx < kRows * kQuads; idx += kPrefillThreads) {
        const int32_t row_id = blockIdx.y * kRows + idx / kQuads, quad = idx % kQuads;
        const int32_t ct = ct0 + (row_id >> 4);
        const int32_t tb = ct / G, hh = ct - tb * G;
        const int32_t tl = tb * 16 + (row_id & 15);
        if (ct >= n_ct || tl >= q_len) continue;
        const float* base = tile + row_id * kPartRow;
        float M = kNoMax;
        for (int32_t r = 0; r < n_ranges; ++r) M = fmaxf(M, base[r * rstride + D]);
        float L = 0.f;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int32_t r = 0; r < n_ranges; ++r) {
            const float* p = base + r * rstride;
            const float f = exp2f(p[D] - M);                 // 0 for a range the row sees nothing of
            L += p[D + 1] * f;
            const f32x4 v = *(const f32x4*)(p + quad * 4);
            acc += v * f;
        }
        const float inv = 1.f / L;
        uint16_t* dst = out + ((int64_t)(t_seq + tl) * Hq + g * G + hh) * D + quad * 4;
        u32x2 w = { E::pack(acc[0] * inv, acc[1] * inv), E::pack(acc[2] * inv, acc[3] * inv) };
        *(u32x2*)dst = w;
    }
}

// (plan_prefill, the host plan of the key-range split and the tile order, is in cs_api.hip with
// the other launch planning.)

template <class E>
static void launch_merge_as(const cs_kv_pool& pool, const cs_batch& b, const PrefillPlan& plan, void* out, int32_t Hq,
                            void* workspace, hipStream_t st)
{
    const int32_t Hkv = pool.num_kv_heads, D = pool.head_dim, G = Hq / Hkv;
    const float* part = (const float*)workspace;
    dim3 mgrid((uint32_t)Hkv * (uint32_t)(plan.num_slots - plan.cut_first_pos), kMergeParts);
    if (D == 128)
        hipLaunchKernelGGL((prefill_merge_kernel<128, E>), mgrid, dim3(kPrefillThreads), 0, st, Hkv, G, b.num_seqs,
                           b.ctx_lens, b.cu_q_lens, (uint16_t*)out, plan.range_steps, plan.max_ranges,
                           plan.base_slot, plan.num_slots, plan.cut_first_pos, (int32_t)plan.backwards, part);
    else
        hipLaunchKernelGGL((prefill_merge_kernel<64, E>), mgrid, dim3(kPrefillThreads), 0, st, Hkv, G, b.num_seqs,
                           b.ctx_lens, b.cu_q_lens, (uint16_t*)out, plan.range_steps, plan.max_ranges,
                           plan.base_slot, plan.num_slots, plan.cut_first_pos, (int32_t)plan.backwards, part);
}

template <class E>
static int launch_prefill_as(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const PrefillPlan& plan,
                             const void* q, void* out, int32_t Hq, float scale, void* workspace, hipStream_t st)
{
    const int32_t Hkv = pool.num_kv_heads, D = pool.head_dim, G = Hq / Hkv;
    const uint16_t* layer_base = (const uint16_t*)pool.base + (int64_t)layer * pool.layer_stride;
    const float scale_log2e = scale * 1.4426950408889634f;
    if ((int64_t)plan.num_slots * Hkv > 2147483647ll || plan.max_ranges > 65535) return CS_ERR_UNSUPPORTED;
    const uint32_t slots = plan.n_ordered > 0 ? (uint32_t)plan.n_ordered : (uint32_t)plan.num_slots;
    dim3 grid((uint32_t)Hkv * slots, (uint32_t)plan.max_ranges);
    float* part = (float*)workspace;
#define CS_LAUNCH_PREFILL(DD, PS)                                                                                   \
    hipLaunchKernelGGL((prefill_kernel<DD, E, PS>), grid, dim3(kPrefillThreads), 0, st, layer_base, pool.page_stride, \
                       pool.num_pages, Hkv, G, b.num_seqs, b.block_tables, b.max_blocks_per_seq,                   \
                       b.ctx_lens, b.cu_q_lens, (const uint16_t*)q, (uint16_t*)out, scale_log2e,                   \
                       plan.range_steps, plan.base_slot, part, plan.n_ordered, plan.order, (int32_t)plan.backwards);
    if (pool.page_size == 16) { if (D == 128) { CS_LAUNCH_PREFILL(128, 16) } else { CS_LAUNCH_PREFILL(64, 16) } }
    else                      { if (D == 128) { CS_LAUNCH_PREFILL(128, 8) } else { CS_LAUNCH_PREFILL(64, 8) } }
#undef CS_LAUNCH_PREFILL
    if (plan.max_ranges > 1) launch_merge_as<E>(pool, b, plan, out, Hq, workspace, st);
    return check_launch("prefill kernels");
}

int launch_prefill_merge(const cs_kv_pool& pool, const cs_batch& b, const PrefillPlan& plan, void* out, int32_t Hq,
                         void* workspace, hipStream_t st, bool f16)
{
    if (plan.max_ranges <= 1) return CS_OK;
    if (f16) launch_merge_as<F16>(pool, b, plan, out, Hq, workspace, st);
    else launch_merge_as<Bf16>(pool, b, plan, out, Hq, workspace, st);
    return check_launch("prefill merge kernel");
}

int launch_prefill(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const PrefillPlan& plan,
                   const void* q, void* out, int32_t Hq, float scale, void* workspace, hipStream_t st, bool f16)
{
    return f16 ? launch_prefill_as<F16>(pool, layer, b, plan, q, out, Hq, scale, workspace, st)
               : launch_prefill_as<Bf16>(pool, layer, b, plan, q, out, Hq, scale, workspace, st);
}

}  // namespace cs
