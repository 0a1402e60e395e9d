// Kernels and launcher of the decode path (the workgroup's work itself is in
// cs_decode_impl.h, shared with the fused mixed-batch kernel).
#include "cs_decode_impl.h"

namespace cs {

constexpr int kPlanThreads = 1024;

__global__ __launch_bounds__(kPlanThreads) void decode_plan_kernel(
    int32_t S, const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    int32_t split_tokens, int32_t total_items, int32_t num_multi,
    DecodeItem* __restrict__ items, int32_t* __restrict__ cu_items, int32_t* __restrict__ multi)
{
    // total_items / num_multi are what the host planned from its copies of the lengths; they
    // bound every write here should the device arrays disagree with those copies
    __shared__ int32_t sh_items[kPlanThreads], sh_multi[kPlanThreads];
    const int tid = threadIdx.x;
    const int32_t per = (S + kPlanThreads - 1) / kPlanThreads;
    const int32_t s0 = min(S, tid * per), s1 = min(S, s0 + per);
    int32_t n_items = 0, n_multi = 0;
    for (int32_t s = s0; s < s1; ++s) {
        if (cu_q_lens[s + 1] - cu_q_lens[s] != 1) continue;
        const int32_t k = decode_num_splits(ctx_lens[s] + 1, split_tokens);
        n_items += k;
        n_multi += k > 1;
    }
    sh_items[tid] = n_items;
    sh_multi[tid] = n_multi;
    __syncthreads();
    for (int off = 1; off < kPlanThreads; off <<= 1) {           // inclusive scan
        const int32_t a = tid >= off ? sh_items[tid - off] : 0;
        const int32_t b = tid >= off ? sh_multi[tid - off] : 0;
        __syncthreads();
        sh_items[tid] += a;
        sh_multi[tid] += b;
        __syncthreads();
    }
    int32_t item = sh_items[tid] - n_items, m = sh_multi[tid] - n_multi;   // exclusive
    for (int32_t s = s0; s < s1; ++s) {
        cu_items[s] = item;
        const int32_t t = cu_q_lens[s];
        if (cu_q_lens[s + 1] - t != 1) continue;
        const int32_t n = ctx_lens[s] + 1;
        const int32_t k = decode_num_splits(n, split_tokens);
        const int32_t chunk = decode_chunk_keys(n, k);
        for (int32_t i = 0; i < k; ++i) {
            DecodeItem it;
            it.seq = s; it.token = t; it.n_keys = n;
            it.key_begin = min(n, i * chunk);
            it.key_end = min(n, (i + 1) * chunk);
            it.n_splits = k; it.pad0 = 0; it.pad1 = 0;
            if (item + i < total_items) items[item + i] = it;
        }
        item += k;
        if (k > 1 && m < num_multi) multi[m++] = s;
    }
    if (tid == kPlanThreads - 1) cu_items[S] = sh_items[tid];
}

// grid = items * Hkv workgroups, kv head fastest (the heads of one page are neighbours
// in memory, so neighbouring workgroups share DRAM pages and translations).
template <int D, class Src, class E, int kAhead, int PS>
__global__ __launch_bounds__(kDecodeThreads, 2) void decode_split_kernel(
    const uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t G,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const Src src,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ q, uint16_t* __restrict__ out,
    float scale_log2e, float* __restrict__ part_o, float* __restrict__ part_ml)
{
    __shared__ DecodeLds<D> lds;
    const int32_t item = blockIdx.x / Hkv, g = blockIdx.x - item * Hkv;
    decode_item<D, Src, E, kAhead, PS>(lds, layer_base, page_stride, num_pages, Hkv, G, block_tables, max_blocks, src, ctx_lens,
                           cu_q_lens, q, out, scale_log2e, part_o, part_ml, item, g);
}

// Merge of the split partials of the sequences that were cut: grid = (Hq, num_multi),
// block = D lanes.  The list of cut sequences comes from the planning kernel or, like the
// items, from the kernel arguments.
struct MultiInMemory { const int32_t* multi; const int32_t* cu_items; };
struct MultiInArgs { ItemsInArgs list; const int32_t* ctx_lens; int32_t split_tokens, total_items; };

__device__ inline void fetch_multi(const MultiInMemory& src, int32_t idx, int32_t& s, int32_t& i0, int32_t& i1) {
    s = src.multi[idx];
    i0 = src.cu_items[s];
    i1 = src.cu_items[s + 1];
}
__device__ inline void fetch_multi(const MultiInArgs& src, int32_t idx, int32_t& s, int32_t& i0, int32_t& i1) {
    const uint32_t w = src.list.e[idx];
    s = (int32_t)(w & 0xffffu);
    i0 = (int32_t)(w >> 16);
    i1 = min(src.total_items, i0 + decode_num_splits(src.ctx_lens[s] + 1, src.split_tokens));
}

template <int D, class Src, class E>
__global__ __launch_bounds__(D) void decode_merge_kernel(
    const Src src, const int32_t* __restrict__ cu_q_lens, int32_t Hq,
    const float* __restrict__ part_o, const float* __restrict__ part_ml, uint16_t* __restrict__ out)
{
    const int32_t hq = blockIdx.x, d = threadIdx.x;
    int32_t s, i0, i1;
    fetch_multi(src, blockIdx.y, s, i0, i1);
    const int32_t t = cu_q_lens[s];
    float M = -INFINITY;
    for (int32_t i = i0; i < i1; ++i) M = fmaxf(M, part_ml[((int64_t)i * Hq + hq) * 2]);
    float L = 0.f, O = 0.f;
    for (int32_t i = i0; i < i1; ++i) {
        const int64_t slot = (int64_t)i * Hq + hq;
        const float mi = part_ml[slot * 2];
        const float f = mi == -INFINITY ? 0.f : exp2f(mi - M);
        L += part_ml[slot * 2 + 1] * f;
        O += part_o[slot * D + d] * f;
    }
    out[((int64_t)t * Hq + hq) * D + d] = (uint16_t)(E::pack(L > 0.f ? O / L : 0.f, 0.f) & 0xffffu);
}

template <class E>
static int launch_decode_as(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& plan,
                            const void* q, void* out, int32_t Hq, float scale, void* workspace, hipStream_t st,
                            bool merge_only)
{
    if (plan.num_decode == 0) return CS_OK;
    const int32_t Hkv = pool.num_kv_heads, D = pool.head_dim, G = Hq / Hkv;
    const uint16_t* layer_base = (const uint16_t*)pool.base + (int64_t)layer * pool.layer_stride;
    const float scale_log2e = scale * 1.4426950408889634f;
    const DecodeWorkspace w = decode_workspace(plan, b.num_seqs, Hq, D);
    char* ws = (char*)workspace;
    DecodeItem* items = (DecodeItem*)(ws + w.items);
    int32_t* cu_items = (int32_t*)(ws + w.cu_items);
    int32_t* multi = (int32_t*)(ws + w.multi);
    float* part_ml = (float*)(ws + w.part_ml);
    float* part_o = (float*)(ws + w.part_o);
    const bool identity = plan.num_multi == 0;
    const uint32_t n_items = plan.in_args ? plan.total_items : identity ? b.num_seqs : plan.total_items;
    dim3 grid(n_items * (uint32_t)Hkv);
    dim3 mgrid((uint32_t)Hq, (uint32_t)plan.num_multi);
#define CS_LAUNCH_DECODE_P(DD, SRC, src, AH, PS)                                                        \
    hipLaunchKernelGGL((decode_split_kernel<DD, SRC, E, AH, PS>), grid, dim3(kDecodeThreads), 0, st, layer_base, \
                       pool.page_stride, pool.num_pages, Hkv, G, b.block_tables, b.max_blocks_per_seq, \
                       src, b.ctx_lens, b.cu_q_lens, (const uint16_t*)q, (uint16_t*)out,               \
                       scale_log2e, part_o, part_ml);
#define CS_LAUNCH_DECODE_A(DD, SRC, src, AH)                                                            \
    if (pool.page_size == 16) { CS_LAUNCH_DECODE_P(DD, SRC, src, AH, 16) } else { CS_LAUNCH_DECODE_P(DD, SRC, src, AH, 8) }
#define CS_LAUNCH_DECODE(DD, SRC, src)                                                                 \
    if (plan.pages_ahead == 2) { CS_LAUNCH_DECODE_A(DD, SRC, src, 2) } else { CS_LAUNCH_DECODE_A(DD, SRC, src, 1) }
#define CS_LAUNCH_MERGE(DD, SRC, src)                                                                  \
    hipLaunchKernelGGL((decode_merge_kernel<DD, SRC, E>), mgrid, dim3(DD), 0, st, src, b.cu_q_lens, Hq,   \
                       part_o, part_ml, (uint16_t*)out);
    if (plan.in_args) {
        // (merge_only: the fused mixed-batch kernel has already done the items' work)
        if (!merge_only) {
            if (D == 128) { CS_LAUNCH_DECODE(128, ItemsInArgs, plan.arg_items) } else { CS_LAUNCH_DECODE(64, ItemsInArgs, plan.arg_items) }
        }
        if (!identity) {
            const MultiInArgs msrc = {plan.arg_multi, b.ctx_lens, plan.split_tokens, plan.total_items};
            if (D == 128) { CS_LAUNCH_MERGE(128, MultiInArgs, msrc) } else { CS_LAUNCH_MERGE(64, MultiInArgs, msrc) }
        }
    } else if (identity) {
        const ItemsIdentity src = {0};
        if (D == 128) { CS_LAUNCH_DECODE(128, ItemsIdentity, src) } else { CS_LAUNCH_DECODE(64, ItemsIdentity, src) }
    } else {
        hipLaunchKernelGGL(decode_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, b.num_seqs, b.ctx_lens,
                           b.cu_q_lens, plan.split_tokens, plan.total_items, plan.num_multi, items, cu_items, multi);
        const ItemsInMemory src = {items};
        const MultiInMemory msrc = {multi, cu_items};
        if (D == 128) { CS_LAUNCH_DECODE(128, ItemsInMemory, src) } else { CS_LAUNCH_DECODE(64, ItemsInMemory, src) }
        if (D == 128) { CS_LAUNCH_MERGE(128, MultiInMemory, msrc) } else { CS_LAUNCH_MERGE(64, MultiInMemory, msrc) }
    }
#undef CS_LAUNCH_DECODE
#undef CS_LAUNCH_DECODE_A
#undef CS_LAUNCH_DECODE_P
#undef CS_LAUNCH_MERGE
    return check_launch("decode kernels");
}

int launch_decode(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const DecodePlan& plan,
                  const void* q, void* out, int32_t Hq, float scale, void* workspace, hipStream_t st, bool f16,
                  bool merge_only)
{
    return f16 ? launch_decode_as<F16>(pool, layer, b, plan, q, out, Hq, scale, workspace, st, merge_only)
               : launch_decode_as<Bf16>(pool, layer, b, plan, q, out, Hq, scale, workspace, st, merge_only);
}

}  // namespace cs
