// Kernels, launch plan and launcher of the prefill-chunk path (the workgroup's work itself is
// in cs_prefill_impl.h, shared with the fused mixed-batch kernel).
#include <cmath>
#include "cs_prefill_impl.h"

namespace cs {

// grid.x = slots * Hkv, kv head fastest; grid.y = key ranges
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
    const int32_t b = n_ordered > 0 ? (int32_t)order.slot[pos] : backwards ? (int32_t)(gridDim.x / Hkv) - 1 - pos : pos;
    prefill_tile<D, E, true, PS, false>(lds, layer_base, page_stride, num_pages, Hkv, G, S, block_tables, max_blocks, ctx_lens, cu_q_lens,
                       q, out, scale_log2e, range_steps, base_slot, part, g, b, blockIdx.y, gridDim.y);
}

// Merge of the key-range partials of the tiles that were cut: grid = Hkv * slots, 256
// lanes, two lanes per query row (half of the features each).
template <int D, class E>
__global__ __launch_bounds__(kPrefillThreads) void prefill_merge_kernel(
    int32_t Hkv, int32_t G, int32_t S, const int32_t* __restrict__ ctx_lens,
    const int32_t* __restrict__ cu_q_lens, uint16_t* __restrict__ out,
    int32_t range_steps, int32_t max_ranges, int32_t base_slot, const float* __restrict__ part)
{
    constexpr int kPartRow = D + 4;
    const int32_t g = blockIdx.x % Hkv, b = blockIdx.x / Hkv + base_slot;
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
    const int32_t row_id = threadIdx.x >> 1, half = threadIdx.x & 1;
    const int32_t ct = ct0 + (row_id >> 4);
    const int32_t tb = ct / G, hh = ct - tb * G;
    const int32_t tl = tb * 16 + (row_id & 15);
    if (ct >= n_ct || tl >= q_len) return;
    const float* base = part + (((int64_t)(b - base_slot) * Hkv + g) * max_ranges) * (kTileCols * 16 * kPartRow)
                      + row_id * kPartRow;
    const int64_t rstride = (int64_t)kTileCols * 16 * kPartRow;
    float M = kNoMax;
    for (int32_t r = 0; r < n_ranges; ++r) M = fmaxf(M, base[r * rstride + D]);
    float L = 0.f;
    float acc[D / 2];
#pragma unroll
    for (int d = 0; d < D / 2; ++d) acc[d] = 0.f;
    for (int32_t r = 0; r < n_ranges; ++r) {
        const float* p = base + r * rstride;
        const float f = exp2f(p[D] - M);                     // 0 for a range the row sees nothing of
        L += p[D + 1] * f;
#pragma unroll
        for (int d = 0; d < D / 2; d += 4) {
            const f32x4 v = *(const f32x4*)(p + half * (D / 2) + d);
            acc[d] += v[0] * f; acc[d + 1] += v[1] * f; acc[d + 2] += v[2] * f; acc[d + 3] += v[3] * f;
        }
    }
    const float inv = 1.f / L;
    const int32_t Hq = Hkv * G;
    uint16_t* dst = out + ((int64_t)(t_seq + tl) * Hq + g * G + hh) * D + half * (D / 2);
#pragma unroll
    for (int d = 0; d < D / 2; d += 4) {
        u32x2 w = { E::pack(acc[d] * inv, acc[d + 1] * inv), E::pack(acc[d + 2] * inv, acc[d + 3] * inv) };
        *(u32x2*)(dst + d) = w;
    }
}

// Host plan of the key-range split (a pure function of the host lengths).
PrefillPlan plan_prefill(const cs_batch* b, int32_t Hq, int32_t Hkv, int32_t D) {
    PrefillPlan p = {};
    const int32_t G = Hq / Hkv;
    int64_t total_steps = 0, tiles = 0;
    int32_t max_steps = 0, first = -1;
    struct Tile { int32_t steps, slot; };
    Tile tile_list[kMaxSlotOrder];
    int32_t n_listed = 0;
    for (int32_t s = 0; s < b->num_seqs; ++s) {
        const int32_t ql = b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s];
        if (ql <= 1) continue;
        if (first < 0) first = s;
        const int32_t C = b->h_ctx_lens[s];
        const int32_t n_ct = ((ql + 15) >> 4) * G;
        for (int32_t ct0 = 0; ct0 < n_ct; ct0 += kTileCols) {
            const int32_t tb_max = (std::min(ct0 + kTileCols, n_ct) - 1) / G;
            const int32_t n_keys = C + std::min(ql, (tb_max + 1) * 16);
            const int32_t steps = (n_keys + kKeysPerStep - 1) / kKeysPerStep;
            total_steps += steps;
            max_steps = std::max(max_steps, steps);
            if (tiles < kMaxSlotOrder)
                tile_list[n_listed++] = Tile{steps, (int32_t)(prefill_slot_start(b->h_cu_q_lens[s], s, G) + ct0 / kTileCols)};
            ++tiles;
        }
    }
    p.range_steps = std::max(max_steps, 1);
    p.max_ranges = 1;
    if (tiles == 0) return p;
    const int64_t wgs = tiles * Hkv;
    // The chip: `cus` compute units, two workgroup slots each.  (The counts in the comments below
    // are those of the 256-CU part the rules were measured on.)
    const int64_t cus = device_cus(), slots = 2 * cus;
    if (wgs <= cus * 3 / 4 && max_steps < 128) {
        // few and short tiles: about four workgroups per CU, ranges of at least 32 steps
        const int64_t rs = std::max<int64_t>(32, (total_steps * Hkv + 4 * cus - 1) / (4 * cus));
        if (rs < max_steps) {
            p.range_steps = (int32_t)rs;
            p.max_ranges = (max_steps + p.range_steps - 1) / p.range_steps;
        }
    } else if (wgs <= 4 * cus) {
        // Up to four workgroups per CU the grid runs as one or two rounds over the 512 workgroup
        // slots (or leaves CUs empty), and a round that is not full costs almost as much as a
        // full one.  Cutting every tile into r key ranges multiplies the workgroups and divides
        // their length: pick the r whose rounds come out fullest.  The cost model is fitted to
        // measurements (it reproduces them within a few percent), in steps of a workgroup that
        // shares its CU: a workgroup with the CU to itself runs a step in 0.76 of that; while all
        // workgroups are resident the longest tile decides, beyond that the average tile and a
        // round count halfway between W/512 and its ceiling (tiles end at different times, so
        // rounds blur); every workgroup pays about 8 steps of start-up and store; the partials
        // cost a launch plus their bytes written and read back at 5 TB/s.
        const double avg_steps = (double)total_steps / (double)tiles;
        auto cost = [&](int r) -> double {
            const double W = (double)wgs * r;
            double c;
            if (W <= cus) c = 0.76 * ((double)max_steps / r + 8);
            else if (W <= slots) c = (0.76 + (W - cus) / cus * 0.24) * ((double)max_steps / r + 8);
            else c = 0.5 * (W / slots + std::ceil(W / slots)) * (avg_steps / r + 8);
            if (r > 1) {
                const double part_bytes = W * kTileCols * 16 * (D + 4) * 4.0;
                c += (10.0 + 2.0 * part_bytes / 5.0e6) / 0.87;     // microseconds -> steps
            }
            return c;
        };
        int best = 1;
        double best_cost = cost(1);
        for (int r = 2; r <= 16; ++r) {
            if (max_steps / r < 32) break;
            const double c = cost(r);
            if (c < best_cost) { best = r; best_cost = c; }
        }
        if (best > 1 && best_cost <= 0.92 * cost(1)) {
            p.range_steps = (max_steps + best - 1) / best;
            p.max_ranges = (max_steps + p.range_steps - 1) / p.range_steps;
        }
    }
    // Uncut tiles in an order that suits the dispatcher, which deals workgroup i to XCD i % 8,
    // gives the first 256 a CU each and puts workgroup i + 256 beside workgroup i (observed with
    // a probe that records where each workgroup runs).  While everything is resident (up to 512
    // workgroups) the call lasts as long as the slowest CU: the longest tiles get the CUs of their
    // own (positions W-256 .. 255) and the rest are paired long with short.  With more tiles than
    // slots the longest go first and the short ones fill the end; the natural order is the
    // opposite (a chunk's later tiles see more keys).  The order travels as a table in the kernel
    // arguments; a batch with more tiles than the table holds is simply walked backwards.
    const int32_t first_round = (int32_t)(cus / Hkv);            // slot positions of the first round (a CU each)
    bool slots_fit = true;                                       // a table entry is 16 bits
    for (int32_t k = 0; k < n_listed; ++k) slots_fit = slots_fit && tile_list[k].slot < 65536;
    if (p.max_ranges == 1 && wgs > cus) {
        const bool listed = tiles == n_listed && slots_fit;
        if (listed && wgs <= slots && cus % Hkv == 0) {
            std::stable_sort(tile_list, tile_list + n_listed, [](const Tile& a, const Tile& c) { return a.steps > c.steps; });
            const int32_t n_pair = (int32_t)tiles - first_round, n_solo = first_round - n_pair;
            for (int32_t k = 0; k < n_solo; ++k) p.order.slot[n_pair + k] = (uint16_t)tile_list[k].slot;
            for (int32_t k = 0; k < n_pair; ++k) {
                p.order.slot[k] = (uint16_t)tile_list[n_solo + k].slot;                                   // long
                p.order.slot[first_round + k] = (uint16_t)tile_list[n_solo + 2 * n_pair - 1 - k].slot;    // short
            }
            p.n_ordered = (int32_t)tiles;
        } else if (wgs > slots) {
            if (listed) {
                std::stable_sort(tile_list, tile_list + n_listed, [](const Tile& a, const Tile& c) { return a.steps > c.steps; });
                for (int32_t k = 0; k < n_listed; ++k) p.order.slot[k] = (uint16_t)tile_list[k].slot;
                p.n_ordered = (int32_t)tiles;
            }
            p.backwards = true;
        }
    }
    if (p.max_ranges > 1) {
        p.base_slot = (int32_t)prefill_slot_start(b->h_cu_q_lens[first], first, G);
        p.num_slots = (int32_t)(prefill_slot_start(b->num_tokens, b->num_seqs, G) - p.base_slot);
        p.bytes = (size_t)p.num_slots * Hkv * p.max_ranges * kTileCols * 16 * (D + 4) * sizeof(float);
    }
    return p;
}

template <class E>
static void launch_merge_as(const cs_kv_pool& pool, const cs_batch& b, const PrefillPlan& plan, void* out, int32_t Hq,
                            void* workspace, hipStream_t st)
{
    const int32_t Hkv = pool.num_kv_heads, D = pool.head_dim, G = Hq / Hkv;
    const float* part = (const float*)workspace;
    dim3 mgrid((uint32_t)Hkv * (uint32_t)plan.num_slots);
    if (D == 128)
        hipLaunchKernelGGL((prefill_merge_kernel<128, E>), mgrid, dim3(kPrefillThreads), 0, st, Hkv, G, b.num_seqs,
                           b.ctx_lens, b.cu_q_lens, (uint16_t*)out, plan.range_steps, plan.max_ranges,
                           plan.base_slot, part);
    else
        hipLaunchKernelGGL((prefill_merge_kernel<64, E>), mgrid, dim3(kPrefillThreads), 0, st, Hkv, G, b.num_seqs,
                           b.ctx_lens, b.cu_q_lens, (uint16_t*)out, plan.range_steps, plan.max_ranges,
                           plan.base_slot, part);
}

template <class E>
static int launch_prefill_as(const cs_kv_pool& pool, int32_t layer, const cs_batch& b, const PrefillPlan& plan,
                             const void* q, void* out, int32_t Hq, float scale, void* workspace, hipStream_t st)
{
    const int32_t Hkv = pool.num_kv_heads, D = pool.head_dim, G = Hq / Hkv;
    const uint16_t* layer_base = (const uint16_t*)pool.base + (int64_t)layer * pool.layer_stride;
    const float scale_log2e = scale * 1.4426950408889634f;
    const int64_t slots64 = prefill_slot_start(b.num_tokens, b.num_seqs, G);
    if (slots64 * Hkv > 2147483647ll || plan.max_ranges > 65535) return CS_ERR_UNSUPPORTED;
    const uint32_t slots = plan.n_ordered > 0 ? (uint32_t)plan.n_ordered : (uint32_t)slots64;
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
