// Prefill-chunk path of the mixed-batch paged attention: q_s > 1 new tokens of a sequence
// attend its prior context and, causally, their own chunk (paper Sec. 4.2: the attention
// term grows as P(P+C); chunked prefill).  Compute-bound, so the tiles run on the bf16
// matrix cores with an fp32 online softmax.
//
// A workgroup (4 wavefronts) owns one kv head and a tile of TQ consecutive chunk tokens
// with all G query heads that share the kv head: 16 "column tiles" of 16 query rows
// (16 tokens of one head), 4 per wavefront.  It walks the sequence's keys 32 at a time
// (two pages): all lanes copy the two pages' K and V blocks into LDS (double buffered, one
// barrier per step), every wavefront reads them back as MFMA operands -- the page format
// is the operand layout, so the LDS reads are linear in the lane id -- and computes
//   S^T[key][query]   = K . Q^T                      v_mfma_f32_16x16x32_bf16
//   O^T[d][query]    += V^T[d][32 keys] . P^T        v_mfma_f32_16x16x32_bf16
// with P^T taken straight from the S^T accumulators of the two pages (their C layout is
// the B layout of the second product).
#include "cs_common.h"

namespace cs {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kPrefillWaves = 4;
constexpr int kPrefillThreads = kPrefillWaves * 64;
constexpr int kNCT = 4;                       // column tiles per wavefront
constexpr int kKeysPerStep = 32;              // two pages

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 v = { (__bf16)lo, (__bf16)hi };
    return __builtin_bit_cast(uint32_t, v);
}

// Tokens per workgroup tile for a group size G: as many 16-token blocks as fit 16 column tiles.
__host__ __device__ inline int32_t prefill_tile_tokens(int32_t G) { return 16 * (16 / G); }

template <int D>
__global__ __launch_bounds__(kPrefillThreads, 1) void prefill_kernel(
    const uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t G, int32_t S,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float scale_log2e)
{
    constexpr int kUnits = D * 2;                     // 16-byte units per K (or V) block
    constexpr int kStepUnits = 4 * kUnits;            // K,V of two pages
    constexpr int kLoads = kStepUnits / kPrefillThreads;
    __shared__ u32x4 lds[2][kStepUnits];

    const int32_t TQ = prefill_tile_tokens(G);
    const int32_t g = blockIdx.x;
    const int32_t b = blockIdx.y;
    // sequence owning tile slot b: slots are dealt as start[s] = cu_q_lens[s] / TQ + s, which
    // leaves every sequence at least ceil(q_s / TQ) slots; find the largest s with start[s] <= b
    int32_t lo = 0, hi = S;
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (cu_q_lens[mid] / TQ + mid <= b) lo = mid; else hi = mid;
    }
    const int32_t s = lo;
    const int32_t t_seq = cu_q_lens[s];
    const int32_t q_len = cu_q_lens[s + 1] - t_seq;
    if (q_len <= 1) return;                            // decode and idle sequences: other path
    const int32_t tok0 = (b - (t_seq / TQ + s)) * TQ;  // first chunk token of this tile
    if (tok0 >= q_len) return;
    const int32_t C = ctx_lens[s];
    const int32_t n_tok = min(TQ, q_len - tok0);
    const int32_t n_seq_keys = C + q_len;              // keys the sequence holds after the append
    const int32_t n_keys = C + tok0 + n_tok;           // keys visible to the tile's last token
    const int32_t n_steps = (n_keys + kKeysPerStep - 1) / kKeysPerStep;
    const int32_t n_pages = min((n_seq_keys + kPage - 1) >> 4, max_blocks);
    const int32_t* table = block_tables + (int64_t)s * max_blocks;
    const int32_t Hq = Hkv * G;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- this wavefront's column tiles: ct = wave*4 + c -> (token block, head) ----
    bf16x8 qb[kNCT][D / 32];
    int32_t pos_q[kNCT];                               // absolute position of this lane's query
    int32_t min_pos[kNCT];                             // of the tile's first token (wave-uniform)
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int c = 0; c < kNCT; ++c) {
        const int32_t ct = wave * kNCT + c;
        const int32_t tb = ct / G, hh = ct - tb * G;
        const int32_t tl = tok0 + tb * 16 + (lane & 15);     // chunk-local token of this column
        const bool valid = tb * 16 < TQ && tl < q_len;
        pos_q[c] = C + tl;
        min_pos[c] = C + tok0 + tb * 16;
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            u32x4 v = zero4;
            if (valid)
                v = *(const u32x4*)(q + ((int64_t)(t_seq + tl) * Hq + g * G + hh) * D + kk * 32 + (lane >> 4) * 8);
            qb[c][kk] = __builtin_bit_cast(bf16x8, v);
        }
    }

    f32x4 o[kNCT][D / 16];
    float m_run[kNCT], l_run[kNCT];
#pragma unroll
    for (int c = 0; c < kNCT; ++c) {
        m_run[c] = -INFINITY;
        l_run[c] = 0.f;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) o[c][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- global -> register stage of one step (two pages, K and V blocks of head g) ----
    u32x4 stage[kLoads];
    auto fetch = [&](int32_t step) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int u = tid + j * kPrefillThreads;
            const int pg_in = u / (2 * kUnits);                 // 0 or 1: page within the step
            const int rem = u - pg_in * 2 * kUnits;
            const int kv = rem / kUnits, idx = rem - kv * kUnits;
            const int32_t pg = step * 2 + pg_in;
            u32x4 v = zero4;
            if (pg < n_pages) {
                const int32_t id = table[pg];
                if (id >= 0 && id < num_pages) {
                    const uint16_t* blk = layer_base + (int64_t)id * page_stride
                                        + ((int64_t)kv * Hkv + g) * (kPage * D);
                    v = *((const u32x4*)blk + idx);
                    if (kv == 1 && (pg + 1) * kPage > n_seq_keys) {
                        // V slots past the end of the sequence hold stale bits: zero them so
                        // that a zero weight times the slot stays zero.  A 16-byte unit holds
                        // two features of one 4-token group.
                        const int32_t valid = n_seq_keys - (pg * kPage + ((idx >> 3) & 3) * 4);
                        const uint32_t m0 = valid >= 2 ? 0xffffffffu : (valid == 1 ? 0x0000ffffu : 0u);
                        const uint32_t m1 = valid >= 4 ? 0xffffffffu : (valid == 3 ? 0x0000ffffu : 0u);
                        v[0] &= m0; v[1] &= m1; v[2] &= m0; v[3] &= m1;
                    }
                }
            }
            stage[j] = v;
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) lds[buf][tid + j * kPrefillThreads] = stage[j];
    };

    fetch(0);
    commit(0);
    __syncthreads();

    for (int32_t step = 0; step < n_steps; ++step) {
        const int buf = step & 1;
        if (step + 1 < n_steps) fetch(step + 1);
        const int32_t kb = step * kKeysPerStep;               // first key of the step
        const u32x4* kA0 = &lds[buf][0];
        const u32x2* vA0 = (const u32x2*)&lds[buf][kUnits];
        const u32x4* kA1 = &lds[buf][2 * kUnits];
        const u32x2* vA1 = (const u32x2*)&lds[buf][3 * kUnits];

        bf16x8 ka[2][D / 32];
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            ka[0][kk] = __builtin_bit_cast(bf16x8, kA0[kk * 64 + lane]);
            ka[1][kk] = __builtin_bit_cast(bf16x8, kA1[kk * 64 + lane]);
        }
        bf16x8 pb[kNCT];
#pragma unroll
        for (int c = 0; c < kNCT; ++c) {
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) {
                s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[0][kk], qb[c][kk], s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[1][kk], qb[c][kk], s1, 0, 0, 0);
            }
            float x[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) { x[i] = s0[i] * scale_log2e; x[4 + i] = s1[i] * scale_log2e; }
            if (kb + kKeysPerStep - 1 > min_pos[c]) {          // causal edge inside this step
                const int32_t key0 = kb + (lane >> 4) * 4;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (key0 + i > pos_q[c]) x[i] = -INFINITY;
                    if (key0 + 16 + i > pos_q[c]) x[4 + i] = -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[c], mx);            // finite from step 0 on (key 0 is visible)
            if (__any(m_new > m_run[c])) {
                const float alpha = exp2f(m_run[c] - m_new);
                l_run[c] *= alpha;
#pragma unroll
                for (int dt = 0; dt < D / 16; ++dt) o[c][dt] *= alpha;
                m_run[c] = m_new;
            }
            float p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) p[i] = exp2f(x[i] - m_run[c]);
            u32x4 pk = { pack2_bf16(p[0], p[1]), pack2_bf16(p[2], p[3]), pack2_bf16(p[4], p[5]), pack2_bf16(p[6], p[7]) };
            float ls = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)        // sum the weights as rounded, the ones that multiply V
                ls += __builtin_bit_cast(float, pk[i] << 16) + __builtin_bit_cast(float, pk[i] & 0xffff0000u);
            l_run[c] += ls;
            pb[c] = __builtin_bit_cast(bf16x8, pk);
        }
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
            const u32x2 a0 = vA0[dt * 64 + lane], a1 = vA1[dt * 64 + lane];
            const u32x4 av = { a0[0], a0[1], a1[0], a1[1] };
            const bf16x8 va = __builtin_bit_cast(bf16x8, av);
#pragma unroll
            for (int c = 0; c < kNCT; ++c)
                o[c][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[c], o[c][dt], 0, 0, 0);
        }
        if (step + 1 < n_steps) commit(buf ^ 1);
        __syncthreads();
    }

    // ---- normalise and store: lane holds 4 consecutive features of one query row per tile ----
#pragma unroll
    for (int c = 0; c < kNCT; ++c) {
        float l = l_run[c];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const int32_t ct = wave * kNCT + c;
        const int32_t tb = ct / G, hh = ct - tb * G;
        const int32_t tl = tok0 + tb * 16 + (lane & 15);
        if (tb * 16 < TQ && tl < q_len) {
            const float inv = 1.f / l;
            uint16_t* dst = out + ((int64_t)(t_seq + tl) * Hq + g * G + hh) * D + (lane >> 4) * 4;
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt) {
                u32x2 w = { pack2_bf16(o[c][dt][0] * inv, o[c][dt][1] * inv),
                            pack2_bf16(o[c][dt][2] * inv, o[c][dt][3] * inv) };
                *(u32x2*)(dst + dt * 16) = w;
            }
        }
    }
}

int launch_prefill(const cs_kv_pool& pool, int32_t layer, const cs_batch& b,
                   const void* q, void* out, int32_t Hq, float scale, hipStream_t st)
{
    const int32_t Hkv = pool.num_kv_heads, D = pool.head_dim, G = Hq / Hkv;
    const int32_t TQ = prefill_tile_tokens(G);
    const uint16_t* layer_base = (const uint16_t*)pool.base + (int64_t)layer * pool.layer_stride;
    const float scale_log2e = scale * 1.4426950408889634f;
    const uint32_t slots = (uint32_t)(b.num_tokens / TQ + b.num_seqs);
    if (slots > 65535u) return CS_ERR_UNSUPPORTED;
    dim3 grid((uint32_t)Hkv, slots);
    if (D == 128)
        hipLaunchKernelGGL(prefill_kernel<128>, grid, dim3(kPrefillThreads), 0, st, layer_base, pool.page_stride,
                           pool.num_pages, Hkv, G, b.num_seqs, b.block_tables, b.max_blocks_per_seq,
                           b.ctx_lens, b.cu_q_lens, (const uint16_t*)q, (uint16_t*)out, scale_log2e);
    else
        hipLaunchKernelGGL(prefill_kernel<64>, grid, dim3(kPrefillThreads), 0, st, layer_base, pool.page_stride,
                           pool.num_pages, Hkv, G, b.num_seqs, b.block_tables, b.max_blocks_per_seq,
                           b.ctx_lens, b.cu_q_lens, (const uint16_t*)q, (uint16_t*)out, scale_log2e);
    return check_launch("prefill_kernel");
}

}  // namespace cs
