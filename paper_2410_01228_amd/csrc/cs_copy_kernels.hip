// Copy kernels: KV append into pages, checkpoint gather / restore of whole pages, and a
// plain copy used as the bandwidth ceiling.  All are HBM-bound streams of 16-byte lanes.
#include <algorithm>
#include "cs_common.h"

namespace cs {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------
// Whole-page copies (paper Sec. 5: gather scattered pages into one contiguous buffer;
// Sec. 4.4: bring them back on resume).  One (layer, page) is contiguous in the pool, so
// both directions are straight 16-byte-per-lane streams.  A workgroup is a single wavefront
// moving kChunkBytes (measured: many one-wavefront workgroups of 1 KiB sustain more HBM
// bandwidth on this part than fewer, fatter ones with several requests per lane in flight).
// ------------------------------------------------------------------------------------
constexpr int kCopyThreads = 64;
constexpr int kCopyUnroll = 1;                                   // 1 KiB per workgroup
constexpr int kChunkBytes = kCopyThreads * 16 * kCopyUnroll;

template <bool kToStaging>
__global__ __launch_bounds__(kCopyThreads) void page_copy_kernel(
    char* __restrict__ pool_base, int64_t layer_stride_b, int64_t page_stride_b,
    int32_t num_pages, int32_t layer_begin, const int32_t* __restrict__ ids,
    char* __restrict__ staging, int64_t stg_layer_stride_b, int64_t stg_page_stride_b,
    int32_t page_bytes, int32_t chunks_per_page)
{
    // grid.x = n * chunks_per_page (page-major), grid.y = layers
    const int32_t i = blockIdx.x / chunks_per_page;
    const int32_t c = blockIdx.x - i * chunks_per_page;
    const int32_t l = blockIdx.y;
    const int32_t id = ids[i];
    if (id < 0 || id >= num_pages) return;                       // never touch a bad page id
    char* p = pool_base + (int64_t)(layer_begin + l) * layer_stride_b + (int64_t)id * page_stride_b;
    char* s = staging + l * stg_layer_stride_b + i * stg_page_stride_b;
    const char* src = kToStaging ? p : s;
    char* dst = kToStaging ? s : p;
    const int32_t off0 = c * kChunkBytes + threadIdx.x * 16;
    u32x4 r[kCopyUnroll];
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) {
        const int32_t off = off0 + u * kCopyThreads * 16;
        if (off < page_bytes) r[u] = __builtin_nontemporal_load((const u32x4*)(src + off));
    }
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) {
        const int32_t off = off0 + u * kCopyThreads * 16;
        if (off < page_bytes) __builtin_nontemporal_store(r[u], (u32x4*)(dst + off));
    }
}

int launch_page_copy(const cs_kv_pool& pool, int32_t layer_begin, int32_t layer_end,
                     const int32_t* ids, int32_t n, void* staging, bool to_staging, hipStream_t st,
                     bool page_major)
{
    const int32_t layers = layer_end - layer_begin;
    if (n == 0 || layers == 0) return CS_OK;
    const int32_t page_bytes = (int32_t)pool_page_bytes(pool);
    const int32_t cpp = (page_bytes + kChunkBytes - 1) / kChunkBytes;
    dim3 grid((uint32_t)n * cpp, (uint32_t)layers);
    // staging[layer][page] (the default) or staging[page][layer] (one page's layers together)
    const int64_t stg_layer = page_major ? (int64_t)page_bytes : (int64_t)n * page_bytes;
    const int64_t stg_page = page_major ? (int64_t)layers * page_bytes : (int64_t)page_bytes;
    if (to_staging)
        hipLaunchKernelGGL(page_copy_kernel<true>, grid, dim3(kCopyThreads), 0, st,
                           (char*)pool.base, pool.layer_stride * 2, pool.page_stride * 2, pool.num_pages,
                           layer_begin, ids, (char*)staging, stg_layer, stg_page, page_bytes, cpp);
    else
        hipLaunchKernelGGL(page_copy_kernel<false>, grid, dim3(kCopyThreads), 0, st,
                           (char*)pool.base, pool.layer_stride * 2, pool.page_stride * 2, pool.num_pages,
                           layer_begin, ids, (char*)staging, stg_layer, stg_page, page_bytes, cpp);
    return check_launch("page_copy_kernel");
}

// ------------------------------------------------------------------------------------
// Token-granular checkpoint copies (paper Sec. 4.4: KV state is kept per token; after a
// generation step only the newly generated tokens are checkpointed).  The staging buffer
// holds plain rows, [layer][token][K|V][kv head][D]; one lane moves one 16-byte unit of a
// row (8 features): a K unit is one 16-byte unit of the page too, a V unit is 8 elements
// that lie 16 bytes apart in the page (one per feature's token group).
// ------------------------------------------------------------------------------------
constexpr int kTokenCopyThreads = 256;

template <bool kToStaging>
__global__ __launch_bounds__(kTokenCopyThreads) void token_copy_kernel(
    uint16_t* __restrict__ pool_base, int64_t layer_stride, int64_t page_stride,
    int32_t num_pages, int32_t layer_begin, const int32_t* __restrict__ token_slots, int32_t n,
    uint16_t* __restrict__ staging, int32_t Hkv, int32_t D, int32_t page_size)
{
    const int32_t units_per_head = D / 8, units_per_side = Hkv * units_per_head;
    const int32_t units_per_token = 2 * units_per_side;
    const int64_t gid = (int64_t)blockIdx.x * kTokenCopyThreads + threadIdx.x;
    if (gid >= (int64_t)n * units_per_token) return;
    const int32_t i = (int32_t)(gid / units_per_token), u = (int32_t)(gid - (int64_t)i * units_per_token);
    const int32_t l = blockIdx.y;
    const int32_t slot = token_slots[i];
    const int32_t page = slot / page_size, t = slot - page * page_size;
    if (slot < 0 || page >= num_pages) return;                   // never touch a bad slot
    const int32_t groups = page_size >> 3;                       // 8-token groups of a page
    const int32_t kv = u / units_per_side, r = u - kv * units_per_side;
    const int32_t h = r / units_per_head, d8 = r - h * units_per_head;
    uint16_t* blk = pool_base + (int64_t)(layer_begin + l) * layer_stride + (int64_t)page * page_stride
                  + (int64_t)(kv * Hkv + h) * (page_size * D);
    uint16_t* row = staging + ((int64_t)l * n + i) * (2 * Hkv * D) + (int64_t)u * 8;
    if (kv == 0) {
        u32x4* unit = (u32x4*)(blk + (d8 * page_size + t) * 8);
        if (kToStaging) *(u32x4*)row = *unit; else *unit = *(const u32x4*)row;
    } else {
        // features d8*8 .. +8 of token t: element (((d/16)*groups + t/8)*16 + d%16)*8 + t%8
        const int32_t d0 = d8 * 8;
        uint16_t* first = blk + ((((d0 >> 4) * groups + (t >> 3)) * 16 + (d0 & 15)) * 8 + (t & 7));
        if (kToStaging) {
            uint16_t e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = first[j * 8];
            u32x4 v = { (uint32_t)e[0] | ((uint32_t)e[1] << 16), (uint32_t)e[2] | ((uint32_t)e[3] << 16),
                        (uint32_t)e[4] | ((uint32_t)e[5] << 16), (uint32_t)e[6] | ((uint32_t)e[7] << 16) };
            *(u32x4*)row = v;
        } else {
            const u32x4 v = *(const u32x4*)row;
#pragma unroll
            for (int j = 0; j < 8; ++j) first[j * 8] = (uint16_t)(v[j >> 1] >> ((j & 1) * 16));
        }
    }
}

int launch_token_copy(const cs_kv_pool& pool, int32_t layer_begin, int32_t layer_end,
                      const int32_t* token_slots, int32_t n, void* staging, bool to_staging, hipStream_t st)
{
    const int32_t layers = layer_end - layer_begin;
    if (n == 0 || layers == 0) return CS_OK;
    const int64_t units = (int64_t)n * 2 * pool.num_kv_heads * pool.head_dim / 8;
    dim3 grid((uint32_t)((units + kTokenCopyThreads - 1) / kTokenCopyThreads), (uint32_t)layers);
    if (to_staging)
        hipLaunchKernelGGL(token_copy_kernel<true>, grid, dim3(kTokenCopyThreads), 0, st, (uint16_t*)pool.base,
                           pool.layer_stride, pool.page_stride, pool.num_pages, layer_begin, token_slots, n,
                           (uint16_t*)staging, pool.num_kv_heads, pool.head_dim, pool.page_size);
    else
        hipLaunchKernelGGL(token_copy_kernel<false>, grid, dim3(kTokenCopyThreads), 0, st, (uint16_t*)pool.base,
                           pool.layer_stride, pool.page_stride, pool.num_pages, layer_begin, token_slots, n,
                           (uint16_t*)staging, pool.num_kv_heads, pool.head_dim, pool.page_size);
    return check_launch("token_copy_kernel");
}

// ------------------------------------------------------------------------------------
// Plain copy: the same inner loop without the page indirection.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kCopyThreads) void plain_copy_kernel(
    char* __restrict__ dst, const char* __restrict__ src, int64_t bytes)
{
    const int64_t off0 = (int64_t)blockIdx.x * kChunkBytes + threadIdx.x * 16;
    u32x4 r[kCopyUnroll];
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) {
        const int64_t off = off0 + u * kCopyThreads * 16;
        if (off < bytes) r[u] = __builtin_nontemporal_load((const u32x4*)(src + off));
    }
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) {
        const int64_t off = off0 + u * kCopyThreads * 16;
        if (off < bytes) __builtin_nontemporal_store(r[u], (u32x4*)(dst + off));
    }
}

int launch_plain_copy(void* dst, const void* src, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return CS_OK;
    const uint64_t blocks = (bytes + kChunkBytes - 1) / kChunkBytes;
    hipLaunchKernelGGL(plain_copy_kernel, dim3((uint32_t)blocks), dim3(kCopyThreads), 0, st,
                       (char*)dst, (const char*)src, (int64_t)bytes);
    return check_launch("plain_copy_kernel");
}

// ------------------------------------------------------------------------------------
// KV append (the cache is append-only: paper Sec. 1, 4.4).  A workgroup of 4 wavefronts
// owns one (page touched this step, kv head) and writes that page's K and V blocks in the
// order they lie in memory, so every store instruction of a wavefront covers 1 KiB of
// consecutive bytes; slots the step does not fill are simply masked out.  Sequences with a
// single new token go through append_token_kernel below instead.
// Workgroup slots are dealt to sequences as start(s) = cu_q_lens[s]/16 + 2s (a step of q
// tokens touches at most q/16 + 2 pages), found by bisection.
// ------------------------------------------------------------------------------------
constexpr int kAppendThreads = 256;
constexpr int kAppendSlotShift = 4;

// The work of workgroup `block` of the chunk path.
template <int PS>
__device__ __forceinline__ void append_page_block(
    int32_t block,
    uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t D, int32_t S,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new)
{
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Groups of 8 page
    // slots are numbered head-major, so the workgroups of one page -- which together read
    // whole token rows and write one whole page -- all land on the same XCD.
    const int32_t per = 8 * Hkv;
    const int32_t group = block / per, in_group = block - group * per;
    const int32_t h = in_group >> 3;
    const int32_t slot_id = group * 8 + (in_group & 7);
    int32_t lo = 0, hi = S;                                       // largest s with start(s) <= slot_id
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if ((cu_q_lens[mid] >> kAppendSlotShift) + 2 * mid <= slot_id) lo = mid; else hi = mid;
    }
    const int32_t s = lo;
    const int32_t t_seq = cu_q_lens[s];
    const int32_t first = ctx_lens[s];                            // the step fills positions [first, last)
    const int32_t last = first + (cu_q_lens[s + 1] - t_seq);
    if (last - first == 1) return;                               // single tokens: append_token_kernel
    // the workgroup's 16 positions: one page, or (pages of 8 tokens) two consecutive table entries
    const int32_t blk = (first >> 4) + (slot_id - ((t_seq >> kAppendSlotShift) + 2 * s));
    const int32_t p0 = blk << 4;                                  // first of the 16 positions
    if (p0 >= last) return;
    const int32_t block_elems = PS * D;
    const int32_t row = Hkv * D;                                  // elements between consecutive tokens
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (wave * 32 >= D) return;                                   // head_dim 64: two wavefronts suffice

    // Wavefront w moves features 32w .. 32w+31 of the page's 16 tokens.
    // K: lane (feature block dl = lane/16, token = lane%16) loads the 16 bytes of its token's
    //    row and stores them as unit dblk*16 + token.
    // V: a 16-byte unit is one feature of 8 consecutive tokens.  Lane (tile = lane/32, token
    //    half th = (lane/16)%2, feature f = lane%16) loads its feature from each of the half's
    //    8 token rows and stores the unit; the unit index is 64w + lane.
    // Either way consecutive lanes store consecutive units: 1 KiB per store instruction.
    const int32_t tok = lane & 15, dblk = wave * 4 + (lane >> 4);
    const int32_t th = (lane >> 4) & 1, feat = wave * 32 + (lane >> 5) * 16 + (lane & 15);
    // table entries of this lane's K token and of its V half (the same entry for pages of 16)
    const int32_t k_entry = PS == 16 ? blk : 2 * blk + (tok >> 3);
    const int32_t v_entry = PS == 16 ? blk : 2 * blk + th;
    const int32_t* table = block_tables + (int64_t)s * max_blocks;
    const int32_t k_page = k_entry < max_blocks ? table[k_entry] : -1;
    const int32_t v_page = v_entry < max_blocks ? table[v_entry] : -1;
    const bool k_page_ok = k_page >= 0 && k_page < num_pages, v_page_ok = v_page >= 0 && v_page < num_pages;
    // packed token index of page position p0 (may lie before the step's first token)
    const int64_t tok_base = (int64_t)t_seq + (p0 - first);
    const int32_t pos = p0 + tok;
    const bool k_ok = k_page_ok && pos >= first && pos < last;
    const int32_t vpos = p0 + th * 8;                             // first position of the half
    const bool v_full = v_page_ok && vpos >= first && vpos + 8 <= last;
    const uint16_t* ksrc = k_new + (tok_base + tok) * row + (int64_t)h * D + dblk * 8;
    const uint16_t* vsrc = v_new + (tok_base + th * 8) * row + (int64_t)h * D + feat;
    uint16_t* kblk = layer_base + (int64_t)(k_page_ok ? k_page : 0) * page_stride + (int64_t)h * block_elems;
    // V unit of this lane: 64*wave + lane in a page of 16 tokens (two halves per feature tile),
    // (2*wave + lane/32)*16 + lane%16 in the page of its half otherwise
    const int32_t v_unit = PS == 16 ? wave * 64 + lane : (wave * 2 + (lane >> 5)) * 16 + (lane & 15);
    uint16_t* dst = layer_base + (int64_t)(v_page_ok ? v_page : 0) * page_stride + (int64_t)(Hkv + h) * block_elems + v_unit * 8;
    u32x4 kv;
    uint16_t e[8];
    if (k_ok) kv = __builtin_nontemporal_load((const u32x4*)ksrc);
    if (v_full) {
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = __builtin_nontemporal_load(vsrc + j * row);
    }
    if (k_ok) __builtin_nontemporal_store(kv, (u32x4*)(kblk + (dblk * PS + (tok & (PS - 1))) * 8));
    if (v_full) {
        const u32x4 unit = { (uint32_t)e[0] | ((uint32_t)e[1] << 16), (uint32_t)e[2] | ((uint32_t)e[3] << 16),
                             (uint32_t)e[4] | ((uint32_t)e[5] << 16), (uint32_t)e[6] | ((uint32_t)e[7] << 16) };
        __builtin_nontemporal_store(unit, (u32x4*)dst);
    } else if (v_page_ok) {
        // a half the step fills only partly: element by element
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (vpos + j >= first && vpos + j < last) dst[j] = vsrc[j * row];
    }
}

// Single new tokens (decode): one lane per 16-byte unit (8 features) of the token's K row
// and V row.  The K unit is stored as it is; the V unit is scattered as 8 two-byte stores
// (the V block keeps 8 consecutive TOKENS of one feature together).  Sequences with more
// than one new token are left to append_page_kernel.
__device__ __forceinline__ void append_token_block(
    int32_t block,
    uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t D, int32_t S, int32_t T,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new, int32_t page_size)
{
    const int32_t units_per_tok = Hkv * (D >> 3);
    const int64_t gid = (int64_t)block * kAppendThreads + threadIdx.x;
    const int32_t t = (int32_t)(gid / units_per_tok);
    if (t >= T) return;
    const int32_t u = (int32_t)(gid - (int64_t)t * units_per_tok);
    const int32_t h = u / (D >> 3);
    const int32_t dblk = u - h * (D >> 3);
    // sequence of token t.  In an online-first batch the decode sequences lead, so token t is
    // usually sequence t: try that before bisecting the prefix sums.
    int32_t s = min(t, S - 1);
    if (!(cu_q_lens[s] <= t && t < cu_q_lens[s + 1])) {
        int32_t lo = 0, hi = S;                                   // invariant: cu[lo] <= t < cu[hi]
        while (hi - lo > 1) {
            const int32_t mid = (lo + hi) >> 1;
            if (cu_q_lens[mid] <= t) lo = mid; else hi = mid;
        }
        s = lo;
    }
    if (cu_q_lens[s + 1] - cu_q_lens[s] != 1) return;
    const int32_t pos = ctx_lens[s];
    const int32_t blk = pos / page_size;
    if (pos < 0 || blk >= max_blocks) return;
    const int32_t page = block_tables[(int64_t)s * max_blocks + blk];
    if (page < 0 || page >= num_pages) return;
    const int32_t slot = pos - blk * page_size;
    const int32_t block_elems = page_size * D;
    uint16_t* kblk = layer_base + (int64_t)page * page_stride + (int64_t)h * block_elems;
    uint16_t* vblk = kblk + (int64_t)Hkv * block_elems;
    const int64_t src = ((int64_t)t * Hkv + h) * D + dblk * 8;
    *(u32x4*)(kblk + (dblk * page_size + slot) * 8) = *(const u32x4*)(k_new + src);
    const u32x4 vv = *(const u32x4*)(v_new + src);
    // feature d = dblk*8 + e  ->  (((d/16)*groups + slot/8)*16 + d%16)*8 + slot%8, groups = page_size/8
    const int32_t vbase = (((dblk >> 1) * (page_size >> 3) + (slot >> 3)) * 16 + (dblk & 1) * 8) * 8 + (slot & 7);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t w = vv[e >> 1];
        vblk[vbase + e * 8] = (uint16_t)((e & 1) ? (w >> 16) : (w & 0xffffu));
    }
}

template <int PS>
__global__ __launch_bounds__(kAppendThreads) void append_page_kernel(
    uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t D, int32_t S,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new)
{
    append_page_block<PS>((int32_t)blockIdx.x, layer_base, page_stride, num_pages, Hkv, D, S, block_tables, max_blocks,
                          ctx_lens, cu_q_lens, k_new, v_new);
}

__global__ __launch_bounds__(kAppendThreads) void append_token_kernel(
    uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t D, int32_t S, int32_t T,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new, int32_t page_size)
{
    append_token_block((int32_t)blockIdx.x, layer_base, page_stride, num_pages, Hkv, D, S, T, block_tables, max_blocks,
                       ctx_lens, cu_q_lens, k_new, v_new, page_size);
}

// A step with both chunks and single tokens (a mixed batch): the workgroups of the chunk path
// first, those of the single-token path behind them, in one launch (the calls are launch-bound
// at the batch sizes of a serving step, so the second launch was a third of the time).
template <int PS>
__global__ __launch_bounds__(kAppendThreads) void append_mixed_kernel(
    uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t D, int32_t S, int32_t T,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new, uint32_t page_blocks)
{
    if (blockIdx.x < page_blocks)
        append_page_block<PS>((int32_t)blockIdx.x, layer_base, page_stride, num_pages, Hkv, D, S, block_tables, max_blocks,
                              ctx_lens, cu_q_lens, k_new, v_new);
    else
        append_token_block((int32_t)(blockIdx.x - page_blocks), layer_base, page_stride, num_pages, Hkv, D, S, T,
                           block_tables, max_blocks, ctx_lens, cu_q_lens, k_new, v_new, PS);
}

int launch_append(const cs_kv_pool& pool, int32_t layer, const cs_batch& b,
                  const void* k_new, const void* v_new, hipStream_t st)
{
    if (b.num_tokens == 0) return CS_OK;
    bool any_single = false, any_chunk = false;
    for (int32_t s = 0; s < b.num_seqs; ++s) {
        const int32_t ql = b.h_cu_q_lens[s + 1] - b.h_cu_q_lens[s];
        any_single |= ql == 1;
        any_chunk |= ql > 1;
    }
    uint16_t* layer_base = (uint16_t*)pool.base + (int64_t)layer * pool.layer_stride;
    const int64_t slots = (((int64_t)(b.num_tokens >> kAppendSlotShift) + 2ll * b.num_seqs) + 7) & ~7ll;   // whole groups of 8
    const int64_t page_blocks = any_chunk ? slots * pool.num_kv_heads : 0;
    const int64_t units = (int64_t)b.num_tokens * pool.num_kv_heads * (pool.head_dim / 8);
    const int64_t token_blocks = any_single ? (units + kAppendThreads - 1) / kAppendThreads : 0;
    if (page_blocks + token_blocks > 2147483647ll) return CS_ERR_UNSUPPORTED;
    const uint16_t* kn = (const uint16_t*)k_new;
    const uint16_t* vn = (const uint16_t*)v_new;
    if (any_chunk && any_single) {
        const dim3 grid((uint32_t)(page_blocks + token_blocks));
        if (pool.page_size == 16)
            hipLaunchKernelGGL(append_mixed_kernel<16>, grid, dim3(kAppendThreads), 0, st,
                               layer_base, pool.page_stride, pool.num_pages, pool.num_kv_heads, pool.head_dim,
                               b.num_seqs, b.num_tokens, b.block_tables, b.max_blocks_per_seq, b.ctx_lens, b.cu_q_lens,
                               kn, vn, (uint32_t)page_blocks);
        else
            hipLaunchKernelGGL(append_mixed_kernel<8>, grid, dim3(kAppendThreads), 0, st,
                               layer_base, pool.page_stride, pool.num_pages, pool.num_kv_heads, pool.head_dim,
                               b.num_seqs, b.num_tokens, b.block_tables, b.max_blocks_per_seq, b.ctx_lens, b.cu_q_lens,
                               kn, vn, (uint32_t)page_blocks);
    } else if (any_chunk) {
        if (pool.page_size == 16)
            hipLaunchKernelGGL(append_page_kernel<16>, dim3((uint32_t)page_blocks), dim3(kAppendThreads), 0, st,
                               layer_base, pool.page_stride, pool.num_pages, pool.num_kv_heads, pool.head_dim,
                               b.num_seqs, b.block_tables, b.max_blocks_per_seq, b.ctx_lens, b.cu_q_lens, kn, vn);
        else
            hipLaunchKernelGGL(append_page_kernel<8>, dim3((uint32_t)page_blocks), dim3(kAppendThreads), 0, st,
                               layer_base, pool.page_stride, pool.num_pages, pool.num_kv_heads, pool.head_dim,
                               b.num_seqs, b.block_tables, b.max_blocks_per_seq, b.ctx_lens, b.cu_q_lens, kn, vn);
    } else if (any_single) {
        hipLaunchKernelGGL(append_token_kernel, dim3((uint32_t)token_blocks), dim3(kAppendThreads), 0, st,
                           layer_base, pool.page_stride, pool.num_pages, pool.num_kv_heads, pool.head_dim,
                           b.num_seqs, b.num_tokens, b.block_tables, b.max_blocks_per_seq, b.ctx_lens,
                           b.cu_q_lens, kn, vn, pool.page_size);
    }
    return check_launch("append kernels");
}

}  // namespace cs
