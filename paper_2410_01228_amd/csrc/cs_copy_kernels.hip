// Copy kernels: KV append into pages, checkpoint gather / restore of whole pages, and a
// plain copy used as the bandwidth ceiling.  All are HBM-bound streams of 16-byte lanes.
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
    int32_t num_pages, int32_t layer_begin, const int32_t* __restrict__ ids, int32_t n,
    char* __restrict__ staging, int32_t page_bytes, int32_t chunks_per_page)
{
    // grid.x = n * chunks_per_page (page-major), grid.y = layers
    const int32_t i = blockIdx.x / chunks_per_page;
    const int32_t c = blockIdx.x - i * chunks_per_page;
    const int32_t l = blockIdx.y;
    const int32_t id = ids[i];
    if (id < 0 || id >= num_pages) return;                       // never touch a bad page id
    char* p = pool_base + (int64_t)(layer_begin + l) * layer_stride_b + (int64_t)id * page_stride_b;
    char* s = staging + ((int64_t)l * n + i) * (int64_t)page_bytes;
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
                     const int32_t* ids, int32_t n, void* staging, bool to_staging, hipStream_t st)
{
    const int32_t layers = layer_end - layer_begin;
    if (n == 0 || layers == 0) return CS_OK;
    const int32_t page_bytes = (int32_t)cs_page_bytes(pool.num_kv_heads, pool.head_dim);
    const int32_t cpp = (page_bytes + kChunkBytes - 1) / kChunkBytes;
    dim3 grid((uint32_t)n * cpp, (uint32_t)layers);
    if (to_staging)
        hipLaunchKernelGGL(page_copy_kernel<true>, grid, dim3(kCopyThreads), 0, st,
                           (char*)pool.base, pool.layer_stride * 2, pool.page_stride * 2, pool.num_pages,
                           layer_begin, ids, n, (char*)staging, page_bytes, cpp);
    else
        hipLaunchKernelGGL(page_copy_kernel<false>, grid, dim3(kCopyThreads), 0, st,
                           (char*)pool.base, pool.layer_stride * 2, pool.page_stride * 2, pool.num_pages,
                           layer_begin, ids, n, (char*)staging, page_bytes, cpp);
    return check_launch("page_copy_kernel");
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
// single new token go through append_token_kernel below instead.  Wavefront w moves features 32w .. 32w+31:
//   K: lane (feature block dl = lane/16, token = lane%16) loads 16 bytes of its token's row
//      and stores them to unit (dblk*16 + token) -- consecutive lanes, consecutive units;
//   V: lane (tile, token half, feature pair) loads one dword (two features) from each of the
//      half's 8 token rows, regroups them into two 16-byte units (one feature x 8 tokens
//      each) and stores 32 consecutive bytes.
// Workgroup slots are dealt to sequences as start(s) = cu_q_lens[s]/16 + 2s (a step of q
// tokens touches at most q/16 + 2 pages), found by bisection.
// ------------------------------------------------------------------------------------
constexpr int kAppendThreads = 256;

__global__ __launch_bounds__(kAppendThreads) void append_page_kernel(
    uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t D, int32_t S,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new)
{
    const int32_t h = blockIdx.x % Hkv;
    const int32_t slot_id = blockIdx.x / Hkv;
    int32_t lo = 0, hi = S;                                       // largest s with start(s) <= slot_id
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if ((cu_q_lens[mid] >> 4) + 2 * mid <= slot_id) lo = mid; else hi = mid;
    }
    const int32_t s = lo;
    const int32_t t_seq = cu_q_lens[s];
    const int32_t first = ctx_lens[s];                            // the step fills positions [first, last)
    const int32_t last = first + (cu_q_lens[s + 1] - t_seq);
    if (last - first == 1) return;                               // single tokens: append_token_kernel
    const int32_t blk = (first >> 4) + (slot_id - ((t_seq >> 4) + 2 * s));
    const int32_t p0 = blk << 4;                                  // first position of the page
    if (p0 >= last || blk >= max_blocks) return;
    const int32_t page = block_tables[(int64_t)s * max_blocks + blk];
    if (page < 0 || page >= num_pages) return;
    const int32_t block_elems = kPage * D;
    uint16_t* kblk = layer_base + (int64_t)page * page_stride + (int64_t)h * block_elems;
    uint16_t* vblk = kblk + (int64_t)Hkv * block_elems;
    const int64_t row = (int64_t)Hkv * D;                         // elements between consecutive tokens
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (wave * 32 >= D) return;                                   // head_dim 64: two wavefronts suffice
    // packed token index of page position p0 (may lie before the step's first token)
    const int64_t tok_base = (int64_t)t_seq + (p0 - first);

    {   // K: features wave*32 + dl*8 .. +8 of token lane%16
        const int32_t tok = lane & 15, dblk = wave * 4 + (lane >> 4);
        const int32_t pos = p0 + tok;
        if (pos >= first && pos < last) {
            const u32x4 v = *(const u32x4*)(k_new + ((tok_base + tok) * Hkv + h) * D + dblk * 8);
            *(u32x4*)(kblk + (dblk * 16 + tok) * 8) = v;
        }
    }
    if (wave * 64 < D) {
        // V: a 16-byte unit is one feature of 8 consecutive tokens.  Lane (tile dtl = lane/16,
        // token half th = (lane/8)%2, feature pair i = lane%8) loads one dword (two features)
        // from each of the half's 8 token rows and regroups them into two units; wavefront w
        // covers features 64w .. 64w+63, the lanes of a (tile, half) write 256 consecutive bytes.
        const int32_t dt = wave * 4 + (lane >> 4), th = (lane >> 3) & 1, i = lane & 7;
        const int32_t pos = p0 + th * 8;                          // first position of the half
        const uint16_t* src = v_new + ((tok_base + th * 8) * Hkv + h) * D + dt * 16 + 2 * i;
        uint16_t* dst = vblk + ((dt * 2 + th) * 16 + 2 * i) * 8;  // two adjacent 16-byte units
        if (pos >= first && pos + 8 <= last) {
            uint32_t w[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) w[j] = *(const uint32_t*)(src + j * row);
            u32x4 lo, hi;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                lo[j] = (w[2 * j] & 0xffffu) | (w[2 * j + 1] << 16);          // feature 2i:   tokens 2j, 2j+1
                hi[j] = (w[2 * j] >> 16) | (w[2 * j + 1] & 0xffff0000u);      // feature 2i+1
            }
            *(u32x4*)dst = lo;
            *(u32x4*)(dst + 8) = hi;
        } else {
            // a half the step fills only partly: element by element
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (pos + j >= first && pos + j < last) {
                    const uint32_t w = *(const uint32_t*)(src + j * row);
                    dst[j] = (uint16_t)(w & 0xffffu);
                    dst[8 + j] = (uint16_t)(w >> 16);
                }
            }
        }
    }
}

// Single new tokens (decode): one lane per 16-byte unit (8 features) of the token's K row
// and V row.  The K unit is stored as it is; the V unit is scattered as 8 two-byte stores
// (the V block keeps 8 consecutive TOKENS of one feature together).  Sequences with more
// than one new token are left to append_page_kernel.
__global__ __launch_bounds__(kAppendThreads) void append_token_kernel(
    uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t D, int32_t S, int32_t T,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new)
{
    const int32_t units_per_tok = Hkv * (D >> 3);
    const int64_t gid = (int64_t)blockIdx.x * kAppendThreads + threadIdx.x;
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
    const int32_t blk = pos >> 4;
    if (pos < 0 || blk >= max_blocks) return;
    const int32_t page = block_tables[(int64_t)s * max_blocks + blk];
    if (page < 0 || page >= num_pages) return;
    const int32_t slot = pos & 15;
    const int32_t block_elems = kPage * D;
    uint16_t* kblk = layer_base + (int64_t)page * page_stride + (int64_t)h * block_elems;
    uint16_t* vblk = kblk + (int64_t)Hkv * block_elems;
    const int64_t src = ((int64_t)t * Hkv + h) * D + dblk * 8;
    *(u32x4*)(kblk + (dblk * 16 + slot) * 8) = *(const u32x4*)(k_new + src);
    const u32x4 vv = *(const u32x4*)(v_new + src);
    // feature d = dblk*8 + e  ->  (((d/16)*2 + slot/8)*16 + d%16)*8 + slot%8
    const int32_t vbase = (((dblk >> 1) * 2 + (slot >> 3)) * 16 + (dblk & 1) * 8) * 8 + (slot & 7);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint32_t w = vv[e >> 1];
        vblk[vbase + e * 8] = (uint16_t)((e & 1) ? (w >> 16) : (w & 0xffffu));
    }
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
    if (any_chunk) {
        const int64_t slots = (int64_t)(b.num_tokens >> 4) + 2ll * b.num_seqs;
        const int64_t blocks = slots * pool.num_kv_heads;
        if (blocks > 2147483647ll) return CS_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(append_page_kernel, dim3((uint32_t)blocks), dim3(kAppendThreads), 0, st,
                           layer_base, pool.page_stride, pool.num_pages, pool.num_kv_heads, pool.head_dim,
                           b.num_seqs, b.block_tables, b.max_blocks_per_seq, b.ctx_lens, b.cu_q_lens,
                           (const uint16_t*)k_new, (const uint16_t*)v_new);
    }
    if (any_single) {
        const int64_t units = (int64_t)b.num_tokens * pool.num_kv_heads * (pool.head_dim / 8);
        const uint32_t blocks = (uint32_t)((units + kAppendThreads - 1) / kAppendThreads);
        hipLaunchKernelGGL(append_token_kernel, dim3(blocks), dim3(kAppendThreads), 0, st,
                           layer_base, pool.page_stride, pool.num_pages, pool.num_kv_heads, pool.head_dim,
                           b.num_seqs, b.num_tokens, b.block_tables, b.max_blocks_per_seq, b.ctx_lens,
                           b.cu_q_lens, (const uint16_t*)k_new, (const uint16_t*)v_new);
    }
    return check_launch("append kernels");
}

}  // namespace cs
