// Decode path of the mixed-batch paged attention: one new token per sequence attends its
// whole cached context (paper Sec. 4.2, memory-access term: the KV cache is streamed from
// HBM once).  Split-KV scheme: a workgroup takes one (sequence, kv head, key range), its
// four wavefronts stream the split's pages straight from HBM into MFMA operand registers
// (the page format IS the operand layout, so there is no LDS staging and no shuffle),
// keep an online softmax per query head in fp32, and leave one partial (max, sum,
// unnormalised output) per split; a second kernel merges the splits.
//
// Tile algebra per 16-token page and kv head (G = query heads sharing it, padded to 16):
//   S^T[token][head] = K[token][:] . Q[head][:]      v_mfma_f32_16x16x32_{bf16,f16}, D/32 steps
//   O^T[d][head]    += V^T[d][token] . P^T[token][head]   v_mfma_f32_16x16x16_{bf16,f16}, D/16 tiles
// The C layout of S^T (lane = head + 16*(token/4), register = token%4) is exactly the B
// layout the second product wants, so P never leaves its registers.
#pragma once
#include "cs_common.h"
#include "cs_elem.h"

namespace cs {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kDecodeWaves = 4;
constexpr int kDecodeThreads = kDecodeWaves * 64;

__device__ __forceinline__ float xor_max(float v, int mask) {
    return fmaxf(v, __shfl_xor(v, mask, 64));
}

template <int D>
struct PageRegs {
    u32x4 k[D / 32];     // K block: unit (kk*64 + lane)
    u32x2 v[D / 16];     // V block: tokens 4*(lane/16)..+4 of feature dt*16 + lane%16
};

// The page ids of one 16-key step: one page of 16 tokens, or two pages of 8 (the second
// repeats the first where the sequence ends inside the first: what it brings is masked).
template <int PS> struct StepIds;
template <> struct StepIds<16> { int32_t a; };
template <> struct StepIds<8> { int32_t a, b; };

// Ids of step `step`, or an invalid id when the step lies outside [0, step_end).  n_entries:
// table entries the sequence has.
template <int PS>
__device__ __forceinline__ StepIds<PS> step_ids(const int32_t* __restrict__ table, int32_t step, int32_t step_end,
                                                int32_t n_entries)
{
    StepIds<PS> ids;
    if constexpr (PS == 16) {
        ids.a = step < step_end ? table[step] : -1;
    } else {
        ids.a = step < step_end ? table[2 * step] : -1;
        ids.b = (step < step_end && 2 * step + 1 < n_entries) ? table[2 * step + 1] : ids.a;
    }
    return ids;
}
template <int PS>
__device__ __forceinline__ bool step_ok(const StepIds<PS>& ids, int32_t num_pages) {
    if constexpr (PS == 16) return ids.a >= 0 && ids.a < num_pages;
    else return ids.a >= 0 && ids.a < num_pages && ids.b >= 0 && ids.b < num_pages;
}

// Ids that can always be read: a step outside the range, or one with a bad id, reads page 0 of
// the pool instead (its result is never used).
template <int PS>
__device__ __forceinline__ StepIds<PS> loadable(const StepIds<PS>& ids, int32_t num_pages) {
    StepIds<PS> r = ids;
    if constexpr (PS == 16) {
        r.a = (ids.a >= 0 && ids.a < num_pages) ? ids.a : 0;
    } else {
        const bool good = ids.a >= 0 && ids.a < num_pages && ids.b >= 0 && ids.b < num_pages;
        r.a = good ? ids.a : 0;
        r.b = good ? ids.b : 0;
    }
    return r;
}

template <int D>
__device__ __forceinline__ void load_page(PageRegs<D>& r, const uint16_t* __restrict__ layer_base,
                                          int64_t page_stride, StepIds<16> ids, int32_t g, int32_t Hkv, int lane)
{
    const uint16_t* kblk = layer_base + (int64_t)ids.a * page_stride + (int64_t)g * (kPage * D);
    const uint16_t* vblk = kblk + (int64_t)Hkv * (kPage * D);
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
        r.k[kk] = __builtin_nontemporal_load((const u32x4*)kblk + kk * 64 + lane);
    // V unit (dt*2 + half)*16 + feature holds 8 tokens of one feature; this lane's 4 tokens
    // 4*(lane/16) .. +4 are the 8-byte half (lane/16)%2 of the unit of token half lane/32.  A
    // wavefront load still covers 512 consecutive bytes.
    const int voff = (((lane >> 5) * 16 + (lane & 15)) * 2) + ((lane >> 4) & 1);   // in 8-byte pieces
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
        r.v[dt] = __builtin_nontemporal_load((const u32x2*)vblk + dt * 64 + voff);
}

// The same registers from two pages of 8 tokens: K rows 0..7 (lanes with bit 3 clear) and the
// V units of token half 0 (lanes below 32) come from the first page, the rest from the second.
// Inside a page of 8 tokens a K feature block holds 8 units and a V feature tile 16, so a
// wavefront load still reads two runs of 512 consecutive bytes.
template <int D>
__device__ __forceinline__ void load_page(PageRegs<D>& r, const uint16_t* __restrict__ layer_base,
                                          int64_t page_stride, StepIds<8> ids, int32_t g, int32_t Hkv, int lane)
{
    const int32_t k_id = (lane & 8) ? ids.b : ids.a;
    const int32_t v_id = (lane & 32) ? ids.b : ids.a;
    const uint16_t* kblk = layer_base + (int64_t)k_id * page_stride + (int64_t)g * (8 * D);
    const uint16_t* vblk = layer_base + (int64_t)v_id * page_stride + (int64_t)(Hkv + g) * (8 * D);
    const int koff = (lane >> 4) * 8 + (lane & 7);                 // in 16-byte units
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
        r.k[kk] = __builtin_nontemporal_load((const u32x4*)kblk + kk * 32 + koff);
    const int voff = (lane & 15) * 2 + ((lane >> 4) & 1);         // in 8-byte pieces
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt)
        r.v[dt] = __builtin_nontemporal_load((const u32x2*)vblk + dt * 32 + voff);
}

// One wavefront's running state.
template <int D>
struct WaveState {
    f32x4 o[D / 16];     // O^T tiles: row d = dt*16 + 4*(lane/16) + i, column head = lane%16
    float m;             // running max (log2 domain) of column lane%16
    float l;             // this lane's share of the running sum
};

template <int D, class E>
__device__ __forceinline__ void process_page(WaveState<D>& st, const PageRegs<D>& r, const u32x4* qb,
                                             float scale_log2e, int32_t tok0, int32_t n_keys, int lane)
{
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
        s = E::mfma32(r.k[kk], qb[kk], s);
    const int32_t row0 = tok0 + (lane >> 4) * 4;      // first of this lane's 4 tokens
    const bool tail = tok0 + kPage > n_keys;           // wave-uniform
    float x[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[i] = s[i] * scale_log2e;
        if (tail && row0 + i >= n_keys) x[i] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
    mx = xor_max(mx, 16);
    mx = xor_max(mx, 32);
    const float m_new = fmaxf(st.m, mx);               // finite: token tok0 is always valid
    if (__any(m_new > st.m)) {
        const float alpha = exp2f(st.m - m_new);       // 0 on the first page (m = -inf)
        st.l *= alpha;
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) st.o[dt] *= alpha;
        st.m = m_new;
    }
    float p[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) p[i] = exp2f(x[i] - st.m);
    u32x2 pb = { E::pack(p[0], p[1]), E::pack(p[2], p[3]) };
    // the sum uses the same rounded weights that multiply V
    st.l += E::sum2(pb[0]) + E::sum2(pb[1]);
    if (tail) {
        // slots past the sequence end hold stale bits (possibly NaN): zero them so 0 * x stays 0
        const int32_t valid = n_keys - row0;           // tokens of this lane's group that exist
        const uint32_t m0 = valid >= 2 ? 0xffffffffu : (valid == 1 ? 0x0000ffffu : 0u);
        const uint32_t m1 = valid >= 4 ? 0xffffffffu : (valid == 3 ? 0x0000ffffu : 0u);
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
            u32x2 v = r.v[dt];
            v[0] &= m0; v[1] &= m1;
            st.o[dt] = E::mfma16(v, pb, st.o[dt]);
        }
    } else {
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt)
            st.o[dt] = E::mfma16(r.v[dt], pb, st.o[dt]);
    }
}

// Work items.  A plan kernel turns the batch's lengths into a compact list of
// (sequence, key range) items, so the split kernel launches exactly one workgroup per item
// and kv head: no workgroup starts only to find it has nothing to do, and a long sequence
// and a short one both break into pieces of about the same size.
struct DecodeItem {
    int32_t seq, token, n_keys, key_begin, key_end, n_splits, pad0, pad1;   // 32 bytes
};

// Where a workgroup's item comes from.
struct ItemsInMemory { const DecodeItem* items; };     // written by decode_plan_kernel
struct ItemsIdentity { int32_t unused; };              // no sequence is cut: item x is sequence x

__device__ inline bool fetch_item(const ItemsInMemory& src, int32_t item, const int32_t*, const int32_t*, DecodeItem& it) {
    it = src.items[item];
    return true;
}
__device__ inline bool fetch_item(const ItemsIdentity&, int32_t item, const int32_t* ctx_lens, const int32_t* cu_q_lens, DecodeItem& it) {
    it.seq = item;
    it.token = cu_q_lens[item];
    if (cu_q_lens[item + 1] - it.token != 1) return false;
    it.n_keys = ctx_lens[item] + 1;
    it.key_begin = 0;
    it.key_end = it.n_keys;
    it.n_splits = 1;
    return true;
}
__device__ inline bool fetch_item(const ItemsInArgs& src, int32_t item, const int32_t* ctx_lens, const int32_t* cu_q_lens, DecodeItem& it) {
    const uint32_t w = src.e[item];
    const int32_t piece = (int32_t)((w >> 16) & 0xffu), k = (int32_t)(w >> 24);
    it.seq = (int32_t)(w & 0xffffu);
    it.token = cu_q_lens[it.seq];
    it.n_keys = ctx_lens[it.seq] + 1;
    const int32_t chunk = decode_chunk_keys(it.n_keys, k);
    it.key_begin = k > 1 ? min(it.n_keys, piece * chunk) : 0;
    it.key_end = k > 1 ? min(it.n_keys, (piece + 1) * chunk) : it.n_keys;
    it.n_splits = k;
    return true;
}

// LDS of one decode workgroup: the four wavefronts' partial results, merged at the end.
template <int D>
struct DecodeLds {
    float o[kDecodeWaves][kMaxGroup][D];
    float m[kDecodeWaves][kMaxGroup];
    float l[kDecodeWaves][kMaxGroup];
};

// The work of one decode workgroup: item `item` (a sequence's key range), kv head g; 4
// wavefronts.  Src says where the item list is: in memory, in the kernel arguments, or
// nowhere (item x is sequence x, and the workgroup leaves at once if that sequence is not a
// decode).  kAhead: pages a wavefront keeps in flight beyond the one it multiplies (1 or 2; a
// page is 32 registers, so 2 costs the third workgroup per CU: it pays for long items on a
// full grid, not for short ones on a small grid).
// kCountedLoads: how a step without a page (past the end of the range, or a bad id) is handled.
// false: its loads are skipped.  The compiler cannot count loads behind a branch, so it waits for
// everything in flight before each multiply: every page's loads are issued early, but a
// wavefront never computes while its own loads fly.  On a grid that fills the chip (several
// workgroups per CU) that is the faster form (2-3% on the decode workloads): the other
// workgroups cover the wait, and no load is wasted.  true: such a step loads page 0 instead, all
// loads are straight-line code, and the compiler waits only for the page about to be multiplied,
// so ONE workgroup per CU streams at 26-48 GB/s instead of 17: what a decode workgroup that
// shares its CU with a prefill tile needs.
template <int D, class Src, class E, int kAhead, int PS, bool kCountedLoads = false>
__device__ __forceinline__ void decode_item(
    DecodeLds<D>& lds,
    const uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t G,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const Src& src,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ q, uint16_t* __restrict__ out,
    float scale_log2e, float* __restrict__ part_o, float* __restrict__ part_ml,
    int32_t item, int32_t g)
{
    DecodeItem it;
    if (!fetch_item(src, item, ctx_lens, cu_q_lens, it)) return;
    const int32_t s = it.seq, t = it.token, n_keys = it.n_keys;
    // steps of 16 keys: pages of 16 tokens, or pairs of pages of 8
    const int32_t n_entries = min((n_keys + PS - 1) / PS, max_blocks);     // table entries in use
    const int32_t page_begin = it.key_begin >> 4;
    // an item can come out empty when a short sequence is cut very finely
    const int32_t page_end = it.key_end > it.key_begin
        ? min((it.key_end + kPage - 1) >> 4, PS == 16 ? max_blocks : (n_entries + 1) >> 1) : page_begin;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int32_t* table = block_tables + (int64_t)s * max_blocks;
    const int32_t Hq = Hkv * G;

    // Q as the B operand of S^T = K.Q^T: lane (head = lane%16, k-group = lane/16) holds
    // features kk*32 + (lane/16)*8 .. +8 of head g*G + lane%16; heads >= G are zero rows.
    u32x4 qb[D / 32];
    {
        const int head = lane & 15;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            u32x4 v = zero;
            if (head < G)
                v = *(const u32x4*)(q + ((int64_t)t * Hq + g * G + head) * D + kk * 32 + (lane >> 4) * 8);
            qb[kk] = v;
        }
    }

    WaveState<D> st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) st.o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    static_assert(kAhead == 1 || kAhead == 2, "one or two pages ahead");
    auto fetch = [&](PageRegs<D>& r, const StepIds<PS>& id) {
        if constexpr (kCountedLoads) {
            load_page<D>(r, layer_base, page_stride, loadable<PS>(id, num_pages), g, Hkv, lane);
        } else {
            if (step_ok<PS>(id, num_pages)) load_page<D>(r, layer_base, page_stride, id, g, Hkv, lane);
        }
    };
    if constexpr (kAhead == 1) {
        // wave w streams pages page_begin + w, + w + 4, ...; the next page's loads are in
        // flight while the current page is multiplied
        PageRegs<D> cur, nxt;
        int32_t pg = page_begin + wave;
        auto id_at = [&](int32_t p) { return step_ids<PS>(table, p, page_end, n_entries); };
        auto ok = [&](const StepIds<PS>& id) { return step_ok<PS>(id, num_pages); };
        StepIds<PS> id_cur = id_at(pg);
        StepIds<PS> id_nxt = id_at(pg + kDecodeWaves);
        fetch(cur, id_cur);
        while (pg < page_end) {
            const int32_t pg_n = pg + kDecodeWaves;
            const StepIds<PS> id_n2 = id_at(pg_n + kDecodeWaves);
            fetch(nxt, id_nxt);
            if (ok(id_cur))
                process_page<D, E>(st, cur, qb, scale_log2e, pg << 4, n_keys, lane);
            cur = nxt;
            id_cur = id_nxt;
            id_nxt = id_n2;
            pg = pg_n;
        }
    } else {
        // wave w streams pages page_begin + w, + w + 4, ...; the loads of the next two pages are
        // in flight while the current page is multiplied
        PageRegs<D> b0, b1, b2;
        int32_t pg = page_begin + wave;
        auto id_at = [&](int32_t p) { return step_ids<PS>(table, p, page_end, n_entries); };
        auto ok = [&](const StepIds<PS>& id) { return step_ok<PS>(id, num_pages); };
        StepIds<PS> id0 = id_at(pg), id1 = id_at(pg + kDecodeWaves), id2 = id_at(pg + 2 * kDecodeWaves);
        fetch(b0, id0);
        fetch(b1, id1);
        auto stage = [&](PageRegs<D>& use, PageRegs<D>& fill) {
            const StepIds<PS> id3 = id_at(pg + 3 * kDecodeWaves);
            fetch(fill, id2);
            if (ok(id0)) process_page<D, E>(st, use, qb, scale_log2e, pg << 4, n_keys, lane);
            id0 = id1; id1 = id2; id2 = id3;
            pg += kDecodeWaves;
        };
        while (pg < page_end) {
            stage(b0, b2);
            if (pg >= page_end) break;
            stage(b1, b0);
            if (pg >= page_end) break;
            stage(b2, b1);
        }
    }
    st.l += __shfl_xor(st.l, 16, 64);
    st.l += __shfl_xor(st.l, 32, 64);

    // merge the four wavefronts through LDS
    auto& sh_o = lds.o;
    auto& sh_m = lds.m;
    auto& sh_l = lds.l;
    {
        const int head = lane & 15;
        if (head < G) {
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    sh_o[wave][head][dt * 16 + (lane >> 4) * 4 + i] = st.o[dt][i];
            if (lane < 16) { sh_m[wave][head] = st.m; sh_l[wave][head] = st.l; }
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * D; idx += kDecodeThreads) {
        const int head = idx / D, d = idx - head * D;
        float M = sh_m[0][head];
#pragma unroll
        for (int w = 1; w < kDecodeWaves; ++w) M = fmaxf(M, sh_m[w][head]);
        float L = 0.f, O = 0.f;
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            const float mw = sh_m[w][head];
            const float f = mw == -INFINITY ? 0.f : exp2f(mw - M);     // a wavefront without pages
            L += sh_l[w][head] * f;
            O += sh_o[w][head][d] * f;
        }
        const int32_t hq = g * G + head;
        if (it.n_splits == 1) {
            const float r = L > 0.f ? O / L : 0.f;                    // no key at all (every page id bad): zeros
            out[((int64_t)t * Hq + hq) * D + d] = (uint16_t)(E::pack(r, 0.f) & 0xffffu);
        } else {
            const int64_t slot = (int64_t)item * Hq + hq;
            part_o[slot * D + d] = O;
            if (d == 0) { part_ml[slot * 2] = M; part_ml[slot * 2 + 1] = L; }
        }
    }
}

}  // namespace cs
