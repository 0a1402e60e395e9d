// Prefill-chunk path of the mixed-batch paged attention: q_s > 1 new tokens of a sequence
// attend its prior context and, causally, their own chunk (paper Sec. 4.2: the attention
// term grows as P(P+C); chunked prefill).  Compute-bound, so the tiles run on the 16-bit
// (bf16 or f16) matrix cores with an fp32 online softmax.
//
// A workgroup (4 wavefronts) owns one kv head and kTileCols "column tiles" of 16 query rows
// each (16 consecutive chunk tokens of one of the G query heads sharing the kv head; tiles
// are numbered token-block major, so any G packs without waste), kNCT per wavefront; two
// workgroups share a CU.  It walks the sequence's keys 32 at a time
// (two pages).  The pages' K and V blocks are copied global -> LDS by LDS-DMA loads into a
// ring of slots several steps ahead (one barrier per step, no staging registers); every
// wavefront reads them back as MFMA operands -- a page's 16-byte units are operand
// fragments, and the copy places them so that the LDS reads are linear in the lane id -- and
//   S^T[key][query]   = K . Q^T                      v_mfma_f32_16x16x32_{bf16,f16}
//   O^T[d][query]    += V^T[d][32 keys] . P^T        v_mfma_f32_16x16x32_{bf16,f16}
// with P^T taken straight from the S^T accumulators of the two pages (their C layout is
// the B layout of the second product).  The softmax denominators come from one more MFMA
// per tile with an all-ones A operand, so they sum exactly the rounded weights that multiply V.
//
// The loop is software-pipelined: iteration i exponentiates the scores of step i and
// multiplies them with V(i) while the matrix cores already compute the scores of step
// i+1, so the exp/convert work of one step overlaps the MFMAs of the next.  The running
// maximum is only raised (and the accumulators rescaled) when a new score exceeds it by
// more than 2^kLazyLog2, which keeps the rescale out of the steady-state loop.
#pragma once
#include "cs_common.h"
#include "cs_elem.h"
#include <algorithm>
#include <type_traits>

namespace cs {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// (kPrefillWaves, kPrefillThreads, kNCT, kKeysPerStep, kTileCols and prefill_slot_start are in
// cs_common.h: the host's launch plan uses them too)
constexpr float kLazyLog2 = 6.0f;             // weights may reach 2^6 before the max is raised
constexpr float kNoMax = -1.0e30f;            // "no score seen yet": finite, so that -inf minus it stays -inf
constexpr int kRing = 4;                      // LDS slots for K and for V steps (copies kRing-1 steps ahead)

// s_waitcnt on the vector-memory counter alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// LDS-DMA (global_load_lds_dwordx4): every active lane's 16 bytes go from global memory
// straight to LDS at base + lane*16, where the wave-uniform base travels in M0.  Written as
// inline assembly so that the compiler's wait-count pass does not see the loads: it cannot
// tell which ring slot a later LDS read touches and would drain the whole copy queue
// (vmcnt(0)) before every read.  The waits are placed by hand with wait_vmcnt<>() instead.
//
// Two LDS-DMA loads for one run of 64 LDS units whose lanes read from two different pages:
// the lanes in mask_a fetch from base_a + off, the others from base_b + off (off = this
// lane's byte offset inside a page's K or V block).  Scalar bases and a per-lane 32-bit
// offset keep all address arithmetic out of the vector ALU; EXEC is narrowed to each lane
// set in turn -- the caller's active lanes inside mask_a, then those outside it -- and put
// back as it was found.  (Every caller here runs with all 64 lanes active, and the counting of
// outstanding copies relies on both instructions being issued; under divergent control flow
// the block would still touch only the caller's lanes.)  The scalar logic instructions write
// SCC, hence the clobber: without it the compiler may keep the carry of a 64-bit address
// addition alive across this block (s_add_u32 before it, s_addc_u32 after it), and the address
// that comes out is 4 GiB off.
__device__ __forceinline__ void lds_dma16_two_pages(const void* base_a, const void* base_b, uint32_t off,
                                                    uint64_t mask_a, void* dst_wave_base) {
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)dst_wave_base;
    uint64_t saved_exec;
    asm volatile("s_mov_b64 %0, exec\n\t"
                 "s_mov_b32 m0, %1\n\t"
                 "s_and_b64 exec, %0, %5\n\t"
                 "global_load_lds_dwordx4 %2, %3\n\t"
                 "s_andn2_b64 exec, %0, %5\n\t"
                 "global_load_lds_dwordx4 %2, %4\n\t"
                 "s_mov_b64 exec, %0"
                 : "=&s"(saved_exec)
                 : "s"(lds_addr), "v"(off), "s"(base_a), "s"(base_b), "s"(mask_a) : "memory", "m0", "scc");
}

// One LDS-DMA load whose lanes bring their own 64-bit global addresses (+ kImm bytes).  The
// instruction's immediate offset moves BOTH ends of the copy -- the global address and the LDS
// address (M0 + offset + lane*16) -- so M0 is set kImm short of the destination.  The s_nop
// keeps the write of M0 one wait state away from the load that reads it.
template <int kImm>
__device__ __forceinline__ void lds_dma16_lane_addr(uint64_t addr, void* dst_wave_base) {
    static_assert(kImm >= 0 && kImm < 4096, "immediate offset field");
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)dst_wave_base - kImm;
    asm volatile("s_mov_b32 m0, %0\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %1, off offset:%2"
                 :: "s"(lds_addr), "v"(addr), "n"(kImm) : "memory", "m0");
}

// max(a, b, c) in one instruction.  fmaxf() makes the compiler canonicalise every operand
// first (one extra v_max per value, to quiet signalling NaNs); the scores need no such care.
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float max8(const float (&x)[8]) {
    return max3(max3(x[0], x[1], x[2]), max3(x[3], x[4], x[5]), max3(x[6], x[7], x[7]));
}


// Floats of one key-range partial: kTileCols * 16 query rows of D outputs, max, sum and padding.
template <int D> constexpr int64_t kPartialFloats = (int64_t)kTileCols * 16 * (D + 4);
// The partials of the cut tile in cut position `cut_pos` (0 = the first cut tile in launch order),
// kv head g: max_ranges partials in a row.
template <int D>
__device__ __forceinline__ float* partials_of(float* part, int32_t cut_pos, int32_t Hkv, int32_t g, int32_t max_ranges) {
    return part + ((int64_t)cut_pos * Hkv + g) * max_ranges * kPartialFloats<D>;
}

// LDS of one prefill workgroup: the ring of K and of V steps.
template <int D>
struct PrefillLds {
    u32x4 k[kRing][4 * D];                            // 2 pages x 2*D 16-byte units per step
    u32x4 v[kRing][4 * D];
};

// The work of one prefill workgroup: the tile in slot b, kv head g, key range `range` (a tile
// whose keys need more than range_steps steps is cut into ranges, each leaving a partial in
// part_tile[range], the caller's block of partials for this tile and kv head; range_steps at
// least the tile's steps: the tile is whole and writes the output itself).  `lds` is the
// workgroup's own.  kPriority > 0: the wavefront alternates its issue priority between the
// halves of an iteration, kPriority - 1 in the score half and kPriority in the P.V half (1: for
// grids whose other wavefronts are mostly tiles too, or become so once a decode workgroup per CU
// is done; 2: the same and always above decode wavefronts, which stay at 0; with decode work of
// equal weight queued behind the tiles either costs more than it gains).
template <int D, class E, int kPriority, int PS, bool kLaneAddr16>
__device__ __forceinline__ void prefill_tile(
    PrefillLds<D>& lds,
    const uint16_t* __restrict__ layer_base, int64_t page_stride, int32_t num_pages,
    int32_t Hkv, int32_t G, int32_t S,
    const int32_t* __restrict__ block_tables, int32_t max_blocks,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ cu_q_lens,
    const uint16_t* __restrict__ q, uint16_t* __restrict__ out, float scale_log2e,
    int32_t range_steps, float* __restrict__ part_tile,
    int32_t g, int32_t b, int32_t range)
{
    constexpr int kUnits = D * 2;                     // 16-byte units per K (or V) block of a page
    constexpr int kStepUnits = 2 * kUnits;            // K (or V) units of one step (two pages)
    constexpr int kLoads = kStepUnits / kPrefillThreads;   // 16-byte loads per lane, for K and for V
    constexpr int kStepPages = kKeysPerStep / PS;     // pages of one step: 2 (of 16 tokens) or 4 (of 8)
    // How a copy instruction's lanes find their pages.  Scalar mode: one instruction per page and
    // lane set (EXEC narrowed to the set), page addresses in scalar registers.  Lane mode: every
    // lane fetches the address of its own page from the lane that holds it (ds_bpermute) and one
    // instruction serves all 64 lanes.  Pages of 8 tokens always take lane mode (four lane sets
    // per instruction otherwise: measured 255 against 210 us on the Qwen-7B chunks); with pages of
    // 16 the caller chooses (kLaneAddr16): the prefill kernel alone is up to 2% faster in scalar
    // mode, the fused grid 1-3% faster in lane mode, where the copy instructions share the
    // memory pipeline with the decode items' loads.
    constexpr bool kLaneAddr = PS == 8 || kLaneAddr16;
    constexpr int kStepLoads = (kLaneAddr ? 2 : 2 * kStepPages) * kLoads;   // LDS-DMA instructions per wavefront and step
    constexpr int kPartRow = D + 4;                   // floats per query row of a partial: D outputs, max, sum, pad
    auto& lds_k = lds.k;
    auto& lds_v = lds.v;

    // sequence owning slot b: the largest s with start(s) <= b
    int32_t lo = 0, hi = S;
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (prefill_slot_start(cu_q_lens[mid], mid, G) <= b) lo = mid; else hi = mid;
    }
    const int32_t s = lo;
    const int32_t t_seq = cu_q_lens[s];
    const int32_t q_len = cu_q_lens[s + 1] - t_seq;
    if (q_len <= 1) return;                            // decode and idle sequences: other path
    const int32_t n_ct = ((q_len + 15) >> 4) * G;      // column tiles of the sequence
    const int32_t ct0 = (int32_t)(b - prefill_slot_start(t_seq, s, G)) * kTileCols;
    if (ct0 >= n_ct) return;
    const int32_t tb_min = ct0 / G;                    // first and last token block of the tile
    const int32_t tb_max = (min(ct0 + kTileCols, n_ct) - 1) / G;
    const int32_t C = ctx_lens[s];
    const int32_t n_seq_keys = C + q_len;              // keys the sequence holds after the append
    const int32_t n_keys = C + min(q_len, (tb_max + 1) * 16);   // keys visible to the tile's last token
    const int32_t n_steps = (n_keys + kKeysPerStep - 1) / kKeysPerStep;
    const int32_t first_edge = (C + tb_min * 16 + 1) / kKeysPerStep;   // steps before it need no causal mask
    // key range of this workgroup: a tile whose keys need more than range_steps steps is cut
    // into ranges handled by different workgroups, each leaving a partial (max, sum, output)
    const int32_t n_ranges = (n_steps + range_steps - 1) / range_steps;
    const int32_t step_begin = range * range_steps;
    if (step_begin >= n_steps) return;
    const int32_t step_end = min(n_steps, step_begin + range_steps);
    const int32_t n_pages = min((n_seq_keys + PS - 1) / PS, max_blocks);
    const int32_t* table = block_tables + (int64_t)s * max_blocks;
    const int32_t Hq = Hkv * G;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // kFold (element types that stand it, see cs_elem.h): Q is scaled once by scale*log2(e), so the
    // matrix unit delivers the scores in the exponent's domain, and the score accumulators start
    // from minus the running offset, so exp2 takes them as they come -- no multiply-add per score.
    constexpr bool kFold = E::kScaleFoldsIntoQ;
    // ---- this wavefront's column tiles: ct = wave*4 + c -> (token block, head) ----
    u32x4 qb[kNCT][D / 32];
    int32_t pos_q[kNCT];                               // absolute position of this lane's query
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int c = 0; c < kNCT; ++c) {
        const int32_t ct = ct0 + wave * kNCT + c;
        const int32_t tb = ct / G, hh = ct - tb * G;
        const int32_t tl = tb * 16 + (lane & 15);            // chunk-local token of this column
        const bool valid = ct < n_ct && tl < q_len;
        pos_q[c] = C + tl;
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            u32x4 v = zero4;
            if (valid)
                v = *(const u32x4*)(q + ((int64_t)(t_seq + tl) * Hq + g * G + hh) * D + kk * 32 + (lane >> 4) * 8);
            if constexpr (kFold) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = E::scale2(v[e], scale_log2e);
            }
            qb[c][kk] = v;
        }
    }

    f32x4 o[kNCT][D / 16];
    f32x4 lacc[kNCT];                                  // softmax denominators (every row equal)
    float m_run[kNCT];
    float x[kNCT][8];                                  // raw scores of the current step
#pragma unroll
    for (int c = 0; c < kNCT; ++c) {
        m_run[c] = kNoMax;
        lacc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) o[c][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const u32x4 ones = {E::kOnes, E::kOnes, E::kOnes, E::kOnes};

    // ---- global -> LDS copies (LDS-DMA: each lane hands its 16 bytes straight to LDS at
    // base + lane*16, no staging registers).  Per step and wavefront kLoads instructions for K
    // and kLoads for V; instruction r covers units (r*4 + wave)*64 .. +64 of the step, which
    // lie inside one page.  A page the sequence does not have is replaced by page 0 of the
    // pool: every step issues the same number of instructions (the vmcnt arithmetic below
    // relies on it) and whatever lands is masked where it is used. ----
    // LDS arrangement of a step (two pages A, B; 32 keys), chosen so that every operand read
    // below is linear in the lane id (b128, conflict-free):
    //   K unit ((kk*2 + tile)*4 + kg)*16 + r : features kk*32 + kg*8 .. +8 of row r of tile X
    //     (tile 0) or Y (tile 1).  Row r = 8*page + 4*half + i stands for token
    //     8*half + i (+4 for tile Y) of that page: a lane group of the S^T accumulators then
    //     owns, over X and Y together, 8 CONSECUTIVE tokens of ONE page -- exactly one 16-byte
    //     V unit;
    //   V unit dt*64 + (page*2 + half)*16 + f : feature dt*16 + f, tokens 8*half .. +8 of page.
    // The copy engine takes one global address per lane, so this regrouping costs nothing.
    // per-lane byte offsets of the units this lane copies, inside a page's K block / V block
    uint32_t k_off[kLoads], v_off_lane[kLoads];
#pragma unroll
    for (int r = 0; r < kLoads; ++r) {
        const int unit0 = (r * kPrefillWaves + wave) * 64;
        const int kk = unit0 >> 7, tile = (unit0 >> 6) & 1, kg = lane >> 4, row = lane & 15;
        // pages of 8 tokens: the half is a page of its own (a K feature block holds 8 units, a V
        // feature tile one group of 16)
        const int tok = (PS == 16 ? ((row >> 2) & 1) * 8 : 0) + (row & 3) + 4 * tile;
        k_off[r] = (uint32_t)(((kk * 4 + kg) * PS + tok) * 16);
        const int dt = unit0 >> 6, half = (lane >> 4) & 1, f = lane & 15;
        v_off_lane[r] = (uint32_t)(PS == 16 ? ((dt * 2 + half) * 16 + f) * 16 : (dt * 16 + f) * 16);
    }
    // Page addresses travel in lane registers: lane j of (pgoff_lo, pgoff_hi) holds the byte
    // offset of page idbase + j (this kv head's K block) from the layer base, already checked
    // against the pool size, and a step's two addresses are read out with v_readlane.  So the
    // steady state has no scalar-memory load (whose unordered return would turn every LDS wait
    // into a full lgkmcnt(0)) and no 64-bit multiply.  The registers are refilled once per 32
    // steps; a page the sequence does not have (or a bad id) reads as page 0.
    int32_t idbase = (kStepPages * step_begin) & ~63;
    uint32_t pgoff_lo, pgoff_hi;
    auto load_window = [&]() {
        const int32_t id = idbase + lane < n_pages ? table[idbase + lane] : 0;
        const uint64_t off = ((uint64_t)((id < 0 || id >= num_pages) ? 0 : id) * (uint64_t)page_stride
                              + (uint64_t)g * (PS * D)) * 2;
        pgoff_lo = (uint32_t)off;
        pgoff_hi = (uint32_t)(off >> 32);
        asm volatile("" : "+v"(pgoff_lo), "+v"(pgoff_hi));   // take the load's wait here, not at every readlane
    };
    load_window();
    // lane mode: which of the step's pages this lane's K units and V units come from
    const int kq = PS == 8 ? (lane >> 2) & 3 : (lane >> 3) & 1;
    const int vq = PS == 8 ? lane >> 4 : lane >> 5;
    const uint32_t v_blk_off = (uint32_t)(Hkv * (PS * D) * 2);           // K block -> V block of a page, bytes
    struct StepPages {
        const char* p[kStepPages];                       // scalar mode: the step's pages (this kv head's K block)
        uint64_t k, v;                                   // lane mode: address of this lane's first K unit and V unit
    };
    auto step_pages = [&](int32_t step) -> StepPages {  // addresses of the step's pages
        if (kStepPages * step - idbase >= 64) {          // steps only ever grow
            idbase += 64;
            load_window();
        }
        const int j = kStepPages * step - idbase;
        StepPages pg;
        if constexpr (kLaneAddr) {
            const uint64_t ko = ((uint64_t)(uint32_t)__builtin_amdgcn_ds_bpermute((j + kq) << 2, (int)pgoff_hi) << 32)
                              | (uint64_t)(uint32_t)__builtin_amdgcn_ds_bpermute((j + kq) << 2, (int)pgoff_lo);
            const uint64_t vo = ((uint64_t)(uint32_t)__builtin_amdgcn_ds_bpermute((j + vq) << 2, (int)pgoff_hi) << 32)
                              | (uint64_t)(uint32_t)__builtin_amdgcn_ds_bpermute((j + vq) << 2, (int)pgoff_lo);
            pg.k = (uint64_t)(uintptr_t)layer_base + ko + k_off[0];
            pg.v = (uint64_t)(uintptr_t)layer_base + vo + (v_blk_off + v_off_lane[0]);
            return pg;
        }
#pragma unroll
        for (int e = 0; e < kStepPages; ++e) {
            // (readlane returns a signed int: widen through uint32_t or the low half's sign bit
            // would smear over the high half)
            const uint64_t o = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane(pgoff_hi, j + e) << 32)
                             | (uint64_t)(uint32_t)__builtin_amdgcn_readlane(pgoff_lo, j + e);
            pg.p[e] = (const char*)layer_base + o;
        }
        return pg;
    };
    auto dma_step = [&](int32_t step, StepPages pg) {
        const uint32_t slot = (uint32_t)step % kRing;
        const int64_t v_blk = (int64_t)Hkv * (PS * D) * 2;                // K block -> V block of a page, bytes
        if constexpr (kLaneAddr) {
            // the second instruction's units lie a fixed 128 * PS bytes behind the first's, in the
            // K block (two feature-block groups on) and in the V block (four feature tiles on) alike
            lds_dma16_lane_addr<0>(pg.k, &lds_k[slot][wave * 64]);
            lds_dma16_lane_addr<0>(pg.v, &lds_v[slot][wave * 64]);
            if constexpr (kLoads > 1) {
                static_assert(kLoads <= 2, "one immediate offset");
                lds_dma16_lane_addr<128 * PS>(pg.k, &lds_k[slot][(kPrefillWaves + wave) * 64]);
                lds_dma16_lane_addr<128 * PS>(pg.v, &lds_v[slot][(kPrefillWaves + wave) * 64]);
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < kLoads; ++r) {
            const int unit0 = (r * kPrefillWaves + wave) * 64;            // wave-uniform
            static_assert(kLaneAddr || PS == 16, "scalar mode is written for two pages per step");
            // K rows 0..7 of a tile come from the first page, rows 8..15 from the second
            lds_dma16_two_pages(pg.p[0], pg.p[1], k_off[r], 0x00ff00ff00ff00ffull, &lds_k[slot][unit0]);
            // V lanes 0..31 hold the first page's two halves, lanes 32..63 the second page's
            lds_dma16_two_pages(pg.p[0] + v_blk, pg.p[1] + v_blk, v_off_lane[r], 0x00000000ffffffffull, &lds_v[slot][unit0]);
        }
    };

    // Raw scores of one step (before the softmax scale).  With hi = lane/16: xs[c][0..3] are
    // rows 4*hi + i of tile X, xs[c][4..7] of tile Y, i.e. together the 8 consecutive keys
    // 32*step + 16*(hi/2) + 8*(hi%2) + 0..7.  Masked entries become -inf.
    // K operands of the step whose scores are computed next.  They are fetched from LDS one
    // phase ahead (while the P.V products of the previous step run), so that the score
    // products never wait for an LDS round trip.
    // kFold: minus the offset the score accumulators start from -- the running maximum once a
    // score has been seen, 0 before (m_run is then still the "none yet" mark)
    f32x4 neg_off[kNCT];
#pragma unroll
    for (int c = 0; c < kNCT; ++c) neg_off[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    u32x4 kreg[2 * (D / 32)];
    auto load_k = [&](int32_t step) {
        const u32x4* kA = &lds_k[(uint32_t)step % kRing][0];
#pragma unroll
        for (int u = 0; u < 2 * (D / 32); ++u) kreg[u] = kA[u * 64 + lane];   // (kk*2 + tile)
    };
    auto scores = [&](auto masked, int32_t step, float (&xs)[kNCT][8]) {
        constexpr bool kMask = decltype(masked)::value;
        f32x4 s0[kNCT], s1[kNCT];
#pragma unroll
        for (int c = 0; c < kNCT; ++c) {
            if constexpr (kFold) { s0[c] = neg_off[c]; s1[c] = neg_off[c]; }
            else { s0[c] = f32x4{0.f, 0.f, 0.f, 0.f}; s1[c] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        }
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
#pragma unroll
            for (int c = 0; c < kNCT; ++c) {
                s0[c] = E::mfma32(kreg[kk * 2 + 0], qb[c][kk], s0[c]);   // tile X
                s1[c] = E::mfma32(kreg[kk * 2 + 1], qb[c][kk], s1[c]);   // tile Y
            }
        }
        const int32_t key0 = step * kKeysPerStep + (lane >> 5) * 16 + ((lane >> 4) & 1) * 8;
#pragma unroll
        for (int c = 0; c < kNCT; ++c) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xs[c][i] = s0[c][i];
                xs[c][4 + i] = s1[c][i];
                if (kMask) {
                    if (key0 + i > pos_q[c]) xs[c][i] = -INFINITY;
                    if (key0 + 4 + i > pos_q[c]) xs[c][4 + i] = -INFINITY;
                }
            }
        }
    };
    // Lazy running maximum.  m_run[c] is the (log2-domain) offset all four lane groups of a
    // column use; it only has to bound the scores loosely.  The hot path merely tests this
    // lane's raw scores against thr[c] = (m_run[c] + kLazyLog2) / scale; the cross-lane maximum
    // and the rescale of the accumulators run only when some lane trips the test.
    float thr[kNCT];
#pragma unroll
    for (int c = 0; c < kNCT; ++c) thr[c] = -INFINITY;
    const float inv_scale = 1.f / scale_log2e;
    auto raise_max = [&](float (&xs)[kNCT][8]) {
        bool need = false;
#pragma unroll
        for (int c = 0; c < kNCT; ++c) {
            need |= max8(xs[c]) > thr[c];
        }
        if (__any(need)) {
#pragma unroll
            for (int c = 0; c < kNCT; ++c) {
                float m = max8(xs[c]);
                m = fmaxf(m, __shfl_xor(m, 16, 64));
                m = fmaxf(m, __shfl_xor(m, 32, 64));
                if constexpr (kFold) {
                    // xs are relative to the offset the accumulators started from; thr likewise
                    // (-inf until a score has been seen, the lazy margin after)
                    const float off = -neg_off[c][0];
                    const float m_new = fmaxf(m_run[c], off + m);
                    const float alpha = __builtin_amdgcn_exp2f(m_run[c] - m_new);
                    lacc[c] *= alpha;
#pragma unroll
                    for (int dt = 0; dt < D / 16; ++dt) o[c][dt] *= alpha;
                    m_run[c] = m_new;
                    const bool seen = m_new > kNoMax;
                    const float off_new = seen ? m_new : 0.f;
                    const float d = off_new - off;
#pragma unroll
                    for (int j = 0; j < 8; ++j) xs[c][j] -= d;             // -inf stays -inf
                    neg_off[c] = f32x4{-off_new, -off_new, -off_new, -off_new};
                    thr[c] = seen ? kLazyLog2 : -INFINITY;
                } else {
                    const float m_new = fmaxf(m_run[c], m * scale_log2e);
                    const float alpha = __builtin_amdgcn_exp2f(m_run[c] - m_new);   // 0 while m_run is -inf
                    lacc[c] *= alpha;
#pragma unroll
                    for (int dt = 0; dt < D / 16; ++dt) o[c][dt] *= alpha;
                    m_run[c] = m_new;
                    thr[c] = (m_new + kLazyLog2) * inv_scale;
                }
            }
        }
    };

    // ---- prologue: the first kRing-1 steps of the range in flight, the first two landed,
    // scores of the first step, K operands of the second ----
#pragma unroll
    for (int j = 0; j < kRing - 1; ++j) dma_step(step_begin + j, step_pages(step_begin + j));
    StepPages pg_next = step_pages(step_begin + kRing - 1);       // pages of the step issued next
    wait_vmcnt<(kRing - 3) * kStepLoads>();
    __syncthreads();
    load_k(step_begin);
    scores(std::true_type{}, step_begin, x);
    raise_max(x);
    load_k(step_begin + 1);

    // ---- iteration i.  First half: scores of step i+1 (into xn, from the K operands already in
    // registers) side by side with the weights of step i (from xc); the V operands of step i
    // leave LDS meanwhile.  Then the barrier: every wavefront is done reading V(i) and K(i+1),
    // and K(i+2), V(i+1) have landed.  Second half: O += V(i) P(i) while the K operands of step
    // i+2 are fetched and the new scores are tested against the running maxima.
    // kMask: causal / end-of-sequence masking (needed from the first edge step on);
    // kLast: there is no step i+1. ----
    auto iteration = [&](auto masked, auto last, int32_t i, float (&xc)[kNCT][8], float (&xn)[kNCT][8]) {
        constexpr bool kMask = decltype(masked)::value;
        constexpr bool kLast = decltype(last)::value;
        // step i+kRing-1 goes into the slot step i-1 left (its last reader finished before the
        // barrier inside iteration i-1)
        // First half at low, second half at high issue priority.  The two wavefronts that share
        // a SIMD (one of each resident workgroup) then settle one half apart: the one in its P.V
        // half gets the matrix pipe whenever it asks, the exp / convert work of the other fills
        // the issue slots in between (measured: 7-9% on every shape).
        if (kPriority) __builtin_amdgcn_s_setprio(kPriority - 1);
        dma_step(i + kRing - 1, pg_next);
        pg_next = step_pages(i + kRing);               // consumed by the next iteration

        if (!kLast) scores(masked, i + 1, xn);
        u32x4 pb[kNCT];
#pragma unroll
        for (int c = 0; c < kNCT; ++c) {
            float p[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                p[j] = kFold ? __builtin_amdgcn_exp2f(xc[c][j])
                             : __builtin_amdgcn_exp2f(__builtin_fmaf(xc[c][j], scale_log2e, -m_run[c]));
            pb[c] = u32x4{ E::pack(p[0], p[1]), E::pack(p[2], p[3]), E::pack(p[4], p[5]), E::pack(p[6], p[7]) };
        }
        const u32x4* vA = &lds_v[(uint32_t)i % kRing][0];
        // V slots at or past the end of the sequence hold stale bits (or nothing at all): zero
        // them so that a zero weight times the slot stays zero.  The lane's unit holds the 8
        // tokens 32*i + 16*(hi/2) + 8*(hi%2) + 0..7, two per dword.
        uint32_t vm[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
        if (kMask && (i + 1) * kKeysPerStep > n_seq_keys) {
            const int32_t valid = n_seq_keys - (i * kKeysPerStep + (lane >> 5) * 16 + ((lane >> 4) & 1) * 8);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                vm[j] = valid >= 2 * j + 2 ? 0xffffffffu : (valid == 2 * j + 1 ? 0x0000ffffu : 0u);
        }
        u32x4 av[D / 16];
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
            av[dt] = vA[dt * 64 + lane];
            if (kMask) { av[dt][0] &= vm[0]; av[dt][1] &= vm[1]; av[dt][2] &= vm[2]; av[dt][3] &= vm[3]; }
        }
        if (!kMask && !kLast) {
            // steady state, first half: tell the scheduler the order we want.  The exp / convert
            // work of step i runs under the score MFMAs of step i+1, and the V operands are
            // fetched under them too.
            constexpr int kQK = 2 * kNCT * (D / 32);
            __builtin_amdgcn_sched_group_barrier(0x002, 4 * kNCT, 0);            // VALU
#pragma unroll
            for (int r = 0; r < kQK; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);               // 1 MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);               // 2 VALU
                if (r < D / 16) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // V: one ds_read_b128
            }
        }
        // K(i+2) and V(i+1) must have landed before anyone reads them: all but the copies of
        // the last kRing-3 steps issued
        __builtin_amdgcn_sched_barrier(0);             // nothing may move across the two halves
        wait_vmcnt<(kRing - 3) * kStepLoads>();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);

        if (kPriority) __builtin_amdgcn_s_setprio(kPriority);
        if (!kLast) load_k(i + 2);
#pragma unroll
        for (int c = 0; c < kNCT; ++c)
            lacc[c] = E::mfma32(ones, pb[c], lacc[c]);
#pragma unroll
        for (int dt = 0; dt < D / 16; ++dt) {
#pragma unroll
            for (int c = 0; c < kNCT; ++c)
                o[c][dt] = E::mfma32(av[dt], pb[c], o[c][dt]);
        }
        if (!kMask && !kLast) {
            // second half: the threshold test of the new scores and the K fetches run under the
            // P.V MFMAs
            constexpr int kPV = kNCT + kNCT * (D / 16);
#pragma unroll
            for (int r = 0; r < kPV; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
                if (r >= 2 && r < 2 + 2 * (D / 32)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // K: one ds_read_b128
            }
        }
        if (!kLast) raise_max(xn);
    };
    float xb[kNCT][8];
    int32_t i = step_begin;
    // steady state in pairs, the scores ping-ponging between x and xb; step i+2 fully visible
    for (; i + 2 < min(first_edge, step_end); i += 2) {
        iteration(std::false_type{}, std::false_type{}, i, x, xb);
        iteration(std::false_type{}, std::false_type{}, i + 1, xb, x);
    }
    for (; i + 1 < step_end; ++i) {
        iteration(std::true_type{}, std::false_type{}, i, x, xb);
#pragma unroll
        for (int c = 0; c < kNCT; ++c)
#pragma unroll
            for (int j = 0; j < 8; ++j) x[c][j] = xb[c][j];
    }
    iteration(std::true_type{}, std::true_type{}, i, x, xb);
    if (kPriority) __builtin_amdgcn_s_setprio(0);
    wait_vmcnt<0>();                                   // no copy may outlive the workgroup's LDS

    // ---- store: lane holds 4 consecutive features of one query row per tile ----
    if (n_ranges == 1) {
#pragma unroll
        for (int c = 0; c < kNCT; ++c) {
            const int32_t ct = ct0 + wave * kNCT + c;
            const int32_t tb = ct / G, hh = ct - tb * G;
            const int32_t tl = tb * 16 + (lane & 15);
            if (ct < n_ct && tl < q_len) {
                const float inv = 1.f / lacc[c][0];
                uint16_t* dst = out + ((int64_t)(t_seq + tl) * Hq + g * G + hh) * D + (lane >> 4) * 4;
#pragma unroll
                for (int dt = 0; dt < D / 16; ++dt) {
                    u32x2 w = { E::pack(o[c][dt][0] * inv, o[c][dt][1] * inv),
                                E::pack(o[c][dt][2] * inv, o[c][dt][3] * inv) };
                    *(u32x2*)(dst + dt * 16) = w;
                }
            }
        }
    } else {
        // partial of this key range: unnormalised output, running max and sum per query row
        if (part_tile == nullptr) return;                 // (a cut tile always has a block: a planning error must not write)
        float* wg = part_tile + (int64_t)range * (kTileCols * 16 * kPartRow);
#pragma unroll
        for (int c = 0; c < kNCT; ++c) {
            float* row = wg + ((wave * kNCT + c) * 16 + (lane & 15)) * kPartRow;
#pragma unroll
            for (int dt = 0; dt < D / 16; ++dt) *(f32x4*)(row + dt * 16 + (lane >> 4) * 4) = o[c][dt];
            if (lane < 16) { row[D] = m_run[c]; row[D + 1] = lacc[c][0]; }
        }
    }
}

}  // namespace cs
