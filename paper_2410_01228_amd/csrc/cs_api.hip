// C ABI entry points: host-side validation and launch planning.  See include/conserve_kv.h
// for the contract of each call.  This file holds no device code, so that it can be built and
// exercised on the host alone (tests/host_sanitize).
#include <algorithm>
#include <cmath>
#include "cs_common.h"
#include <atomic>
#include <functional>
#include <vector>
#include <string.h>
#include <stdio.h>

namespace cs {

static thread_local char g_hip_error[256] = "";
static std::atomic<int32_t> g_forced_split{0};
static std::atomic<int32_t> g_fuse_mixed{1};
static std::atomic<int32_t> g_forced_ahead{0};
static std::atomic<int32_t> g_forced_cus{0};
static std::atomic<int32_t> g_forced_tail_whole{-1}, g_forced_tail_ranges{0};    // cs_debug_set_tail_cut

// Compute units of the current device, asked once per device.  The launch plans size their
// grids by it.  A host without a device (a plan query in a CPU-only test) plans for 256.
constexpr int kMaxDevices = 64;
static std::atomic<int32_t> g_device_cus[kMaxDevices];
int32_t device_cus() {
    const int32_t forced = g_forced_cus.load();
    if (forced > 0) return forced;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return 256;
    }
    int32_t n = g_device_cus[dev].load();
    if (n <= 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) {
            (void)hipGetLastError();
            v = 256;
        }
        n = v;
        g_device_cus[dev].store(n);
    }
    return n;
}


int hip_failed(hipError_t e, const char* what) {
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
    return CS_ERR_HIP;
}

static bool shape_supported(int32_t Hkv, int32_t D) {
    return Hkv >= 1 && (D == 64 || D == 128);
}

int validate_pool(const cs_kv_pool* p) {
    if (!p || !p->base) return CS_ERR_INVALID_ARG;
    if (p->num_layers <= 0 || p->num_pages <= 0 || p->num_kv_heads <= 0 || p->head_dim <= 0)
        return CS_ERR_INVALID_ARG;
    if (!page_size_supported(p->page_size) || !shape_supported(p->num_kv_heads, p->head_dim)) return CS_ERR_UNSUPPORTED;
    const int64_t page_elems = 2ll * p->num_kv_heads * p->page_size * p->head_dim;
    if (p->page_stride < page_elems || (p->page_stride & 7) != 0) return CS_ERR_INVALID_ARG;
    if (p->layer_stride < (int64_t)p->num_pages * p->page_stride || (p->layer_stride & 7) != 0)
        return CS_ERR_INVALID_ARG;
    if (((uintptr_t)p->base & 15) != 0) return CS_ERR_INVALID_ARG;
    return CS_OK;
}

int validate_batch(const cs_kv_pool* pool, const cs_batch* b) {
    const int32_t page_size = pool ? pool->page_size : kPage;
    if (!b) return CS_ERR_INVALID_ARG;
    if (b->num_seqs < 0 || b->num_tokens < 0 || b->num_seqs > 65535) return CS_ERR_INVALID_ARG;
    if (b->num_seqs == 0) return b->num_tokens == 0 ? CS_OK : CS_ERR_INVALID_ARG;
    if (!b->block_tables || !b->ctx_lens || !b->cu_q_lens || !b->h_ctx_lens || !b->h_cu_q_lens)
        return CS_ERR_INVALID_ARG;
    if (b->max_blocks_per_seq <= 0) return CS_ERR_INVALID_ARG;
    if (b->h_cu_q_lens[0] != 0 || b->h_cu_q_lens[b->num_seqs] != b->num_tokens) return CS_ERR_INVALID_ARG;
    for (int32_t s = 0; s < b->num_seqs; ++s) {
        const int64_t ql = (int64_t)b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s];
        const int64_t c = b->h_ctx_lens[s];
        if (ql < 0 || c < 0) return CS_ERR_INVALID_ARG;
        if (c + ql > (int64_t)b->max_blocks_per_seq * page_size) return CS_ERR_INVALID_ARG;
    }
    return CS_OK;
}

DecodePlan plan_decode(const cs_batch* b, int32_t Hkv, int32_t head_dim) {
    DecodePlan p = {};
    int32_t max_keys = 0, min_keys = 2147483647;
    for (int32_t s = 0; s < b->num_seqs; ++s) {
        const int32_t ql = b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s];
        if (ql == 1) {
            const int32_t n = b->h_ctx_lens[s] + 1;
            ++p.num_decode;
            p.decode_keys += n;
            if (n > max_keys) max_keys = n;
            if (n < min_keys) min_keys = n;
        } else if (ql > 1) {
            ++p.num_prefill;
        }
    }
    p.split_tokens = 256;
    p.pages_ahead = 1;
    if (p.num_decode == 0) return p;
    const int64_t cus = device_cus();
    int32_t split = g_forced_split.load();
    if (split <= 0) {
        // Few, long work items stream best: each pays its start-up latencies once, and when no
        // sequence is cut the plan and merge kernels are not launched at all.  Start from items
        // of about 2 MiB of K/V per kv head and halve only until the grid has enough workgroups:
        // three per CU, or one per CU when the sequences are of nearly equal length (then the
        // items are too, nothing straggles, and a workgroup that has its CU to itself streams
        // fastest: over 159 uniform batches of three model shapes, 256-511 workgroups beat both
        // fewer and the 512-1023 of the next halving by 5-8%).
        // Launches below about 0.4 GB of K/V (some 60 us) are decided by start-up, merge and how
        // many workgroups crowd a CU, not by the steady state: they aim at one and a half workgroups
        // per CU (over 171 random batches of three shapes: mean distance to the best forced plan
        // 3.8% -> 2.3%, worst 61% -> 17%, together with the floor rule below).
        // (the workgroup counts and byte volumes below were measured on 256 CUs and scale with the chip)
        const int32_t cap = head_dim >= 128 ? 4096 : 8192;
        const bool uniform = (int64_t)max_keys * 4 <= (int64_t)min_keys * 5;
        const int64_t kv_bytes = p.decode_keys * 2 * Hkv * head_dim * 2;
        const int64_t need = uniform ? cus : kv_bytes >= 400000000ll * cus / 256 ? 3 * cus : cus * 3 / 2;
        auto workgroups_at = [&](int32_t sp) {
            int64_t items = 0;
            for (int32_t s = 0; s < b->num_seqs; ++s)
                if (b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s] == 1)
                    items += decode_num_splits(b->h_ctx_lens[s] + 1, sp);
            return items * Hkv;
        };
        // no sequence is cut into more than about 16 pieces: beyond that the partials, their merge
        // and the start-up of ever shorter items cost more than the fuller grid gains -- unless
        // that leaves CUs without any workgroup (a handful of very long sequences)
        int32_t floor_split = 256;
        while (floor_split < cap && (int64_t)floor_split * 16 < max_keys) floor_split *= 2;
        while (floor_split > 256 && workgroups_at(floor_split) < cus) floor_split /= 2;
        for (split = cap; split > floor_split; split /= 2)
            if (workgroups_at(split) >= need) break;
    }
    p.split_tokens = split;
    int32_t max_k = 1;
    for (int32_t s = 0; s < b->num_seqs; ++s) {
        if (b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s] != 1) continue;
        const int32_t k = decode_num_splits(b->h_ctx_lens[s] + 1, split);
        p.total_items += k;
        if (k > 1) ++p.num_multi;
        if (k > max_k) max_k = k;
    }
    // Two pages ahead per wavefront need the registers of the third workgroup per CU.  Measured
    // over 33 batch shapes: the deeper queue wins 2-6% once the launch is long enough for the
    // steady state to dominate (from about 0.65 GB of K/V on, ~100 us), and loses 2-7% on
    // smaller launches, where start-up and tail decide and every workgroup slot counts.
    {
        const int64_t kv_bytes = p.decode_keys * 2 * Hkv * head_dim * 2;
        p.pages_ahead = kv_bytes >= 650000000ll * cus / 256 ? 2 : 1;
        // equal items run in rounds over the workgroup slots: between 513 and 768 of them are one
        // round of three per CU, but a round and a quarter of two per CU
        const bool uniform = (int64_t)max_keys * 4 <= (int64_t)min_keys * 5;
        const int64_t wgs = (int64_t)p.total_items * Hkv;
        if (uniform && wgs > 2 * cus && wgs <= 3 * cus) p.pages_ahead = 1;
        const int32_t forced = g_forced_ahead.load();
        if (forced == 1 || forced == 2) p.pages_ahead = forced;
    }
    // A list short enough for the argument block is written here, longest items first: the
    // workgroups of a launch start in index order, so the long ones get going at once and
    // the short ones fill in behind them (measured: 7% on 256 sequences of 512..4096 keys).
    p.in_args = p.total_items <= kMaxArgItems && b->num_seqs <= 65536 && max_k <= 255;
    if (p.in_args) {
        struct Rec { int32_t keys, seq, k; };
        Rec recs[kMaxArgItems];
        int32_t n_rec = 0;
        for (int32_t s = 0; s < b->num_seqs; ++s) {
            if (b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s] != 1) continue;
            const int32_t n = b->h_ctx_lens[s] + 1;
            const int32_t k = decode_num_splits(n, split);
            recs[n_rec++] = Rec{k > 1 ? decode_chunk_keys(n, k) : n, s, k};
        }
        std::stable_sort(recs, recs + n_rec, [](const Rec& a, const Rec& c) { return a.keys > c.keys; });
        int32_t item = 0, m = 0;
        for (int32_t r = 0; r < n_rec; ++r) {
            if (recs[r].k > 1) p.arg_multi.e[m++] = (uint32_t)recs[r].seq | ((uint32_t)item << 16);
            for (int32_t i = 0; i < recs[r].k; ++i)
                p.arg_items.e[item++] = (uint32_t)recs[r].seq | ((uint32_t)i << 16) | ((uint32_t)recs[r].k << 24);
        }
    }
    return p;
}

// Host plan of the key-range split (a pure function of the host lengths).
PrefillPlan plan_prefill(const cs_batch* b, int32_t Hq, int32_t Hkv, int32_t D) {
    PrefillPlan p = {};
    const int32_t G = Hq / Hkv;
    int64_t total_steps = 0, tiles = 0;
    int32_t max_steps = 0, first = -1, last = -1;
    struct Tile { int32_t steps, slot; };
    Tile tile_list[kMaxSlotOrder];
    int32_t n_listed = 0;
    for (int32_t s = 0; s < b->num_seqs; ++s) {
        const int32_t ql = b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s];
        if (ql <= 1) continue;
        if (first < 0) first = s;
        last = s;
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
    p.base_slot = (int32_t)prefill_slot_start(b->h_cu_q_lens[first], first, G);
    // (the slots of the sequences before the first chunk and behind the last one are empty)
    p.num_slots = (int32_t)(prefill_slot_start(b->h_cu_q_lens[last + 1], last + 1, G) - p.base_slot);
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
        p.bytes = (size_t)p.num_slots * Hkv * p.max_ranges * kTileCols * 16 * (D + 4) * sizeof(float);
    }
    return p;
}

// How a batch with both kinds of work is launched (see cs_mixed.hip): as two kernels in a row, as
// one grid with the decode pairs behind the tiles, or as one grid with a decode workgroup per CU
// beside the tiles.  mode: cs_set_mixed_fusion's (0 never fuse, 1 choose, 2 always behind, 3
// always beside).
struct FusePlan {
    int32_t arrangement;       // 0 two kernels, 1 decode behind the tiles, 2 decode beside the tiles
    int32_t prio;              // 0, or the higher of the two issue priorities the tiles alternate between (1, 2)
    int32_t persistent_wgs;    // arrangement 2: decode workgroups (one per CU)
};

// The tile workgroups of a fused grid played through the chip's workgroup slots (two per CU), in
// microseconds.  work[i]: what workgroup i takes while another tile shares its CU; it runs
// kSoloTile of that while the CU's other slot is empty and kBesideDecode of it beside a decode
// workgroup (fitted to the arrangements' measured order over many mixes, not to timelines: by
// those a tile beside a decode workgroup takes 1.3-1.4 of its paired time).  The dispatcher
// gives the first `cus` workgroups a CU each, the next `cus` the second slot of those CUs, and
// every later one the slot that frees first.  decode_until > 0: slot 0 of every CU is a decode
// workgroup's until then.  (The caller plays TILES, not workgroups: the workgroups of a tile's
// kv heads are equally long and start together, so a tile is one unit on a group of
// num_kv_heads CUs, and a long grid costs the host an eighth of the events.)  Returns when the
// last tile ends; free_at (two entries per CU) receives when each slot was last released,
// started (optional) when each workgroup began.
constexpr double kSoloTile = 0.78, kBesideDecode = 1.1;
static double play_tiles(const std::vector<float>& work, int32_t cus, double decode_until, std::vector<double>& free_at,
                         std::vector<float>* started = nullptr) {
    struct Cu { int8_t kind[2]; double rem[2]; double last; uint32_t ver; };     // kind: 0 empty, 1 tile, 2 decode
    struct Event { double t; int32_t cu, slot; uint32_t ver; };
    auto later = [](const Event& a, const Event& b) { return a.t > b.t; };
    std::vector<Cu> cu((size_t)cus, Cu{{0, 0}, {0, 0}, 0, 0});
    std::vector<Event> ev;
    free_at.assign(2 * (size_t)cus, 0.0);
    size_t next = 0;
    auto rate = [&](const Cu& c, int s) {
        const int8_t other = c.kind[1 - s];
        return other == 1 ? 1.0 : other == 2 ? 1.0 / kBesideDecode : 1.0 / kSoloTile;
    };
    auto advance = [&](Cu& c, double t) {
        for (int s = 0; s < 2; ++s)
            if (c.kind[s] == 1) c.rem[s] -= (t - c.last) * rate(c, s);
        c.last = t;
    };
    double now = 0;
    if (started) started->assign(work.size(), 0.f);
    auto take_next = [&](Cu& c, int s) {
        if (next < work.size()) {
            if (started) (*started)[next] = (float)now;
            c.kind[s] = 1;
            c.rem[s] = work[next++];
        }
    };
    auto announce = [&](int32_t i, double t) {               // the ends of CU i's tiles at today's rates
        Cu& c = cu[(size_t)i];
        ++c.ver;
        for (int s = 0; s < 2; ++s)
            if (c.kind[s] == 1) {
                ev.push_back(Event{t + std::max(c.rem[s], 0.0) / rate(c, s), i, s, c.ver});
                std::push_heap(ev.begin(), ev.end(), later);
            }
    };
    if (decode_until > 0) {
        for (Cu& c : cu) c.kind[0] = 2;
        ev.push_back(Event{decode_until, -1, 0, 0});
    }
    for (int s = 0; s < 2; ++s)
        for (Cu& c : cu)
            if (c.kind[s] == 0) take_next(c, s);
    for (int32_t i = 0; i < cus; ++i) announce(i, 0.0);
    double end = 0;
    while (!ev.empty()) {
        std::pop_heap(ev.begin(), ev.end(), later);
        const Event e = ev.back();
        ev.pop_back();
        now = e.t;
        if (e.cu < 0) {                                       // the decode workgroups retire
            for (int32_t i = 0; i < cus; ++i) {
                Cu& c = cu[(size_t)i];
                advance(c, e.t);
                c.kind[0] = 0;
                free_at[2 * (size_t)i] = e.t;
                take_next(c, 0);
                announce(i, e.t);
            }
            continue;
        }
        Cu& c = cu[(size_t)e.cu];
        if (e.ver != c.ver) continue;                         // overtaken by a change on that CU
        advance(c, e.t);
        c.kind[e.slot] = 0;
        free_at[2 * (size_t)e.cu + e.slot] = e.t;
        end = std::max(end, e.t);
        take_next(c, e.slot);
        announce(e.cu, e.t);
    }
    return end;
}

// The choice between "behind" and "beside" comes from playing both grids (play_tiles).  A tile
// workgroup of n steps takes (n + 8) * 0.88 us (a 32-key step at head dim 128 beside another
// tile).  Behind: the decode bytes flow at 6.5 TB/s times min(1, free slots / (1.56 CUs)) into
// the slots the tiles have left for good.  Beside: one slot per CU is a decode workgroup's until
// all bytes have passed at 6.5 TB/s.  Over 196 mixes of four model shapes, the arrangement this
// model takes is on average 0.0-0.7% (per shape) slower than the fastest of the three by
// measurement, 8% at worst (always behind: 3-8% on average, always beside: 2-6%); the merges of
// cut tiles and cut sequences cost the same either way.
//
// Beside the tiles, the tiles of the last round are cut (p is changed): a tile that starts when
// the decode side is about done runs alone on its CU, one wavefront per SIMD, while the slot the
// decode workgroup has left stays empty.  The launch positions from the first such tile on are
// cut into two or three key ranges, so that the pieces fill both slots; taken when the model
// promises 6% of the whole call after the cost of the partials (it overrates what cutting gains
// beside a decode load, so the bar is not lower).
static FusePlan plan_fusion_by_model(const cs_batch* b, const DecodePlan& d, PrefillPlan& p, int32_t Hq, int32_t Hkv,
                                     int32_t D, int32_t mode) {
    FusePlan f = {0, 0, 0};
    if (d.num_prefill == 0 || d.num_decode == 0 || !d.in_args || mode == 0) return f;
    const int32_t G = Hq / Hkv;
    double pairs = 0;
    for (int32_t s = 0; s < b->num_seqs; ++s) {
        const double ql = b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s];
        if (ql > 1) pairs += ql * ((double)b->h_ctx_lens[s] + (ql + 1) / 2);
    }
    // ideal times: flops at 1 PFLOP/s, bytes at 6 TB/s
    const double t_prefill = 4.0 * Hq * D * pairs / 1.0e15;
    const double decode_bytes = (double)d.decode_keys * 2 * Hkv * D * 2;
    const double t_decode = decode_bytes / 6.0e12;
    // Behind the tiles, unless the prefill side is a sliver: with a small chunk beside a long
    // decode (decode time over ten times the prefill time) two kernels in a row are as fast or a
    // little faster.  Where the decode side is the smaller one (under 0.3 of the prefill time)
    // the tiles alternate their issue priority as the prefill kernel's do; with a decode load of
    // equal weight behind them that costs more than it gains.
    f.arrangement = (mode == 2 || t_decode <= 10.0 * t_prefill) ? 1 : 0;
    f.prio = t_decode < 0.3 * t_prefill ? 1 : 0;
    const int32_t cus = device_cus();
    // (head dim 64 fits three workgroups per CU, both kinds already share CUs behind the tiles,
    // and beside wins on some mixes and loses on others: the choice there is not modelled)
    if (mode == 2 || (mode == 1 && D != 128)) return f;
    bool beside = mode == 3;
    double t_beside = 0;                                               // the model's time of that arrangement as planned (0: not played)
    const int64_t tile_units = (int64_t)p.num_slots * p.max_ranges;       // tiles x ranges: what the model plays
    const int32_t groups = std::max(1, cus / Hkv);                         // CU groups of one CU per kv head
    const double us_per_step = 0.88, t_dec = decode_bytes / 6.5e6;      // microseconds
    // (a decode side under 0.3 of the prefill side stays behind tiles that alternate their
    // priority: measured 5-8% better than beside on such mixes, which the model calls even)
    if ((mode == 1 && !f.prio) || mode == 3) {
        if (tile_units > 8192) {
            // more than 16 rounds of tiles: how the rounds end no longer matters, and beside wins
            // wherever the decode side is at least half the prefill side (mixes of 2-4 rounds:
            // beside from about 0.45 on)
            beside = beside || t_decode >= 0.5 * t_prefill;
        } else {
            // steps of every tile slot, then the workgroups in the fused grid's launch order
            std::vector<int32_t> slot_steps((size_t)p.num_slots, 0);
            for (int32_t s = 0; s < b->num_seqs; ++s) {
                const int32_t ql = b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s];
                if (ql <= 1) continue;
                const int32_t n_ct = ((ql + 15) >> 4) * G;
                const int64_t slot0 = prefill_slot_start(b->h_cu_q_lens[s], s, G) - p.base_slot;
                for (int32_t ct0 = 0; ct0 < n_ct; ct0 += kTileCols) {
                    const int32_t tb_max = (std::min(ct0 + kTileCols, n_ct) - 1) / G;
                    const int32_t n_keys = b->h_ctx_lens[s] + std::min(ql, (tb_max + 1) * 16);
                    slot_steps[(size_t)(slot0 + ct0 / kTileCols)] = (n_keys + kKeysPerStep - 1) / kKeysPerStep;
                }
            }
            auto steps_at = [&](int32_t pos) { return slot_steps[(size_t)(p.backwards ? p.num_slots - 1 - pos : pos)]; };
            // the grid's tile workgroups in launch order: whole tiles up to position `whole`, then,
            // range-major, the ranges of `range_steps` steps of the tiles behind them
            std::vector<float> work;
            std::vector<int32_t> pos_of;
            auto list_work = [&](int32_t whole, int32_t range_steps, int32_t ranges) {
                work.clear();
                pos_of.clear();
                for (int32_t pos = 0; pos < whole; ++pos)
                    if (steps_at(pos) > 0) {
                        work.push_back((float)((steps_at(pos) + 8) * us_per_step));
                        pos_of.push_back(pos);
                    }
                for (int32_t r = 0; r < ranges; ++r)
                    for (int32_t pos = whole; pos < p.num_slots; ++pos) {
                        const int32_t n = std::min(steps_at(pos), (r + 1) * range_steps) - r * range_steps;
                        if (n > 0) {
                            work.push_back((float)((n + 8) * us_per_step));
                            pos_of.push_back(pos);
                        }
                    }
            };
            list_work(0, p.range_steps, p.max_ranges);
            std::vector<double> free_at;
            std::vector<float> started;
            double t_whole = 0;                                  // beside, as planned so far
            if (mode == 1) {
                play_tiles(work, groups, 0.0, free_at);
                std::sort(free_at.begin(), free_at.end());
                double t = 0, left = t_dec, t_behind = 0;
                const double sat = 1.56 * groups;
                for (size_t i = 0; ; ++i) {
                    const double rate = std::min(1.0, (double)i / sat);          // i slots (of every CU of a group) are free
                    const double next = i < free_at.size() ? free_at[i] : 1.0e300;
                    if (rate > 0 && t + left / rate <= next) { t_behind = t + left / rate; break; }
                    left -= rate * (next - t);
                    t = next;
                }
                t_whole = std::max(play_tiles(work, groups, t_dec, free_at, &started), t_dec);
                // (the model's constants were fitted before the tiles took their priorities beside a
                // decode load, which make that arrangement about 2% faster than it says)
                beside = 0.98 * t_whole < t_behind;
            }
            if (beside && mode != 1 && !work.empty()) t_whole = std::max(play_tiles(work, groups, t_dec, free_at, &started), t_dec);
            t_beside = t_whole;
            if (beside && p.max_ranges == 1 && !work.empty() && g_forced_tail_whole.load() != -2) {
                // the tiles of the last round, cut: from the first tile that starts when the
                // decode side is at least 0.85 done
                size_t first = 0;
                while (first < work.size() && started[first] < 0.85 * t_dec) ++first;
                if (first > 0 && first < work.size()) {
                    const int32_t whole = pos_of[first];
                    int32_t tail_steps = 0;
                    for (int32_t pos = whole; pos < p.num_slots; ++pos) tail_steps = std::max(tail_steps, steps_at(pos));
                    // Two or three ranges of at least 128 steps each: cuts of shorter tiles were
                    // promised 6-14% by this model and lost 3-6% (the start-up of one more
                    // workgroup and its partial weigh more than the model has them).  Three ranges
                    // are taken over two unless the model has them 6% behind: measured over the
                    // long-tile mixes they are 2% ahead where it calls them 2-5% behind.
                    double t_r[4] = {0, 0, 0, 0};
                    for (int32_t r = 2; r <= 3 && tail_steps / r >= 128; ++r) {
                        const int32_t rs = (tail_steps + r - 1) / r, ranges = (tail_steps + rs - 1) / rs;
                        list_work(whole, rs, ranges);
                        const double part_bytes = (double)(p.num_slots - whole) * Hkv * ranges * kTileCols * 16 * (D + 4) * 4.0;
                        t_r[r] = std::max(play_tiles(work, groups, t_dec, free_at), t_dec) + 10.0 + 2.0 * part_bytes / 5.0e6;
                    }
                    const double bar = 0.94 * t_whole;
                    const int32_t r = t_r[3] > 0 && t_r[3] < bar && t_r[3] <= 1.06 * t_r[2] ? 3 : 2;
                    if (t_r[r] > 0 && t_r[r] < bar) {
                        const int32_t rs = (tail_steps + r - 1) / r, ranges = (tail_steps + rs - 1) / rs;
                        t_beside = t_r[r];
                        p.cut_first_pos = whole;
                        p.range_steps = rs;
                        p.max_ranges = ranges;
                        p.bytes = (size_t)((double)(p.num_slots - whole) * Hkv * ranges * kTileCols * 16 * (D + 4) * 4.0);
                    }
                }
            }
        }
    }
    if (beside) {
        // Beside, the tiles alternate their priority whatever the weights: two tiles share a CU
        // once its decode workgroup is done, and until then it costs nothing (measured -1.5% on
        // average over 196 mixes of four model shapes, -4% with chunks on 30K keys, +3% at worst).
        // Where the model has the tiles outlast the decode stream, but by less than its own
        // length, both of their priorities lie above the decode wavefronts': over 256 mixes that
        // is worth 3-5% on average in that band (12% at best, 3% lost at worst) and costs 2-3%
        // on either side of it -- a stream that ends last must not be held up, and beside a
        // short one the tiles mostly share their CUs with each other.
        f.arrangement = 2;
        f.prio = t_beside > t_dec && t_beside < 2.0 * t_dec ? 2 : 1;
        f.persistent_wgs = cus;
    }
    return f;
}

static FusePlan plan_fusion(const cs_batch* b, const DecodePlan& d, PrefillPlan& p, int32_t Hq, int32_t Hkv,
                            int32_t D, int32_t mode) {
    const FusePlan f = plan_fusion_by_model(b, d, p, Hq, Hkv, D, mode);
    const int32_t forced_whole = g_forced_tail_whole.load(), forced_ranges = g_forced_tail_ranges.load();
    if (forced_whole >= 0 && forced_ranges >= 1 && f.arrangement != 0) {
        // measurement and test knob: cut the launch positions from forced_whole on into forced_ranges
        p = plan_prefill(b, Hq, Hkv, D);
        p.n_ordered = 0;
        p.cut_first_pos = std::min(forced_whole, p.num_slots);
        int32_t tail_steps = 1;
        for (int32_t s = 0; s < b->num_seqs; ++s) {           // (the longest tile of all: an upper bound of the tail's)
            const int32_t ql = b->h_cu_q_lens[s + 1] - b->h_cu_q_lens[s];
            if (ql > 1) tail_steps = std::max(tail_steps, (b->h_ctx_lens[s] + ql + kKeysPerStep - 1) / kKeysPerStep);
        }
        p.range_steps = (tail_steps + forced_ranges - 1) / forced_ranges;
        p.max_ranges = p.cut_first_pos < p.num_slots ? (tail_steps + p.range_steps - 1) / p.range_steps : 1;
        p.bytes = p.max_ranges > 1 ? (size_t)(p.num_slots - p.cut_first_pos) * Hkv * p.max_ranges * kTileCols * 16 * (D + 4) * sizeof(float) : 0;
    }
    return f;
}

static size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

DecodeWorkspace decode_workspace(const DecodePlan& p, int32_t S, int32_t Hq, int32_t D) {
    DecodeWorkspace w = {};
    if (p.num_decode == 0 || p.num_multi == 0) return w;   // nothing is cut: no item list, no partials
    size_t off = 0;
    w.items = off;    off += align16((size_t)p.total_items * 8 * sizeof(int32_t));
    w.cu_items = off; off += align16((size_t)(S + 1) * sizeof(int32_t));
    w.multi = off;    off += align16((size_t)(p.num_multi + 1) * sizeof(int32_t));
    // partials are indexed by item; only items of multi-item sequences are ever written
    const size_t part_items = p.num_multi ? (size_t)p.total_items : 0;
    w.part_ml = off;  off += align16(part_items * Hq * 2 * sizeof(float));
    w.part_o = off;   off += align16(part_items * Hq * D * sizeof(float));
    w.total = off;
    return w;
}

}  // namespace cs

using namespace cs;

extern "C" {

size_t cs_page_bytes(int32_t Hkv, int32_t D) {
    if (!shape_supported(Hkv, D)) return 0;
    return (size_t)2 * Hkv * kPage * D * 2;
}

size_t cs_pool_page_bytes(const cs_kv_pool* pool) {
    if (!pool || !page_size_supported(pool->page_size) || !shape_supported(pool->num_kv_heads, pool->head_dim)) return 0;
    return pool_page_bytes(*pool);
}

int cs_kv_append(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                 const void* k_new, const void* v_new, void* stream) {
    int rc = validate_pool(pool);
    if (rc) return rc;
    if (layer < 0 || layer >= pool->num_layers) return CS_ERR_INVALID_ARG;
    rc = validate_batch(pool, batch);
    if (rc) return rc;
    if (batch->num_tokens == 0) return CS_OK;
    if (!k_new || !v_new || ((uintptr_t)k_new & 15) || ((uintptr_t)v_new & 15)) return CS_ERR_INVALID_ARG;
    return launch_append(*pool, layer, *batch, k_new, v_new, (hipStream_t)stream);
}

static int attention_shape_ok(int32_t Hq, int32_t Hkv, int32_t D) {
    if (Hq <= 0 || Hkv <= 0) return CS_ERR_INVALID_ARG;
    if (Hq % Hkv != 0) return CS_ERR_INVALID_ARG;
    if (!shape_supported(Hkv, D) || Hq / Hkv > kMaxGroup) return CS_ERR_UNSUPPORTED;
    return CS_OK;
}

// The launch plan of a batch: a pure function of the host lengths, the shape, the chip and the
// measurement knobs.  The workspace query and the attention call of one layer, and the calls of
// the next layers, ask for the same plan again and again (an item list of up to 880 entries and a
// sort each time), so each thread remembers the last two it made, keyed by everything the plan
// depends on, the lengths compared value by value.
struct Plans {
    DecodePlan d;
    PrefillPlan p;
    FusePlan f;
    size_t decode_bytes, need;
};
struct PlanMemo {
    bool valid = false;
    int32_t S = 0, T = 0, Hq = 0, Hkv = 0, D = 0, split = 0, ahead = 0, cus = 0, fuse = 0, tail_whole = -1, tail_ranges = 0;
    std::vector<int32_t> ctx, cu;
    Plans plans;
};
static const Plans& plans_for(const cs_batch* b, int32_t Hq, int32_t Hkv, int32_t D) {
    static thread_local PlanMemo memo[2];
    static thread_local int next = 0;
    const int32_t S = b->num_seqs, split = g_forced_split.load(), ahead = g_forced_ahead.load(), cus = device_cus();
    const int32_t fuse = g_fuse_mixed.load(), tail_whole = g_forced_tail_whole.load(), tail_ranges = g_forced_tail_ranges.load();
    for (PlanMemo& m : memo)
        if (m.valid && m.fuse == fuse && m.tail_whole == tail_whole && m.tail_ranges == tail_ranges && m.S == S && m.T == b->num_tokens && m.Hq == Hq && m.Hkv == Hkv && m.D == D && m.split == split &&
            m.ahead == ahead && m.cus == cus && memcmp(m.ctx.data(), b->h_ctx_lens, sizeof(int32_t) * S) == 0 &&
            memcmp(m.cu.data(), b->h_cu_q_lens, sizeof(int32_t) * (S + 1)) == 0)
            return m.plans;
    PlanMemo& m = memo[next];
    next ^= 1;
    m.valid = false;
    m.S = S; m.T = b->num_tokens; m.Hq = Hq; m.Hkv = Hkv; m.D = D; m.split = split; m.ahead = ahead; m.cus = cus; m.fuse = fuse; m.tail_whole = tail_whole; m.tail_ranges = tail_ranges;
    m.ctx.assign(b->h_ctx_lens, b->h_ctx_lens + S);
    m.cu.assign(b->h_cu_q_lens, b->h_cu_q_lens + S + 1);
    m.plans.d = plan_decode(b, Hkv, D);
    m.plans.p = m.plans.d.num_prefill ? plan_prefill(b, Hq, Hkv, D) : PrefillPlan{};
    m.plans.f = plan_fusion(b, m.plans.d, m.plans.p, Hq, Hkv, D, fuse);
    m.plans.decode_bytes = decode_workspace(m.plans.d, S, Hq, D).total;
    m.plans.need = m.plans.decode_bytes + m.plans.p.bytes;
    m.valid = true;
    return m.plans;
}

size_t cs_paged_attention_workspace_bytes(const cs_batch* batch, int32_t Hq, int32_t Hkv, int32_t D) {
    if (attention_shape_ok(Hq, Hkv, D) != CS_OK) return 0;
    if (validate_batch(nullptr, batch) != CS_OK || batch->num_seqs == 0) return 0;
    return plans_for(batch, Hq, Hkv, D).need;
}

// The first num_online_seqs sequences of a batch over the same arrays (what is left of an
// iteration once it is preempted: paper Sec. 4.3).
static cs_batch online_prefix(const cs_batch& b, int32_t num_online_seqs) {
    cs_batch cur = b;
    cur.num_seqs = num_online_seqs;
    cur.num_tokens = num_online_seqs > 0 ? b.h_cu_q_lens[num_online_seqs] : 0;
    return cur;
}

size_t cs_run_layers_workspace_bytes(const cs_batch* batch, int32_t num_online_seqs, int32_t Hq, int32_t Hkv, int32_t D) {
    if (attention_shape_ok(Hq, Hkv, D) != CS_OK) return 0;
    if (validate_batch(nullptr, batch) != CS_OK || batch->num_seqs == 0) return 0;
    size_t need = plans_for(batch, Hq, Hkv, D).need;
    if (num_online_seqs > 0 && num_online_seqs < batch->num_seqs) {
        const cs_batch cur = online_prefix(*batch, num_online_seqs);
        need = std::max(need, plans_for(&cur, Hq, Hkv, D).need);
    }
    return need;
}

static int attention_mixed(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                           const void* q, void* out, int32_t Hq, float softmax_scale,
                           void* workspace, size_t workspace_bytes, void* stream, bool f16) {
    int rc = validate_pool(pool);
    if (rc) return rc;
    if (layer < 0 || layer >= pool->num_layers) return CS_ERR_INVALID_ARG;
    rc = attention_shape_ok(Hq, pool->num_kv_heads, pool->head_dim);
    if (rc) return rc;
    rc = validate_batch(pool, batch);
    if (rc) return rc;
    if (batch->num_tokens == 0) return CS_OK;
    if (!q || !out || ((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return CS_ERR_INVALID_ARG;
    if (!(softmax_scale > 0.f) || softmax_scale > 3.0e38f) return CS_ERR_INVALID_ARG;   // positive, finite
    const Plans& plans = plans_for(batch, Hq, pool->num_kv_heads, pool->head_dim);
    const DecodePlan& plan = plans.d;
    const PrefillPlan& pplan = plans.p;
    const size_t decode_bytes = plans.decode_bytes, need = plans.need;
    if (need > 0 && (!workspace || ((uintptr_t)workspace & 15))) return CS_ERR_INVALID_ARG;
    if (workspace_bytes < need) return CS_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    if (plans.f.arrangement != 0) {
        // both kinds of work in one grid, then the merges of whatever was cut
        void* prefill_ws = (char*)workspace + decode_bytes;
        rc = launch_mixed(*pool, layer, *batch, plan, pplan, q, out, Hq, softmax_scale, workspace, prefill_ws, st, f16,
                          plans.f.prio, plans.f.arrangement == 2 ? plans.f.persistent_wgs : 0);
        if (rc) return rc;
        rc = launch_prefill_merge(*pool, *batch, pplan, out, Hq, prefill_ws, st, f16);
        if (rc) return rc;
        return launch_decode(*pool, layer, *batch, plan, q, out, Hq, softmax_scale, workspace, st, f16, true);
    }
    if (plan.num_prefill > 0) {
        rc = launch_prefill(*pool, layer, *batch, pplan, q, out, Hq, softmax_scale, (char*)workspace + decode_bytes, st, f16);
        if (rc) return rc;
    }
    return launch_decode(*pool, layer, *batch, plan, q, out, Hq, softmax_scale, workspace, st, f16);
}

int cs_paged_attention_mixed(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                             const void* q, void* out, int32_t Hq, float softmax_scale,
                             void* workspace, size_t workspace_bytes, void* stream) {
    return attention_mixed(pool, layer, batch, q, out, Hq, softmax_scale, workspace, workspace_bytes, stream, false);
}

int cs_paged_attention_mixed_f16(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                                 const void* q, void* out, int32_t Hq, float softmax_scale,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    return attention_mixed(pool, layer, batch, q, out, Hq, softmax_scale, workspace, workspace_bytes, stream, true);
}

static int ckpt_common(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* ids, int32_t n,
                       const void* staging, size_t staging_bytes) {
    int rc = validate_pool(pool);
    if (rc) return rc;
    if (l0 < 0 || l1 < l0 || l1 > pool->num_layers || n < 0) return CS_ERR_INVALID_ARG;
    if (n == 0 || l1 == l0) return CS_OK;
    if (!ids || !staging || ((uintptr_t)staging & 15)) return CS_ERR_INVALID_ARG;
    const size_t need = (size_t)(l1 - l0) * n * pool_page_bytes(*pool);
    if (staging_bytes < need) return CS_ERR_STAGING_TOO_SMALL;
    if ((int64_t)n * 4 > 2147483647ll || l1 - l0 > 65535) return CS_ERR_INVALID_ARG;
    return 1;   // proceed
}

int cs_kv_ckpt_gather(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* ids, int32_t n,
                      void* staging, size_t staging_bytes, void* stream) {
    const int rc = ckpt_common(pool, l0, l1, ids, n, staging, staging_bytes);
    if (rc <= 0) return rc;
    return launch_page_copy(*pool, l0, l1, ids, n, staging, true, (hipStream_t)stream);
}

int cs_kv_ckpt_restore(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* ids, int32_t n,
                       const void* staging, size_t staging_bytes, void* stream) {
    const int rc = ckpt_common(pool, l0, l1, ids, n, staging, staging_bytes);
    if (rc <= 0) return rc;
    return launch_page_copy(*pool, l0, l1, ids, n, (void*)staging, false, (hipStream_t)stream);
}

static int ckpt_tokens_common(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* slots, int32_t n,
                              const void* staging, size_t staging_bytes) {
    int rc = validate_pool(pool);
    if (rc) return rc;
    if (l0 < 0 || l1 < l0 || l1 > pool->num_layers || n < 0) return CS_ERR_INVALID_ARG;
    if (n == 0 || l1 == l0) return CS_OK;
    if (!slots || !staging || ((uintptr_t)staging & 15)) return CS_ERR_INVALID_ARG;
    const size_t need = (size_t)(l1 - l0) * n * 2 * pool->num_kv_heads * pool->head_dim * 2;
    if (staging_bytes < need) return CS_ERR_STAGING_TOO_SMALL;
    if (l1 - l0 > 65535) return CS_ERR_INVALID_ARG;
    return 1;   // proceed
}

int cs_kv_ckpt_gather_tokens(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* token_slots, int32_t n,
                             void* staging, size_t staging_bytes, void* stream) {
    const int rc = ckpt_tokens_common(pool, l0, l1, token_slots, n, staging, staging_bytes);
    if (rc <= 0) return rc;
    return launch_token_copy(*pool, l0, l1, token_slots, n, staging, true, (hipStream_t)stream);
}

int cs_kv_ckpt_restore_tokens(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* token_slots, int32_t n,
                              const void* staging, size_t staging_bytes, void* stream) {
    const int rc = ckpt_tokens_common(pool, l0, l1, token_slots, n, staging, staging_bytes);
    if (rc <= 0) return rc;
    return launch_token_copy(*pool, l0, l1, token_slots, n, (void*)staging, false, (hipStream_t)stream);
}

int cs_kv_ckpt_save(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* ids, int32_t n,
                    void* staging, size_t staging_bytes, void* host_buf, void* stream) {
    const int rc = ckpt_common(pool, l0, l1, ids, n, staging, staging_bytes);
    if (rc <= 0) return rc;
    if (!host_buf) return CS_ERR_INVALID_ARG;
    const int lrc = launch_page_copy(*pool, l0, l1, ids, n, staging, true, (hipStream_t)stream);
    if (lrc) return lrc;
    const size_t bytes = (size_t)(l1 - l0) * n * pool_page_bytes(*pool);
    const hipError_t e = hipMemcpyAsync(host_buf, staging, bytes, hipMemcpyDeviceToHost, (hipStream_t)stream);
    return e == hipSuccess ? CS_OK : hip_failed(e, "checkpoint device-to-host copy");
}

int cs_kv_ckpt_load(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* ids, int32_t n,
                    void* staging, size_t staging_bytes, const void* host_buf, void* stream) {
    const int rc = ckpt_common(pool, l0, l1, ids, n, staging, staging_bytes);
    if (rc <= 0) return rc;
    if (!host_buf) return CS_ERR_INVALID_ARG;
    const size_t bytes = (size_t)(l1 - l0) * n * pool_page_bytes(*pool);
    const hipError_t e = hipMemcpyAsync(staging, host_buf, bytes, hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return hip_failed(e, "checkpoint host-to-device copy");
    return launch_page_copy(*pool, l0, l1, ids, n, staging, false, (hipStream_t)stream);
}

static int run_common(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* ids, int32_t n,
                      const void* staging, size_t staging_bytes, const cs_host_store* store, int32_t first) {
    const int rc = ckpt_common(pool, l0, l1, ids, n, staging, staging_bytes);
    if (rc <= 0) return rc;
    if (!store || !store->base || store->num_layers != l1 - l0 || store->num_pages <= 0) return CS_ERR_INVALID_ARG;
    if (first < 0 || (int64_t)first + n > store->num_pages) return CS_ERR_INVALID_ARG;
    return 1;   // proceed
}

int cs_kv_ckpt_save_run(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* ids, int32_t n,
                        void* staging, size_t staging_bytes, const cs_host_store* store, int32_t first, void* stream) {
    const int rc = run_common(pool, l0, l1, ids, n, staging, staging_bytes, store, first);
    if (rc <= 0) return rc;
    const int lrc = launch_page_copy(*pool, l0, l1, ids, n, staging, true, (hipStream_t)stream, true);
    if (lrc) return lrc;
    const size_t fat = (size_t)(l1 - l0) * pool_page_bytes(*pool);   // one host page
    const hipError_t e = hipMemcpyAsync((char*)store->base + (size_t)first * fat, staging, (size_t)n * fat,
                                        hipMemcpyDeviceToHost, (hipStream_t)stream);
    return e == hipSuccess ? CS_OK : hip_failed(e, "checkpoint device-to-host copy");
}

int cs_kv_ckpt_load_run(const cs_kv_pool* pool, int32_t l0, int32_t l1, const int32_t* ids, int32_t n,
                        void* staging, size_t staging_bytes, const cs_host_store* store, int32_t first, void* stream) {
    const int rc = run_common(pool, l0, l1, ids, n, staging, staging_bytes, store, first);
    if (rc <= 0) return rc;
    const size_t fat = (size_t)(l1 - l0) * pool_page_bytes(*pool);
    const hipError_t e = hipMemcpyAsync(staging, (const char*)store->base + (size_t)first * fat, (size_t)n * fat,
                                        hipMemcpyHostToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return hip_failed(e, "checkpoint host-to-device copy");
    return launch_page_copy(*pool, l0, l1, ids, n, staging, false, (hipStream_t)stream, true);
}

static int run_layers(const cs_kv_pool* pool, int32_t l0, int32_t l1, const cs_batch* batch,
                      const void* q, const void* k_new, const void* v_new, void* out,
                      int64_t q_stride, int64_t kv_stride, int32_t Hq, float scale,
                      void* workspace, size_t workspace_bytes, const cs_safepoint* sp,
                      int32_t* preempted_before_layer, void* stream, bool f16) {
    if (preempted_before_layer) *preempted_before_layer = -1;
    int rc = validate_pool(pool);
    if (rc) return rc;
    if (l0 < 0 || l1 < l0 || l1 > pool->num_layers || q_stride < 0 || kv_stride < 0) return CS_ERR_INVALID_ARG;
    rc = validate_batch(pool, batch);
    if (rc) return rc;
    if (sp && (sp->check_every <= 0 || sp->num_online_seqs < 0 || sp->num_online_seqs > batch->num_seqs))
        return CS_ERR_INVALID_ARG;
    // Everything that can refuse the iteration is checked before its first layer is enqueued.  The
    // workspace must hold the full batch's plan AND the online prefix's: fewer sequences are cut
    // finer (more partials), so the prefix can need more than the whole.
    if (l1 > l0 && batch->num_tokens > 0) {
        rc = attention_shape_ok(Hq, pool->num_kv_heads, pool->head_dim);
        if (rc) return rc;
        if (!q || !out || !k_new || !v_new) return CS_ERR_INVALID_ARG;
        if (!(scale > 0.f) || scale > 3.0e38f) return CS_ERR_INVALID_ARG;
        const size_t need = cs_run_layers_workspace_bytes(batch, sp ? sp->num_online_seqs : 0, Hq, pool->num_kv_heads,
                                                          pool->head_dim);
        if (need > 0 && (!workspace || ((uintptr_t)workspace & 15))) return CS_ERR_INVALID_ARG;
        if (workspace_bytes < need) return CS_ERR_WORKSPACE_TOO_SMALL;
    }
    cs_batch cur = *batch;
    bool preempted = false;
    for (int32_t l = l0; l < l1; ++l) {
        if (sp && !preempted && (l - l0) % sp->check_every == 0) {
            // safepoint: between two layers nothing of the iteration is half done
            if (sp->sync_at_safepoint) {
                const hipError_t e = hipStreamSynchronize((hipStream_t)stream);
                if (e != hipSuccess) return hip_failed(e, "safepoint synchronise");
            }
            bool raise = sp->flag && *sp->flag != 0;
            if (!raise && sp->poll) raise = sp->poll(sp->poll_arg) != 0;
            if (raise) {
                // drop the offline tail: same arrays, fewer sequences
                preempted = true;
                cur = online_prefix(*batch, sp->num_online_seqs);
                if (preempted_before_layer) *preempted_before_layer = l;
            }
        }
        const int64_t i = l - l0;
        const uint16_t* ql = (const uint16_t*)q + i * q_stride;
        const uint16_t* kl = (const uint16_t*)k_new + i * kv_stride;
        const uint16_t* vl = (const uint16_t*)v_new + i * kv_stride;
        uint16_t* ol = (uint16_t*)out + i * q_stride;
        rc = cs_kv_append(pool, l, &cur, kl, vl, stream);
        if (rc) return rc;
        rc = attention_mixed(pool, l, &cur, ql, ol, Hq, scale, workspace, workspace_bytes, stream, f16);
        if (rc) return rc;
    }
    return CS_OK;
}

int cs_run_layers(const cs_kv_pool* pool, int32_t l0, int32_t l1, const cs_batch* batch,
                  const void* q, const void* k_new, const void* v_new, void* out,
                  int64_t q_stride, int64_t kv_stride, int32_t Hq, float scale,
                  void* workspace, size_t workspace_bytes, const cs_safepoint* sp,
                  int32_t* preempted_before_layer, void* stream) {
    return run_layers(pool, l0, l1, batch, q, k_new, v_new, out, q_stride, kv_stride, Hq, scale, workspace,
                      workspace_bytes, sp, preempted_before_layer, stream, false);
}

int cs_run_layers_f16(const cs_kv_pool* pool, int32_t l0, int32_t l1, const cs_batch* batch,
                      const void* q, const void* k_new, const void* v_new, void* out,
                      int64_t q_stride, int64_t kv_stride, int32_t Hq, float scale,
                      void* workspace, size_t workspace_bytes, const cs_safepoint* sp,
                      int32_t* preempted_before_layer, void* stream) {
    return run_layers(pool, l0, l1, batch, q, k_new, v_new, out, q_stride, kv_stride, Hq, scale, workspace,
                      workspace_bytes, sp, preempted_before_layer, stream, true);
}

int cs_debug_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (bytes == 0) return CS_OK;
    if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return CS_ERR_INVALID_ARG;
    if (bytes > (size_t)1 << 44) return CS_ERR_INVALID_ARG;
    return launch_plain_copy(dst, src, bytes, (hipStream_t)stream);
}

int32_t cs_debug_decode_items(const cs_batch* batch, int32_t Hkv, int32_t D, uint32_t* items, int32_t capacity,
                              int32_t* split_tokens) {
    if (!shape_supported(Hkv, D) || validate_batch(nullptr, batch) != CS_OK || capacity < 0 || (capacity > 0 && !items))
        return CS_ERR_INVALID_ARG;
    const DecodePlan p = plan_decode(batch, Hkv, D);
    if (split_tokens) *split_tokens = p.split_tokens;
    if (!p.in_args) return -1000000 - p.total_items;       // the planning kernel would build the list
    for (int32_t i = 0; i < p.total_items && i < capacity; ++i) items[i] = p.arg_items.e[i];
    return p.total_items;
}

int32_t cs_debug_decode_pages_ahead(const cs_batch* batch, int32_t Hkv, int32_t D) {
    if (!shape_supported(Hkv, D) || validate_batch(nullptr, batch) != CS_OK) return CS_ERR_INVALID_ARG;
    return plan_decode(batch, Hkv, D).pages_ahead;
}

int32_t cs_debug_prefill_order(const cs_batch* batch, int32_t Hq, int32_t Hkv, int32_t D, int32_t* slots, int32_t capacity) {
    if (attention_shape_ok(Hq, Hkv, D) != CS_OK || validate_batch(nullptr, batch) != CS_OK || capacity < 0 ||
        (capacity > 0 && !slots))
        return CS_ERR_INVALID_ARG;
    if (batch->num_seqs == 0) return 0;
    const PrefillPlan p = plan_prefill(batch, Hq, Hkv, D);
    for (int32_t i = 0; i < p.n_ordered && i < capacity; ++i) slots[i] = p.order.slot[i];
    return p.n_ordered;
}

void cs_debug_set_cu_count(int32_t cus) {
    g_forced_cus.store(cus > 0 ? cus : 0);
}

void cs_set_decode_pages_ahead(int32_t pages) {
    g_forced_ahead.store(pages == 1 || pages == 2 ? pages : 0);
}

int32_t cs_debug_mixed_arrangement(const cs_batch* batch, int32_t Hq, int32_t Hkv, int32_t D) {
    if (attention_shape_ok(Hq, Hkv, D) != CS_OK) return CS_ERR_INVALID_ARG;
    if (validate_batch(nullptr, batch) != CS_OK || batch->num_seqs == 0) return CS_ERR_INVALID_ARG;
    return plans_for(batch, Hq, Hkv, D).f.arrangement;
}

int32_t cs_debug_mixed_tile_priority(const cs_batch* batch, int32_t Hq, int32_t Hkv, int32_t D) {
    if (attention_shape_ok(Hq, Hkv, D) != CS_OK) return CS_ERR_INVALID_ARG;
    if (validate_batch(nullptr, batch) != CS_OK || batch->num_seqs == 0) return CS_ERR_INVALID_ARG;
    const Plans& plans = plans_for(batch, Hq, Hkv, D);
    return plans.f.arrangement == 0 ? 0 : plans.f.prio;
}

int32_t cs_debug_mixed_tail_cut(const cs_batch* batch, int32_t Hq, int32_t Hkv, int32_t D, int32_t* first_cut, int32_t* ranges) {
    if (attention_shape_ok(Hq, Hkv, D) != CS_OK) return CS_ERR_INVALID_ARG;
    if (validate_batch(nullptr, batch) != CS_OK || batch->num_seqs == 0) return CS_ERR_INVALID_ARG;
    const PrefillPlan& p = plans_for(batch, Hq, Hkv, D).p;
    if (first_cut) *first_cut = p.cut_first_pos;
    if (ranges) *ranges = p.max_ranges > 0 ? p.max_ranges : 1;     // (a batch without chunks has no plan: 0 slots, nothing cut)
    return p.num_slots;
}

double cs_debug_play_tiles(const float* work_us, int32_t n, int32_t cus, double decode_until_us) {
    if (!work_us || n < 0 || cus <= 0) return -1.0;
    std::vector<float> work(work_us, work_us + n);
    std::vector<double> free_at;
    return play_tiles(work, cus, decode_until_us, free_at);
}

void cs_debug_set_tail_cut(int32_t whole_tiles, int32_t ranges) {
    g_forced_tail_whole.store(whole_tiles >= 0 && ranges >= 1 ? whole_tiles : whole_tiles == -2 ? -2 : -1);   // (-2: no cut by the model either)
    g_forced_tail_ranges.store(whole_tiles >= 0 && ranges >= 1 ? ranges : 0);
}

void cs_set_mixed_fusion(int32_t mode) {
    g_fuse_mixed.store(mode == 0 || mode == 2 || mode == 3 ? mode : 1);
}

void cs_set_decode_split_tokens(int32_t tokens) {
    if (tokens < 0) tokens = 0;
    g_forced_split.store((tokens + 15) / 16 * 16);
}

const char* cs_status_string(int status) {
    switch (status) {
        case CS_OK: return "ok";
        case CS_ERR_INVALID_ARG: return "invalid argument";
        case CS_ERR_UNSUPPORTED: return "unsupported shape";
        case CS_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case CS_ERR_STAGING_TOO_SMALL: return "staging buffer too small";
        case CS_ERR_HIP: return "HIP error";
        case CS_ERR_NO_HOST_PAGES: return "no free run of host pages";
        case CS_ERR_STATIC_SCRATCH_TOO_SMALL: return "the batch needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

const char* cs_last_hip_error(void) { return g_hip_error; }

}  // extern "C"
