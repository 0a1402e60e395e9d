// Host-side exercise of libconserve_kv under AddressSanitizer / UndefinedBehaviorSanitizer.
// Everything here returns before a kernel launch: the page map, the launch-plan queries and the
// argument checks.  Device pointers are fakes that are never dereferenced on the host.
// Prints "ok <count>" and exits 0; any sanitizer report makes the process exit non-zero.
#include <cstdint>
#include <cstdio>
#include <algorithm>
#include <cstdlib>
#include <random>
#include <vector>
#include "conserve_kv.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed line %d: %s\n", __LINE__, #c); std::exit(3); } } while (0)

static cs_batch make_batch(const std::vector<int32_t>& ctx, const std::vector<int32_t>& cu, int32_t max_blocks) {
    cs_batch b = {};
    b.num_seqs = (int32_t)ctx.size();
    b.num_tokens = cu.back();
    b.block_tables = (const int32_t*)0x20000;      // device pointers: fakes
    b.max_blocks_per_seq = max_blocks;
    b.ctx_lens = (const int32_t*)0x30000;
    b.cu_q_lens = (const int32_t*)0x40000;
    b.h_ctx_lens = ctx.data();
    b.h_cu_q_lens = cu.data();
    return b;
}

int main() {
    std::mt19937 rng(12345);
    long checks = 0;
    // ---- launch plans over random batches, three chip sizes, all shapes ----
    const int shapes[][3] = {{32, 8, 128}, {28, 4, 128}, {64, 8, 128}, {40, 8, 128}, {4, 2, 64}, {16, 1, 64}};
    std::vector<uint32_t> items(1024);
    std::vector<int32_t> order(512);
    for (int round = 0; round < 300; ++round) {
        const int* sh = shapes[rng() % 6];
        const int S = round == 0 ? 65535 : round == 1 ? 881 : round == 2 ? 880 : 1 + (int)(rng() % 300);
        std::vector<int32_t> ctx(S), cu(S + 1, 0);
        int32_t max_need = 1;
        for (int s = 0; s < S; ++s) {
            const int kind = rng() % 10;
            const int32_t q = S > 1000 ? 1 : kind < 6 ? 1 : kind < 7 ? 0 : 2 + (int32_t)(rng() % 3000);
            ctx[s] = S > 1000 ? (int32_t)(rng() % 64) : (int32_t)(rng() % (kind == 9 ? 200000 : 9000));
            cu[s + 1] = cu[s] + q;
            max_need = std::max(max_need, (ctx[s] + q + 7) / 8);
        }
        cs_batch b = make_batch(ctx, cu, max_need);
        cs_debug_set_cu_count(round % 3 == 0 ? 0 : round % 3 == 1 ? 128 : 512);
        // where a mixed batch's decode work runs, and forced cuts of the last tiles, change the plan
        cs_set_mixed_fusion((int32_t)(rng() % 4));
        if (round % 4 == 1) cs_debug_set_tail_cut((int32_t)(rng() % 50), 2 + (int32_t)(rng() % 2));
        else cs_debug_set_tail_cut(-1, 0);
        const size_t need = cs_paged_attention_workspace_bytes(&b, sh[0], sh[1], sh[2]);
        CHECK(cs_paged_attention_workspace_bytes(&b, sh[0], sh[1], sh[2]) == need);      // remembered, same answer
        int32_t split = 0;
        const int32_t n = cs_debug_decode_items(&b, sh[1], sh[2], items.data(), (int32_t)items.size(), &split);
        CHECK(n >= 0 || n <= -1000000);
        CHECK(split >= 256 && split % 16 == 0);
        const int32_t ahead = cs_debug_decode_pages_ahead(&b, sh[1], sh[2]);
        CHECK(ahead == 1 || ahead == 2);
        const int32_t n_ord = cs_debug_prefill_order(&b, sh[0], sh[1], sh[2], order.data(), (int32_t)order.size());
        CHECK(n_ord >= 0 && n_ord <= 512);
        int32_t first_cut = -1, ranges = -1;
        const int32_t n_slots = cs_debug_mixed_tail_cut(&b, sh[0], sh[1], sh[2], &first_cut, &ranges);
        CHECK(n_slots == CS_ERR_INVALID_ARG || (n_slots >= 0 && first_cut >= 0 && first_cut <= n_slots && ranges >= 1));
        if (n_slots > 0 && ranges > 1)
            CHECK(need >= (size_t)(n_slots - first_cut) * sh[1] * ranges * (8 * 16 * (sh[2] + 4) * sizeof(float)));
        const int32_t arrangement = cs_debug_mixed_arrangement(&b, sh[0], sh[1], sh[2]);
        CHECK(arrangement == CS_ERR_INVALID_ARG || (arrangement >= 0 && arrangement <= 2));
        const int32_t n_on = (int32_t)(rng() % (S + 1));
        CHECK(cs_run_layers_workspace_bytes(&b, n_on, sh[0], sh[1], sh[2]) >= need);
        // the attention call itself with a workspace one byte short: refused on the host
        cs_kv_pool pool = {(void*)0x100000, 2, 1 << 22, (int32_t)(rng() % 2 ? 16 : 8), sh[1], sh[2], 0, 0};
        pool.page_stride = 2ll * sh[1] * pool.page_size * sh[2];
        pool.layer_stride = pool.page_stride * pool.num_pages;
        if (need > 0 && b.num_tokens > 0 && (int64_t)max_need * 8 >= 0) {
            const int rc = cs_paged_attention_mixed(&pool, 0, &b, (void*)0x50000, (void*)0x60000, sh[0], 0.1f, (void*)0x70000,
                                                    need - 1, nullptr);
            CHECK(rc == CS_ERR_WORKSPACE_TOO_SMALL || rc == CS_ERR_INVALID_ARG);
        }
        checks += 8;
    }
    cs_debug_set_cu_count(0);
    cs_set_mixed_fusion(1);
    cs_debug_set_tail_cut(-1, 0);
    // ---- the slot model of the fused grid: any work list ends, no earlier than its longest piece alone ----
    for (int round = 0; round < 200; ++round) {
        const int32_t n = 1 + (int32_t)(rng() % 700), cus = 1 + (int32_t)(rng() % 300);
        std::vector<float> work(n);
        float longest = 0.f;
        for (auto& w : work) { w = (float)(rng() % 100000) * 0.01f; longest = std::max(longest, w); }
        const double until = rng() % 2 ? 0.0 : (double)(rng() % 2000);
        const double end = cs_debug_play_tiles(work.data(), n, cus, until);
        CHECK(end >= 0.78 * longest - 1e-3);
        CHECK(cs_debug_play_tiles(work.data(), n, 0, until) == -1.0);
        ++checks;
    }
    // ---- the page map against a plain model ----
    const int32_t G = 500, H = 300;
    cs_page_map* m = cs_page_map_create(G, H);
    CHECK(m != nullptr);
    std::vector<int32_t> host_of(G, -1), gpu_of(H, -2);
    for (int round = 0; round < 4000; ++round) {
        const int op = rng() % 4;
        const int32_t n = 1 + (int32_t)(rng() % 12);
        std::vector<int32_t> a(n), out(n);
        if (op == 0) {                                   // checkpoint
            for (auto& x : a) x = (int32_t)(rng() % G);
            int32_t first = -7;
            const int32_t k = cs_page_map_checkpoint(m, a.data(), n, out.data(), &first);
            if (k > 0) {
                for (int32_t i = 0; i < k; ++i) {
                    CHECK(host_of[out[i]] == -1 && gpu_of[first + i] == -2);
                    host_of[out[i]] = first + i;
                    gpu_of[first + i] = out[i];
                }
            } else {
                CHECK(k == 0 || k == CS_ERR_NO_HOST_PAGES);
            }
        } else if (op == 1) {                            // evict
            for (auto& x : a) x = (int32_t)(rng() % G);
            CHECK(cs_page_map_evict(m, a.data(), n, out.data()) == CS_OK);
            for (int32_t i = 0; i < n; ++i) {
                if (host_of[a[i]] >= 0) { CHECK(out[i] == host_of[a[i]]); gpu_of[host_of[a[i]]] = -1; host_of[a[i]] = -1; }
            }
        } else if (op == 2) {                            // drop whatever is allocated among n random host pages
            std::vector<int32_t> d;
            for (int32_t i = 0; i < n; ++i) { const int32_t h = (int32_t)(rng() % H); bool dup = false; for (int32_t y : d) dup |= y == h; if (gpu_of[h] != -2 && !dup) d.push_back(h); }
            if (!d.empty()) {
                CHECK(cs_page_map_drop(m, d.data(), (int32_t)d.size()) == CS_OK);
                for (int32_t h : d) { if (gpu_of[h] >= 0) host_of[gpu_of[h]] = -1; gpu_of[h] = -2; }
            }
        } else {                                         // bad arguments leave the map alone
            a[0] = G + 5;
            int32_t first = 0;
            CHECK(cs_page_map_checkpoint(m, a.data(), n, out.data(), &first) == CS_ERR_INVALID_ARG);
            CHECK(cs_page_map_host_of(m, -1) == -1 && cs_page_map_gpu_of(m, H) == -2);
        }
        if (round % 97 == 0) {
            int32_t free_model = 0;
            for (int32_t h = 0; h < H; ++h) { CHECK(cs_page_map_gpu_of(m, h) == gpu_of[h]); free_model += gpu_of[h] == -2; }
            for (int32_t g = 0; g < G; ++g) CHECK(cs_page_map_host_of(m, g) == host_of[g]);
            CHECK(cs_page_map_free_host_pages(m) == free_model);
        }
        ++checks;
    }
    cs_page_map_destroy(m);
    cs_page_map_destroy(nullptr);
    std::printf("ok %ld\n", checks);
    return 0;
}
