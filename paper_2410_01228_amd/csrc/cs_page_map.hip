// The page table's extra field of the incremental checkpoints (paper Sec. 5): GPU page ->
// host page, host page -> GPU page, and the allocator of host pages in ascending runs.
// Host code only; see include/conserve_kv.h for the contract.
#include "cs_common.h"
#include <new>
#include <vector>

struct cs_page_map {
    std::vector<int32_t> host_of;     // per GPU page: host page, -1 none
    std::vector<int32_t> gpu_of;      // per host page: GPU page, kEvicted, kFree
    std::vector<uint8_t> mark;        // per GPU page: scratch of one checkpoint call
    int32_t free_pages;
    int32_t hint;                     // where the last run ended: next search starts here
};

namespace {

constexpr int32_t kEvicted = -1, kFree = -2;

// first free run of `len` pages at or after `from` (wrapping once); -1 if none
int32_t find_run(const cs_page_map& m, int32_t len, int32_t from) {
    const int32_t H = (int32_t)m.gpu_of.size();
    for (int pass = 0; pass < 2; ++pass) {
        const int32_t lo = pass == 0 ? from : 0, hi = pass == 0 ? H : std::min(H, from + len - 1);
        int32_t run = 0;
        for (int32_t p = lo; p < hi; ++p) {
            run = m.gpu_of[p] == kFree ? run + 1 : 0;
            if (run == len) return p - len + 1;
        }
    }
    return -1;
}

}  // namespace

extern "C" {

cs_page_map* cs_page_map_create(int32_t num_gpu_pages, int32_t num_host_pages) {
    if (num_gpu_pages <= 0 || num_host_pages <= 0) return nullptr;
    cs_page_map* m = new (std::nothrow) cs_page_map;
    if (!m) return nullptr;
    try {
        m->host_of.assign((size_t)num_gpu_pages, -1);
        m->gpu_of.assign((size_t)num_host_pages, kFree);
        m->mark.assign((size_t)num_gpu_pages, 0);
    } catch (const std::bad_alloc&) {
        delete m;
        return nullptr;
    }
    m->free_pages = num_host_pages;
    m->hint = 0;
    return m;
}

void cs_page_map_destroy(cs_page_map* m) { delete m; }

int32_t cs_page_map_host_of(const cs_page_map* m, int32_t gpu_page) {
    if (!m || gpu_page < 0 || gpu_page >= (int32_t)m->host_of.size()) return -1;
    return m->host_of[gpu_page];
}

int32_t cs_page_map_gpu_of(const cs_page_map* m, int32_t host_page) {
    if (!m || host_page < 0 || host_page >= (int32_t)m->gpu_of.size()) return kFree;
    return m->gpu_of[host_page];
}

int32_t cs_page_map_free_host_pages(const cs_page_map* m) { return m ? m->free_pages : 0; }

int32_t cs_page_map_checkpoint(cs_page_map* m, const int32_t* gpu_pages, int32_t n,
                               int32_t* dirty_out, int32_t* first_host) {
    if (!m || n < 0 || (n > 0 && (!gpu_pages || !dirty_out)) || !first_host) return CS_ERR_INVALID_ARG;
    const int32_t G = (int32_t)m->host_of.size();
    for (int32_t i = 0; i < n; ++i)
        if (gpu_pages[i] < 0 || gpu_pages[i] >= G) return CS_ERR_INVALID_ARG;
    int32_t count = 0;
    for (int32_t i = 0; i < n; ++i) {
        const int32_t g = gpu_pages[i];
        if (m->host_of[g] < 0 && !m->mark[g]) { m->mark[g] = 1; dirty_out[count++] = g; }
    }
    for (int32_t i = 0; i < count; ++i) m->mark[dirty_out[i]] = 0;
    *first_host = -1;
    if (count == 0) return 0;
    const int32_t first = count <= m->free_pages ? find_run(*m, count, m->hint) : -1;
    if (first < 0) return CS_ERR_NO_HOST_PAGES;
    for (int32_t i = 0; i < count; ++i) {
        m->host_of[dirty_out[i]] = first + i;
        m->gpu_of[first + i] = dirty_out[i];
    }
    m->free_pages -= count;
    m->hint = first + count < (int32_t)m->gpu_of.size() ? first + count : 0;
    *first_host = first;
    return count;
}

int cs_page_map_evict(cs_page_map* m, const int32_t* gpu_pages, int32_t n, int32_t* host_out) {
    if (!m || n < 0 || (n > 0 && (!gpu_pages || !host_out))) return CS_ERR_INVALID_ARG;
    const int32_t G = (int32_t)m->host_of.size();
    for (int32_t i = 0; i < n; ++i)
        if (gpu_pages[i] < 0 || gpu_pages[i] >= G) return CS_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i) {
        const int32_t g = gpu_pages[i], h = m->host_of[g];
        host_out[i] = h;
        if (h >= 0) { m->gpu_of[h] = kEvicted; m->host_of[g] = -1; }
    }
    return CS_OK;
}

int cs_page_map_bind(cs_page_map* m, const int32_t* host_pages, const int32_t* gpu_pages, int32_t n) {
    if (!m || n < 0 || (n > 0 && (!host_pages || !gpu_pages))) return CS_ERR_INVALID_ARG;
    const int32_t G = (int32_t)m->host_of.size(), H = (int32_t)m->gpu_of.size();
    int32_t i = 0;
    bool ok = true;
    for (; i < n && ok; ++i) {
        const int32_t h = host_pages[i], g = gpu_pages[i];
        ok = h >= 0 && h < H && g >= 0 && g < G && m->gpu_of[h] == kEvicted && m->host_of[g] < 0;
        if (ok) { m->gpu_of[h] = g; m->host_of[g] = h; }     // tentatively: catches repeats within the call
    }
    if (!ok) {
        for (int32_t j = 0; j < i - 1; ++j) { m->gpu_of[host_pages[j]] = kEvicted; m->host_of[gpu_pages[j]] = -1; }
        return CS_ERR_INVALID_ARG;
    }
    return CS_OK;
}

int cs_page_map_drop(cs_page_map* m, const int32_t* host_pages, int32_t n) {
    if (!m || n < 0 || (n > 0 && !host_pages)) return CS_ERR_INVALID_ARG;
    const int32_t H = (int32_t)m->gpu_of.size();
    // all or nothing (a repeat inside the list counts as freeing a free page): free as we go,
    // remembering what each page was tied to, and put everything back on the first bad entry
    std::vector<int32_t> was;
    try { was.reserve((size_t)n); } catch (const std::bad_alloc&) { return CS_ERR_INVALID_ARG; }
    for (int32_t i = 0; i < n; ++i) {
        const int32_t h = host_pages[i];
        if (h < 0 || h >= H || m->gpu_of[h] == kFree) {
            for (int32_t j = 0; j < i; ++j) m->gpu_of[host_pages[j]] = was[(size_t)j];
            return CS_ERR_INVALID_ARG;
        }
        was.push_back(m->gpu_of[h]);
        m->gpu_of[h] = kFree;
    }
    for (int32_t i = 0; i < n; ++i)
        if (was[(size_t)i] >= 0) m->host_of[was[(size_t)i]] = -1;
    m->free_pages += n;
    return CS_OK;
}

}  // extern "C"
