/*
 * conserve_kv.h -- C ABI of the MI355X (gfx950) kernels for the per-layer GPU hot path of
 * online/offline LLM co-serving: KV append, paged attention over a mixed batch of decode
 * and chunked-prefill tokens, and the gather / restore copies of incremental KV
 * checkpointing (paper Sec. 4.2, 4.3, 4.4, 5).
 *
 * Conventions for every call
 *   - returns a cs_status (0 = CS_OK, negative = error); all checks that need only host
 *     data are made before anything is enqueued, and a failed call enqueues nothing;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream);
 *     calls never synchronise and never allocate or free device memory.  State kept between
 *     calls: the host-side cs_page_map object at the end of this file; the measurement knobs
 *     cs_set_decode_split_tokens / cs_set_decode_pages_ahead / cs_set_mixed_fusion /
 *     cs_debug_set_cu_count / cs_debug_set_tail_cut, which are process-wide, change launch plans and workspace sizes,
 *     and are meant for benchmarks and tests only (a serving process leaves them alone); and,
 *     invisible to the caller, each thread's memo of the last launch plans it made and each
 *     device's compute-unit count, asked once;
 *   - every pointer is owned by the caller and must stay valid until the enqueued work has
 *     run.  "device" pointers are HIP device memory of the current device, "host" pointers
 *     are ordinary host memory read during the call only;
 *   - 16-bit data (bf16; fp16 through cs_paged_attention_mixed_f16), 16 tokens per page (the
 *     paper's page granularity, Sec. 5) or 8 (cs_kv_pool.page_size), head_dim 64 or 128,
 *     num_q_heads / num_kv_heads <= 16;
 *   - each call works on ONE decoder layer (attention, append) or a layer range (gather,
 *     restore), so that a scheduler can stop between layers (layer-wise preemption,
 *     Sec. 4.3): sequences are expected online-first, and passing a smaller num_seqs /
 *     num_tokens with the same arrays drops the offline tail without rebuilding metadata;
 *   - device index arrays (block tables, page id lists) are not validated on the host (that
 *     would need a synchronisation).  A page id outside [0, num_pages) is never dereferenced:
 *     the copies (append, gather, restore) skip it.  The attention output of a sequence whose
 *     block table holds such an id within its length is unspecified (the decode path leaves
 *     the page's keys out and writes zeros if no key is left; the chunk path reads page 0 of
 *     the pool in its place); every other sequence of the batch is unaffected;
 *   - the explicit K/V, head and token strides a generic paged pool would carry are absent on
 *     purpose: inside a (layer, page) the format below is fixed, because it is what lets the
 *     kernels load matrix operands without shuffles; only the layer and page strides vary.
 *
 * KV pool format (this library's own; the paper fixes only the 16-token page and the
 * per-request page table).  In bf16 elements:
 *
 *     pool[layer][page][kv: 0 = K, 1 = V][kv_head][16 * head_dim]
 *
 * with layer_stride and page_stride given explicitly, so one (layer, page) is a contiguous
 * blob of 2 * num_kv_heads * 16 * head_dim elements ("page_elems").  Inside a block
 * (token t = 0..15 of the page, feature d):
 *     K:  ((d / 8) * 16 + t) * 8 + d % 8                 [D/8][16 tokens][8 features]
 *     V:  (((d / 16) * 2 + t / 8) * 16 + d % 16) * 8 + t % 8
 *                                                        [D/16][2 token halves][16][8 tokens]
 * A 16-byte unit of K is 8 features of one token, a 16-byte unit of V is one feature of 8
 * tokens: these are the operand registers the gfx950 matrix instructions take for Q.K^T and
 * P.V, so wavefronts read blocks with fully coalesced loads and no shuffles.
 *
 * Pages of 8 tokens (page_size 8; a finer unit for the per-token management of Sec. 4.4)
 * use the same format with 8 in place of 16 tokens and one token group in place of two:
 *     pool[layer][page][kv][kv_head][8 * head_dim],  t = 0..7
 *     K:  ((d / 8) * 8 + t) * 8 + d % 8                  [D/8][8 tokens][8 features]
 *     V:  ((d / 16) * 16 + d % 16) * 8 + t               [D/16][16][8 tokens]
 * Wherever a comment below says 16 tokens or "/16", read page_size.  The attention kernels
 * then take two (decode) or four (prefill) pages per step instead of one or two.
 */
#ifndef CONSERVE_KV_H
#define CONSERVE_KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CS_OK = 0,
    CS_ERR_INVALID_ARG = -1,        /* null pointer, negative count, inconsistent lengths */
    CS_ERR_UNSUPPORTED = -2,        /* page size, head_dim or head ratio not supported   */
    CS_ERR_WORKSPACE_TOO_SMALL = -3,
    CS_ERR_STAGING_TOO_SMALL = -4,
    CS_ERR_HIP = -5,                /* a launch failed; see cs_last_hip_error()          */
    CS_ERR_NO_HOST_PAGES = -6,      /* the host page store has no free run long enough   */
    CS_ERR_STATIC_SCRATCH_TOO_SMALL = -7   /* the batch's plan needs more than CS_STATIC_SCRATCH_BYTES */
} cs_status;

#define CS_PAGE_SIZE 16

/* The caller's KV pool.  Strides are in bf16 ELEMENTS. */
typedef struct {
    void*   base;                   /* device                                            */
    int32_t num_layers;
    int32_t num_pages;
    int32_t page_size;              /* 16 or 8                                           */
    int32_t num_kv_heads;
    int32_t head_dim;               /* 64 or 128                                         */
    int64_t layer_stride;           /* >= num_pages * page_stride                        */
    int64_t page_stride;            /* >= page_elems, multiple of 8                      */
} cs_kv_pool;

/* One step's batch: S sequences, sequence s has ctx_lens[s] tokens already in the cache
 * (the paper's C) and q_s = cu_q_lens[s+1] - cu_q_lens[s] new tokens this step (the paper's
 * P; 1 for a decode token, >1 for a prefill chunk, 0 for an idle sequence).  New token i of
 * sequence s has absolute position ctx_lens[s] + i. */
typedef struct {
    int32_t        num_seqs;            /* S, at most 65535 */
    int32_t        num_tokens;          /* T = cu_q_lens[S] */
    const int32_t* block_tables;        /* device [S][max_blocks_per_seq] page ids; entries
                                           past ceil((ctx+q)/16) are never read          */
    int32_t        max_blocks_per_seq;
    const int32_t* ctx_lens;            /* device [S]                                    */
    const int32_t* cu_q_lens;           /* device [S+1]                                  */
    const int32_t* h_ctx_lens;          /* host copy of ctx_lens, for launch planning    */
    const int32_t* h_cu_q_lens;         /* host copy of cu_q_lens                        */
} cs_batch;

/* Bytes of one (layer, page) of 16 tokens: K and V of every kv head.  0 if the shape is
 * unsupported.  cs_pool_page_bytes: the same for the page size of `pool`. */
size_t cs_page_bytes(int32_t num_kv_heads, int32_t head_dim);
size_t cs_pool_page_bytes(const cs_kv_pool* pool);

/* KV append (the cache is append-only, Sec. 1 and 4.4; pages of 16 tokens, Sec. 5).
 * For every new token t = cu_q_lens[s] + i: copy k_new[t][h][:] and v_new[t][h][:] into
 * page block_tables[s][(ctx_lens[s]+i)/16], slot (ctx_lens[s]+i)%16 of layer `layer`, in
 * the pool format above.  No other slot is written.  k_new, v_new: device [T][Hkv][D] bf16.
 * T == 0 is a no-op. */
int cs_kv_append(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                 const void* k_new, const void* v_new, void* stream);

/* Workspace the attention call needs for this batch: the fp32 partial results of decode
 * sequences cut into work items and of prefill tiles cut into key ranges (the launch plan is
 * made here from the host arrays of `batch` and the shape, and again, identically, in the
 * attention call, which finds it remembered).  Zero for many batches; a few MB to a few hundred
 * MB when chunks of up to a few thousand tokens are cut to fill the chip.  Returns 0 on bad
 * arguments. */
size_t cs_paged_attention_workspace_bytes(const cs_batch* batch, int32_t num_q_heads,
                                          int32_t num_kv_heads, int32_t head_dim);

/* Paged attention of one layer over a mixed batch (Sec. 4.2: a batch holds online and
 * offline tokens together; the attention term P(P+C); chunked prefill).  For new token t of
 * sequence s at position p and query head h (kv head h / (Hq/Hkv)):
 *     out[t][h][:] = sum_{j<=p} softmax_j(scale * <q[t][h], K_s[j]>) * V_s[j]
 * where K_s, V_s are read from the pool through block_tables[s].  The step's own new K/V
 * must already be in the pool (call cs_kv_append first on the same stream).  Sequences with
 * one new token take the split-KV decode path, longer chunks the MFMA tile path.
 * softmax_scale must be positive and finite.
 * q, out: device [T][Hq][D] bf16.  workspace: device, at least
 * cs_paged_attention_workspace_bytes(); contents are scratch. */
int cs_paged_attention_mixed(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                             const void* q, void* out, int32_t num_q_heads,
                             float softmax_scale, void* workspace, size_t workspace_bytes,
                             void* stream);

/* The same call for IEEE half data (the precision the paper's system served in, Sec. 6.1):
 * the pool, q and out hold fp16 instead of bf16; scores, softmax and accumulation stay in
 * fp32.  The pool format and every other call (append, gather, restore) only move 16-bit
 * words and serve both element types unchanged. */
int cs_paged_attention_mixed_f16(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                                 const void* q, void* out, int32_t num_q_heads,
                                 float softmax_scale, void* workspace, size_t workspace_bytes,
                                 void* stream);

/* For callers that cannot allocate device memory or bring a workspace -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: cs_paged_attention_mixed (bf16)
 * with its workspace taken from a buffer of CS_STATIC_SCRATCH_BYTES that lives in the library's
 * code object (one copy per device the library runs on, held until the process ends).  The call
 * allocates and frees nothing, on the device or through any library.  Inputs and outputs are the
 * caller's as before; results are bit-identical to cs_paged_attention_mixed on the same batch.
 *   - a batch whose launch plan needs more than the buffer holds is refused with
 *     CS_ERR_STATIC_SCRATCH_TOO_SMALL and nothing is enqueued (ask
 *     cs_paged_attention_workspace_bytes() beforehand; most batches need nothing at all);
 *   - all calls on one device share that device's buffer, which keeps the last call's contents:
 *     nothing in it needs clearing, but two calls that overlap in time on one device (two
 *     streams, two threads) race on it.  Calls on one stream, or otherwise ordered, are safe;
 *   - the buffer's device address is looked up on the first call on each device
 *     (hipGetSymbolAddress); make that first call outside a stream capture. */
#define CS_STATIC_SCRATCH_BYTES (64u << 20)
size_t cs_static_scratch_bytes(void);
int cs_paged_attention_mixed_static(const cs_kv_pool* pool, int32_t layer, const cs_batch* batch,
                                    const void* q, void* out, int32_t num_q_heads,
                                    float softmax_scale, void* stream);

/* Checkpoint gather (Sec. 5: the KV of scattered pages is gathered into one contiguous
 * buffer and transferred once; Sec. 4.4: only newly filled pages are checkpointed).
 *     staging[l - layer_begin][i][0 .. page_elems) = pool[l][page_ids[i]][...]
 * for layer_begin <= l < layer_end, 0 <= i < n.  page_ids: device [n]; duplicates allowed.
 * staging: device, (layer_end-layer_begin) * n * cs_pool_page_bytes() bytes, 16-byte aligned.
 * n == 0 is a no-op. */
int cs_kv_ckpt_gather(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end,
                      const int32_t* page_ids, int32_t n,
                      void* staging, size_t staging_bytes, void* stream);

/* Restore (Sec. 4.4: evicted KV is brought back in the background on resume): the inverse
 * copy, pool[l][page_ids[i]] = staging[l - layer_begin][i].  Ids must be distinct. */
int cs_kv_ckpt_restore(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end,
                       const int32_t* page_ids, int32_t n,
                       const void* staging, size_t staging_bytes, void* stream);

/* Token-granular checkpoint (Sec. 4.4: the KV state is managed per token, and after each
 * generation step only the newly generated tokens are checkpointed).  token_slots[i] =
 * page * page_size + slot names one cached token;
 *     staging[l - layer_begin][i][0][h][:] = its K row of kv head h,  [...][1][h][:] = its V row
 * (plain rows of head_dim bf16, the layout of k_new / v_new; nothing of the page format is
 * left in the buffer).  token_slots: device [n]; a slot outside the pool is skipped.
 * staging: device, (layer_end-layer_begin) * n * 2 * num_kv_heads * head_dim * 2 bytes,
 * 16-byte aligned.  n == 0 is a no-op.  Whole pages are cheaper through cs_kv_ckpt_gather. */
int cs_kv_ckpt_gather_tokens(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end,
                             const int32_t* token_slots, int32_t n,
                             void* staging, size_t staging_bytes, void* stream);

/* The inverse copy: the rows of staging[l][i] go to token slot token_slots[i] of every layer
 * in range; nothing else in the pool is written.  Slots must be distinct. */
int cs_kv_ckpt_restore_tokens(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end,
                              const int32_t* token_slots, int32_t n,
                              const void* staging, size_t staging_bytes, void* stream);

/* Incremental checkpoint to host memory and back (Sec. 4.4: checkpoint the newly filled
 * pages after each step, prefetch them back on resume; Sec. 5: gather into one contiguous
 * buffer, transfer it once, on a stream of its own so the copy overlaps the model's work --
 * full pages are immutable, so no synchronisation with the compute stream is needed).
 *   save: cs_kv_ckpt_gather into `staging`, then ONE device-to-host copy of the gathered
 *         bytes to `host_buf`, both enqueued on `stream`;
 *   load: ONE host-to-device copy from `host_buf` into `staging`, then cs_kv_ckpt_restore.
 * host_buf: PINNED host memory (hipHostMalloc) of at least the gathered size, laid out like
 * staging ([layers][n][page bytes]); it must stay valid until the stream has run.  Pageable
 * memory would make the copy synchronous and is the caller's mistake to avoid.  Errors as
 * for gather / restore. */
int cs_kv_ckpt_save(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end,
                    const int32_t* page_ids, int32_t n, void* staging, size_t staging_bytes,
                    void* host_buf, void* stream);
int cs_kv_ckpt_load(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end,
                    const int32_t* page_ids, int32_t n, void* staging, size_t staging_bytes,
                    const void* host_buf, void* stream);

/* Layer-wise preemption (Sec. 4.3, Alg. 1): the layers of one iteration are enqueued one
 * call at a time, and every `check_every` layers (a safepoint; the paper uses 4) the driver
 * looks at a preemption signal that a scheduler thread raises when an online request
 * arrives.  Once it is raised, the remaining layers run with only the first
 * `num_online_seqs` sequences (the batch is ordered online-first, so this is a smaller
 * num_seqs / num_tokens over the same arrays -- nothing is rebuilt).
 *   flag: host memory shared with the scheduler (pinned or ordinary), nonzero = preempt;
 *   poll: optional callback asked at each safepoint instead of / in addition to the flag;
 *   sync_at_safepoint: nonzero = wait for the stream before looking (preemption takes effect
 *   within check_every layers of GPU work, at the price of draining the launch queue);
 *   zero = look without waiting (no bubble; takes effect for layers not yet enqueued). */
typedef struct {
    const volatile int32_t* flag;
    int32_t (*poll)(void* arg);
    void*   poll_arg;
    int32_t check_every;
    int32_t num_online_seqs;
    int32_t sync_at_safepoint;
} cs_safepoint;

/* Runs cs_kv_append + cs_paged_attention_mixed for layers [layer_begin, layer_end) with the
 * safepoints above (safepoint == NULL: none).  Per-layer tensors: layer l uses
 * q + (l - layer_begin) * q_layer_stride elements, likewise k_new / v_new (kv_layer_stride)
 * and out (q_layer_stride); strides in bf16 elements.  *preempted_before_layer (host,
 * nullable) receives the first layer that ran online-only, or -1.  workspace: at least
 * cs_run_layers_workspace_bytes() -- the larger of what the full batch and what its online
 * prefix need (fewer sequences are cut finer, so the prefix can need more than the whole).
 * Everything that can refuse the iteration (shapes, pointers, workspace size for both plans)
 * is checked before the first layer is enqueued.  Errors as for the two calls. */
int cs_run_layers(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end, const cs_batch* batch,
                  const void* q, const void* k_new, const void* v_new, void* out,
                  int64_t q_layer_stride, int64_t kv_layer_stride,
                  int32_t num_q_heads, float softmax_scale, void* workspace, size_t workspace_bytes,
                  const cs_safepoint* safepoint, int32_t* preempted_before_layer, void* stream);

/* Workspace of cs_run_layers for this batch when a safepoint may cut it down to its first
 * num_online_seqs sequences (0 or num_seqs: no cut).  Host only.  Returns 0 on bad arguments. */
size_t cs_run_layers_workspace_bytes(const cs_batch* batch, int32_t num_online_seqs, int32_t num_q_heads,
                                     int32_t num_kv_heads, int32_t head_dim);

/* The same loop for fp16 data (see cs_paged_attention_mixed_f16). */
int cs_run_layers_f16(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end, const cs_batch* batch,
                      const void* q, const void* k_new, const void* v_new, void* out,
                      int64_t q_layer_stride, int64_t kv_layer_stride,
                      int32_t num_q_heads, float softmax_scale, void* workspace, size_t workspace_bytes,
                      const cs_safepoint* safepoint, int32_t* preempted_before_layer, void* stream);

/* ---- The page table's extra field (Sec. 5): which host page holds the checkpoint of a GPU
 * page.  Host-side bookkeeping only; it is the one object of this library that keeps state
 * (create allocates it with malloc, destroy frees it), and it is not thread-safe: one
 * scheduler thread owns it.
 *
 * The host page store it indexes is caller-owned PINNED memory laid out
 *     store[host page][layer][page bytes]
 * so one host page is the contiguous checkpoint of one GPU page in all layers of the store,
 * and a checkpoint round, which takes its host pages as ONE ascending run, is one contiguous
 * device-to-host copy (Sec. 5: gather into a contiguous buffer, transfer once).
 *
 * Life of a page: cs_page_map_checkpoint gives every listed GPU page that has no host copy
 * yet the next page of a fresh run (those pages are what cs_kv_ckpt_save_run then copies);
 * cs_page_map_evict (preemption) forgets the GPU side and reports the host pages, which stay
 * allocated; cs_page_map_bind (resume) ties them to the fresh GPU pages they were loaded
 * into by cs_kv_ckpt_load_run; cs_page_map_drop frees host pages (request finished). ---- */
typedef struct cs_page_map cs_page_map;

typedef struct cs_host_store {
    void*   base;            /* PINNED host memory: num_pages * num_layers * page bytes   */
    int32_t num_layers;      /* layers a host page holds                                 */
    int32_t num_pages;       /* host pages                                               */
} cs_host_store;

/* NULL if a count is not positive or memory is short. */
cs_page_map* cs_page_map_create(int32_t num_gpu_pages, int32_t num_host_pages);
void cs_page_map_destroy(cs_page_map* map);

/* Host page of a GPU page, -1 if it has none (or the id is out of range). */
int32_t cs_page_map_host_of(const cs_page_map* map, int32_t gpu_page);
/* GPU page a host page is tied to; -1: allocated but evicted; -2: free or out of range. */
int32_t cs_page_map_gpu_of(const cs_page_map* map, int32_t host_page);
int32_t cs_page_map_free_host_pages(const cs_page_map* map);

/* One checkpoint round over gpu_pages[0..n): the pages without a host copy (each once, in
 * the order given) are written to dirty_out (room for n) and get the host pages
 * *first_host, *first_host + 1, ...  Returns how many (0: everything was saved already),
 * CS_ERR_NO_HOST_PAGES if no free run of that length exists, CS_ERR_INVALID_ARG for a page
 * id out of range or a null pointer; on error the map is unchanged. */
int32_t cs_page_map_checkpoint(cs_page_map* map, const int32_t* gpu_pages, int32_t n,
                               int32_t* dirty_out, int32_t* first_host);

/* Preemption: the GPU pages go back to the allocator.  host_out[i] (room for n) = the host
 * page of gpu_pages[i], -1 if it never was checkpointed (its tokens must be recomputed). */
int cs_page_map_evict(cs_page_map* map, const int32_t* gpu_pages, int32_t n, int32_t* host_out);

/* Resume: host_pages[i] (allocated, evicted) now backs gpu_pages[i] (no host copy).  All or
 * nothing: CS_ERR_INVALID_ARG leaves the map unchanged. */
int cs_page_map_bind(cs_page_map* map, const int32_t* host_pages, const int32_t* gpu_pages, int32_t n);

/* Free host pages, tied to a GPU page or not.  Freeing a free page is an error (all or
 * nothing). */
int cs_page_map_drop(cs_page_map* map, const int32_t* host_pages, int32_t n);

/* cs_kv_ckpt_save / cs_kv_ckpt_load into and out of the host page store: the n pages go to /
 * come from the host pages first_host_page .. + n.  The staging buffer is used page-major
 * ([n][layers][page bytes]) so that the host side is one contiguous copy.
 * layer_end - layer_begin must equal store->num_layers. */
int cs_kv_ckpt_save_run(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end,
                        const int32_t* page_ids, int32_t n, void* staging, size_t staging_bytes,
                        const cs_host_store* store, int32_t first_host_page, void* stream);
int cs_kv_ckpt_load_run(const cs_kv_pool* pool, int32_t layer_begin, int32_t layer_end,
                        const int32_t* page_ids, int32_t n, void* staging, size_t staging_bytes,
                        const cs_host_store* store, int32_t first_host_page, void* stream);

/* Plain device-to-device copy kernel of `bytes` (multiple of 16, both pointers 16-byte
 * aligned): the measured copy ceiling of the device and the calibration point for hardware
 * byte counters. */
int cs_debug_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Host-only view of the decode path's launch plan, for tests: the work items of `batch` in
 * launch order, one word each -- sequence (bits 0-15), piece (16-23), pieces of that sequence
 * (24-31) -- as they would travel in the kernel arguments; sequence s with n keys in k pieces
 * has pieces of ceil(n/k) keys rounded up to a page.  Writes min(items, capacity) words and
 * returns the number of items; returns -1000000 - items when the list is too long for the
 * kernel arguments (then a planning kernel builds it on the device, in sequence order).
 * *split_tokens (optional) receives the target keys per item.  No device work. */
int32_t cs_debug_decode_items(const cs_batch* batch, int32_t num_kv_heads, int32_t head_dim,
                              uint32_t* items, int32_t capacity, int32_t* split_tokens);

/* The launch plans size their grids by the compute-unit count of the current device
 * (hipDeviceAttributeMultiprocessorCount, asked once per device; 256 where no device answers).
 * For host tests: plan as if the device had `cus` compute units; 0 = ask the device again.
 * Process-wide; changes launch plans and workspace sizes. */
void cs_debug_set_cu_count(int32_t cus);

/* Tuning knob for measurements: force the decode path's tokens per split (multiple of 16,
 * 0 = automatic).  Process-wide; affects cs_paged_attention_workspace_bytes() as well. */
void cs_set_decode_split_tokens(int32_t tokens);

/* Host-only view of the prefill path's tile order, for tests.  The host deals uncut tiles to
 * grid positions for the dispatcher (which gives the first 256 workgroups a CU each and
 * workgroup i + 256 the CU of workgroup i): between one and two workgroups per CU the longest
 * tiles get a CU to themselves and the others share one long with short; with more tiles than
 * workgroup slots the longest go first.  Writes the tile slot of every slot position
 * (min(n, capacity) entries; a slot is 8 column tiles of 16 query rows of one kv head group,
 * numbered as the prefill kernel numbers them) and returns n; 0 when the order is the natural
 * one or (beyond 512 tiles) simply reversed; CS_ERR_INVALID_ARG on bad arguments.  No device
 * work. */
int32_t cs_debug_prefill_order(const cs_batch* batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                               int32_t* slots, int32_t capacity);

/* Host-only view of one more launch decision, for tests: the pages a wavefront of the decode
 * kernel will keep in flight for this batch (1 or 2; see cs_set_decode_pages_ahead), or
 * CS_ERR_INVALID_ARG. */
int32_t cs_debug_decode_pages_ahead(const cs_batch* batch, int32_t num_kv_heads, int32_t head_dim);

/* Tuning knob for measurements and tests: pages (of 16 keys) a wavefront of the decode kernel
 * keeps in flight beyond the one it is multiplying: 1 or 2; 0 = automatic (by item length and
 * grid size).  Process-wide. */
void cs_set_decode_pages_ahead(int32_t pages);

/* Tuning knob for measurements and tests.  A call that holds both prefill chunks and decode
 * tokens can run as two kernels in a row, as one grid with the decode work behind the tiles, or
 * as one grid with one decode workgroup per CU beside the tiles (paper Sec. 4.2: both kinds of
 * work share an iteration).  1 (default): the host chooses from the batch's lengths; 0: always
 * two kernels; 2: always behind; 3: always beside.  All give the same bits.  Process-wide. */
void cs_set_mixed_fusion(int32_t mode);

/* Host-only view of that choice, for tests: 0 two kernels (also when the batch has only one kind
 * of work), 1 decode behind the tiles, 2 decode beside the tiles; CS_ERR_INVALID_ARG on bad
 * arguments.  No device work. */
int32_t cs_debug_mixed_arrangement(const cs_batch* batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim);

/* Host-only view of one more choice of a fused launch, for tests: the higher of the two issue
 * priorities its tile wavefronts alternate between -- 0: they stay at the default (also when the
 * call is not fused); 1: beside a decode workgroup per CU, and behind tiles that far outweigh the
 * decode work; 2 (always above the decode wavefronts, which stay at 0): beside, where the host's
 * model has the tiles outlast the decode stream by less than its own length.
 * CS_ERR_INVALID_ARG on bad arguments.  No device work. */
int32_t cs_debug_mixed_tile_priority(const cs_batch* batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim);

/* Host-only view of the key-range cut of the batch's prefill tiles, for tests: returns the number
 * of tile slots in launch order (a slot is 8 column tiles of 16 query rows of one kv head group;
 * slots of sequences without a chunk are empty), *first_cut the launch position from which tiles
 * are cut (0: every tile that is long enough; beside the tiles the host cuts only the last
 * round's), *ranges the ranges of the longest cut tile (1: nothing is cut; a batch without chunks
 * has 0 slots and 1 range).  CS_ERR_INVALID_ARG on bad arguments.  No device work. */
int32_t cs_debug_mixed_tail_cut(const cs_batch* batch, int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                                int32_t* first_cut, int32_t* ranges);

/* The host's model of a fused grid's tile workgroups, for tests (no device work): n workgroups
 * that take work_us[i] microseconds each beside another tile, 0.78 of that alone on their CU
 * and 1.1 of it beside a decode workgroup, are played in order through `cus` CUs of two
 * workgroup slots each (the first `cus` get a CU each, the next `cus` the second slot of those
 * CUs, later ones the slot that frees first); with decode_until_us > 0 one slot of every CU is a
 * decode workgroup's until then.  Returns when the last workgroup ends, or -1 on bad arguments. */
double cs_debug_play_tiles(const float* work_us, int32_t n, int32_t cus, double decode_until_us);

/* Tuning knob for measurements and tests: in a fused mixed launch, leave the tiles of the launch
 * positions before `whole_tiles` whole and cut those from it on into `ranges` key ranges (of the
 * longest tile's steps / ranges), whatever the host's model says; whole_tiles < 0 or ranges < 1:
 * the host decides again.  Process-wide; changes launch plans and workspace sizes. */
void cs_debug_set_tail_cut(int32_t whole_tiles, int32_t ranges);

const char* cs_status_string(int status);
/* Text of the last HIP error seen by this thread inside the library ("" if none). */
const char* cs_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CONSERVE_KV_H */
