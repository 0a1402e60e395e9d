"""KV-pool format and the reference copies over it (test infrastructure only).

The paper fixes only that the KV cache is managed in pages of 16 tokens reached through a
per-request page table, that it is append-only, and that checkpointing gathers scattered
pages into one contiguous buffer (Sec. 4.4 and Sec. 5).  The byte format inside a page is
this library's own and is restated here independently, as plain index arithmetic.

Pool, in bf16 elements:   pool[layer][page][kv (0 = K, 1 = V)][kv_head][16 * D]
so one (layer, page) is one contiguous blob of 2 * Hkv * 16 * D elements.  (Pages of 8 tokens,
a finer granularity than the paper's own, use the same format with 8 in place of 16 tokens
and one token group in place of two: every function takes page_size, default 16.)

Inside a K block (one page, one kv head; token t in 0..15, feature d in 0..D-1):
    element index = ((d // 8) * 16 + t) * 8 + d % 8
    i.e. [D/8 feature blocks][16 tokens][8 features]: a 16-byte unit is 8 consecutive
    features of one token, and the 16 tokens of a feature block are adjacent.
Inside a V block:
    element index = (((d // 16) * 2 + t // 8) * 16 + d % 16) * 8 + t % 8
    i.e. [D/16 feature tiles][2 token halves][16 features][8 tokens]: a 16-byte unit is one
    feature of 8 consecutive tokens.

Arrays here are numpy uint16 (bf16 bit patterns); copies are bit copies.
"""
import numpy as np

PAGE = 16


def k_index(t, d, D, page_size=PAGE):
    """Element index of K[token t][feature d] inside its block (pages of `page_size` tokens)."""
    t = np.asarray(t)
    d = np.asarray(d)
    return ((d // 8) * page_size + t) * 8 + d % 8


def v_index(t, d, D, page_size=PAGE):
    """Element index of V[token t][feature d] inside its block (pages of `page_size` tokens, a
    multiple of 8: a page holds page_size // 8 token groups)."""
    t = np.asarray(t)
    d = np.asarray(d)
    return (((d // 16) * (page_size // 8) + t // 8) * 16 + d % 16) * 8 + t % 8


def page_elems(Hkv, D, page_size=PAGE):
    """bf16 elements of one (layer, page): K and V of every kv head."""
    return 2 * Hkv * page_size * D


def kv_bytes_per_token(Hkv, D, L):
    """Bytes of KV cache one token occupies over L layers (bf16)."""
    return 2 * Hkv * D * 2 * L


def new_pool(L, P, Hkv, D, fill=0, page_size=PAGE):
    return np.full((L, P, 2, Hkv, page_size * D), fill, dtype=np.uint16)


def ref_append(pool, layer, block_tables, ctx_lens, cu_q_lens, k_new, v_new, page_size=PAGE):
    """Append this step's new K/V rows (paper Sec. 1 / 4.4: the cache is append-only).

    New token i of request s goes to position pos = ctx_lens[s] + i, i.e. to page
    block_tables[s][pos // page_size], token slot pos % page_size.  k_new / v_new: uint16 [T, Hkv, D],
    packed in request order (cu_q_lens = prefix sums of the requests' new-token counts).
    Every other slot of the pool is left untouched.  In place.
    """
    L, P, _, Hkv, BD = pool.shape
    D = BD // page_size
    d = np.arange(D)
    for s in range(len(ctx_lens)):
        for i in range(int(cu_q_lens[s + 1]) - int(cu_q_lens[s])):
            tok = int(cu_q_lens[s]) + i
            pos = int(ctx_lens[s]) + i
            page = int(block_tables[s][pos // page_size])
            assert 0 <= page < P, "block table entry out of range"
            t = pos % page_size
            for h in range(Hkv):
                pool[layer, page, 0, h, k_index(t, d, D, page_size)] = k_new[tok, h, :]
                pool[layer, page, 1, h, v_index(t, d, D, page_size)] = v_new[tok, h, :]
    return pool


def read_logical(pool, layer, block_table_row, n, page_size=PAGE):
    """Logical K, V (uint16 [n, Hkv, D]) of a request holding n tokens, read through its
    block table row: the inverse of the format above."""
    L, P, _, Hkv, BD = pool.shape
    D = BD // page_size
    K = np.empty((n, Hkv, D), dtype=np.uint16)
    V = np.empty((n, Hkv, D), dtype=np.uint16)
    d = np.arange(D)
    t = np.arange(page_size)
    ki = k_index(t[:, None], d[None, :], D, page_size)      # [page_size, D]
    vi = v_index(t[:, None], d[None, :], D, page_size)
    for b in range((n + page_size - 1) // page_size):
        page = int(block_table_row[b])
        cnt = min(page_size, n - b * page_size)
        kb = pool[layer, page, 0][:, ki]          # [Hkv, page_size, D]
        vb = pool[layer, page, 1][:, vi]
        K[b * page_size:b * page_size + cnt] = kb.transpose(1, 0, 2)[:cnt]
        V[b * page_size:b * page_size + cnt] = vb.transpose(1, 0, 2)[:cnt]
    return K, V


def ref_gather(pool, layer_begin, layer_end, page_ids):
    """Checkpoint gather (paper Sec. 5: scattered pages -> one contiguous buffer):
    staging[l - layer_begin][i] = whole page pool[l][page_ids[i]] (K and V)."""
    L, P, _, Hkv, BD = pool.shape
    n = len(page_ids)
    staging = np.empty((layer_end - layer_begin, n, 2 * Hkv * BD), dtype=np.uint16)
    for l in range(layer_begin, layer_end):
        for i in range(n):
            staging[l - layer_begin, i, :] = pool[l, int(page_ids[i])].reshape(-1)
    return staging


def ref_restore(pool, layer_begin, layer_end, page_ids, staging):
    """Restore (paper Sec. 4.4, prefetch on resume): pool[l][page_ids[i]] = staging[l][i].
    In place; the ids are distinct."""
    L, P, _, Hkv, BD = pool.shape
    for l in range(layer_begin, layer_end):
        for i in range(len(page_ids)):
            pool[l, int(page_ids[i])] = staging[l - layer_begin, i].reshape(2, Hkv, BD)
    return pool


def ref_gather_tokens(pool, layer_begin, layer_end, token_slots, page_size=PAGE):
    """Token-granular checkpoint gather (paper Sec. 4.4: KV state is managed per token, and
    after each generation step only the newly generated tokens are checkpointed).
    token_slots[i] = page * page_size + slot names one cached token;
        staging[l - layer_begin][i][0] = its K rows [Hkv][D],  staging[...][i][1] = its V rows,
    i.e. plain row layout, no page format left in the buffer."""
    L, P, _, Hkv, BD = pool.shape
    D = BD // page_size
    d = np.arange(D)
    n = len(token_slots)
    staging = np.empty((layer_end - layer_begin, n, 2, Hkv, D), dtype=np.uint16)
    for l in range(layer_begin, layer_end):
        for i in range(n):
            page, t = divmod(int(token_slots[i]), page_size)
            assert 0 <= page < P, "token slot out of range"
            for h in range(Hkv):
                staging[l - layer_begin, i, 0, h, :] = pool[l, page, 0, h, k_index(t, d, D, page_size)]
                staging[l - layer_begin, i, 1, h, :] = pool[l, page, 1, h, v_index(t, d, D, page_size)]
    return staging


def ref_restore_tokens(pool, layer_begin, layer_end, token_slots, staging, page_size=PAGE):
    """Inverse of ref_gather_tokens: the rows of staging[l][i] go to the token slot
    token_slots[i] of every layer; every other element of the pool is left untouched.
    In place; the slots are distinct."""
    L, P, _, Hkv, BD = pool.shape
    D = BD // page_size
    d = np.arange(D)
    for l in range(layer_begin, layer_end):
        for i in range(len(token_slots)):
            page, t = divmod(int(token_slots[i]), page_size)
            assert 0 <= page < P, "token slot out of range"
            for h in range(Hkv):
                pool[l, page, 0, h, k_index(t, d, D, page_size)] = staging[l - layer_begin, i, 0, h, :]
                pool[l, page, 1, h, v_index(t, d, D, page_size)] = staging[l - layer_begin, i, 1, h, :]
    return pool


def bf16_bits_to_f32(bits):
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    return (np.asarray(bits).astype(np.uint32) << 16).view(np.float32)
