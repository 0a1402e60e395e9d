"""Pins for the page format and the reference append / gather / restore copies."""
import os

import numpy as np
import pytest
import torch

from oracle import attention, kv_layout
from paper_2410_01228_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def test_paper_kv_bytes_per_token():
    g = dict(l.split() for l in open(os.path.join(GOLD, "paper_kv_sizes.txt"))
             if l.strip() and not l.startswith("#"))
    per_tok = kv_layout.kv_bytes_per_token(int(g["hkv"]), int(g["head_dim"]), int(g["layers"]))
    assert per_tok == int(g["kv_kib_per_token"]) * 1024
    # the paper's checkpoint-rate figure follows from it
    tok_s = int(g["pcie_gb_per_s"]) * 1024 ** 3 / per_tok
    assert int(tok_s / 1000) == int(g["tokens_per_s_thousands"])
    # page bytes per layer used by the copy kernels: 16 tokens of K and V
    assert kv_layout.page_elems(8, 128) * 2 == 64 * 1024
    assert synth.Shape(40, 8, 128, 48).page_elems == kv_layout.page_elems(8, 128)


def test_format_offsets_from_fixture():
    for line in open(os.path.join(GOLD, "page_format_offsets.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        kind, t, d, idx = line.split()
        f = kv_layout.k_index if kind == "K" else kv_layout.v_index
        assert int(f(int(t), int(d), 128)) == int(idx), line


@pytest.mark.parametrize("D", [64, 128])
def test_format_is_a_bijection_with_the_stated_units(D):
    t, d = np.meshgrid(np.arange(16), np.arange(D), indexing="ij")
    ki = kv_layout.k_index(t, d, D)
    vi = kv_layout.v_index(t, d, D)
    assert sorted(ki.ravel()) == list(range(16 * D))
    assert sorted(vi.ravel()) == list(range(16 * D))
    # K: a 16-byte unit = 8 consecutive features of one token; tokens of a block adjacent
    assert np.all(ki[:, 1:8] - ki[:, 0:7] == 1)
    assert np.all(ki[1:, 0] - ki[:-1, 0] == 8)
    assert np.all(ki[:, 8:] - ki[:, :-8] == 128)
    # V: a 16-byte unit = one feature of 8 consecutive tokens
    assert np.all(vi[1:8, :] - vi[0:7, :] == 1)
    assert np.all(vi[0, 1:16] - vi[0, 0:15] == 8)
    assert np.all(vi[8:, :] - vi[:-8, :] == 128)
    assert np.all(vi[:, 16:] - vi[:, :-16] == 256)


def _tiny_pool_and_step(fill=0xDEAD):
    b = synth.config_tiny()
    sh = b.shape
    g = synth.generator(0)
    k_new = bits(synth.randn_bf16((b.T, sh.Hkv, sh.D), g))
    v_new = bits(synth.randn_bf16((b.T, sh.Hkv, sh.D), g))
    pool = kv_layout.new_pool(1, b.num_pages, sh.Hkv, sh.D, fill)
    return b, pool, k_new, v_new


def test_append_touches_only_the_new_slots_and_reads_back():
    b, pool, k_new, v_new = _tiny_pool_and_step()
    sh = b.shape
    before = pool.copy()
    kv_layout.ref_append(pool, 0, b.block_tables.numpy(), b.ctx_lens.numpy(), b.cu_q_lens.numpy(), k_new, v_new)
    changed = pool != before
    # N(0,1) bf16 never equals the fill pattern, so every written element shows
    assert changed.sum() == b.T * 2 * sh.Hkv * sh.D
    # independent slot-by-slot check of where each element went
    for s in range(b.S):
        for i in range(int(b.q_lens[s])):
            pos = int(b.ctx_lens[s]) + i
            page, t = int(b.block_tables[s, pos // 16]), pos % 16
            tok = int(b.cu_q_lens[s]) + i
            for h in range(sh.Hkv):
                for d in (0, 7, 8, 31, sh.D - 1):
                    assert pool[0, page, 0, h, ((d // 8) * 16 + t) * 8 + d % 8] == k_new[tok, h, d]
                    assert pool[0, page, 1, h, (((d // 16) * 2 + t // 8) * 16 + d % 16) * 8 + t % 8] == v_new[tok, h, d]
    # reading back through the block table returns the appended rows at the new positions
    for s in range(b.S):
        c, q = int(b.ctx_lens[s]), int(b.q_lens[s])
        K, V = kv_layout.read_logical(pool, 0, b.block_tables[s].numpy(), c + q)
        lo = int(b.cu_q_lens[s])
        np.testing.assert_array_equal(K[c:], k_new[lo:lo + q])
        np.testing.assert_array_equal(V[c:], v_new[lo:lo + q])
        assert np.all(K[:c] == 0xDEAD) and np.all(V[:c] == 0xDEAD)


def test_append_twice_is_append_only():
    # a second step never rewrites what the first step stored
    b, pool, k_new, v_new = _tiny_pool_and_step()
    bt, cu = b.block_tables.numpy(), b.cu_q_lens.numpy()
    kv_layout.ref_append(pool, 0, bt, b.ctx_lens.numpy(), cu, k_new, v_new)
    snap = pool.copy()
    ctx2 = (b.ctx_lens + b.q_lens).numpy()
    one = np.arange(b.S + 1, dtype=np.int32)
    # next step: every request decodes one token (block tables of the tiny config have room
    # except where the next slot opens a new page; give those a spare page)
    bt2 = bt.copy()
    spare = list(b.spare_pages.numpy())
    for s in range(b.S):
        blk = ctx2[s] // 16
        if bt2[s, blk] < 0:
            bt2[s, blk] = spare.pop()
    kv_layout.ref_append(pool, 0, bt2, ctx2, one, k_new[:b.S], v_new[:b.S])
    changed = pool != snap
    assert changed.sum() == b.S * 2 * b.shape.Hkv * b.shape.D
    for s in range(b.S):
        K, _ = kv_layout.read_logical(pool, 0, bt2[s], int(ctx2[s]) + 1)
        K0, _ = kv_layout.read_logical(snap, 0, bt[s], int(ctx2[s]))
        np.testing.assert_array_equal(K[:-1], K0)


def test_tiny_config_fills_five_pages():
    # 2 pages by the first chunk (positions 0..31), 2 by the second (48..79), 1 by the decode
    # whose new token lands on slot 15 of its page (context 63); contexts 17, 40, 100 fill none
    b = synth.config_tiny()
    dirty = synth.newly_filled_pages(b)
    assert len(dirty) == 5 and len(set(dirty)) == 5
    bt = b.block_tables
    assert dirty == [int(bt[2, 3]), int(bt[4, 0]), int(bt[4, 1]), int(bt[5, 3]), int(bt[5, 4])]


def test_gather_restore_roundtrip_and_attention_unchanged():
    b, pool, k_new, v_new = _tiny_pool_and_step(fill=0)
    sh = b.shape
    g = synth.generator(0)
    pool[:] = bits(synth.randn_bf16(tuple(pool.shape), g))          # whole pool random
    bt = b.block_tables.numpy().copy()
    kv_layout.ref_append(pool, 0, bt, b.ctx_lens.numpy(), b.cu_q_lens.numpy(), k_new, v_new)
    dirty = synth.newly_filled_pages(b)
    staging = kv_layout.ref_gather(pool, 0, 1, dirty)
    assert staging.shape == (1, 5, sh.page_elems)
    for i, p in enumerate(dirty):
        np.testing.assert_array_equal(staging[0, i], pool[0, p].reshape(-1))
    # restore in place is the identity
    same = pool.copy()
    kv_layout.ref_restore(same, 0, 1, dirty, staging)
    np.testing.assert_array_equal(same, pool)
    # preempt: wipe the dirty pages, resume into fresh pages, rewrite the block tables
    fresh = [int(x) for x in b.spare_pages[:5]]
    moved = pool.copy()
    for p in dirty:
        moved[0, p] = 0x7FC0                                         # NaN pattern
    kv_layout.ref_restore(moved, 0, 1, fresh, staging)
    bt2 = bt.copy()
    for old, new in zip(dirty, fresh):
        bt2[bt == old] = new
    q = synth.randn_bf16((b.T, sh.Hq, sh.D), g).float().numpy()
    for s in range(b.S):
        n = int(b.ctx_lens[s] + b.q_lens[s])
        K1, V1 = kv_layout.read_logical(pool, 0, bt[s], n)
        K2, V2 = kv_layout.read_logical(moved, 0, bt2[s], n)
        np.testing.assert_array_equal(K1, K2)
        np.testing.assert_array_equal(V1, V2)
        lo, hi = int(b.cu_q_lens[s]), int(b.cu_q_lens[s + 1])
        o1 = attention.attention_chunk(q[lo:hi], kv_layout.bf16_bits_to_f32(K1), kv_layout.bf16_bits_to_f32(V1),
                                       int(b.ctx_lens[s]), sh.scale)
        o2 = attention.attention_chunk(q[lo:hi], kv_layout.bf16_bits_to_f32(K2), kv_layout.bf16_bits_to_f32(V2),
                                       int(b.ctx_lens[s]), sh.scale)
        np.testing.assert_array_equal(o1, o2)


def test_gather_layer_range_and_duplicates():
    rng = np.random.default_rng(3)
    pool = rng.integers(0, 2 ** 16, size=(3, 7, 2, 2, 16 * 64), dtype=np.uint16)
    ids = [5, 0, 5, 3]
    st = kv_layout.ref_gather(pool, 1, 3, ids)
    assert st.shape == (2, 4, 2 * 2 * 16 * 64)
    np.testing.assert_array_equal(st[0, 0], st[0, 2])
    np.testing.assert_array_equal(st[1, 3], pool[2, 3].reshape(-1))
    empty = kv_layout.ref_gather(pool, 0, 3, [])
    assert empty.shape == (3, 0, 2 * 2 * 16 * 64)
    p2 = pool.copy()
    kv_layout.ref_restore(p2, 0, 3, [], empty)
    np.testing.assert_array_equal(p2, pool)


def test_token_gather_returns_the_appended_rows_and_restore_inverts_it():
    """Token-granular checkpoint: gathering the slots a step has just appended to returns
    exactly that step's k_new / v_new rows (the append is pinned slot by slot above); restoring
    them into other slots moves those rows and nothing else."""
    b, pool, k_new, v_new = _tiny_pool_and_step()
    sh = b.shape
    kv_layout.ref_append(pool, 0, b.block_tables.numpy(), b.ctx_lens.numpy(), b.cu_q_lens.numpy(), k_new, v_new)
    slots = []
    for s in range(b.S):
        for i in range(int(b.q_lens[s])):
            pos = int(b.ctx_lens[s]) + i
            slots.append(int(b.block_tables[s, pos // 16]) * 16 + pos % 16)
    st = kv_layout.ref_gather_tokens(pool, 0, 1, slots)
    assert st.shape == (1, b.T, 2, sh.Hkv, sh.D)
    np.testing.assert_array_equal(st[0, :, 0], k_new)
    np.testing.assert_array_equal(st[0, :, 1], v_new)
    # restore into the slots of spare pages, in a different order of slots within the pages
    spare = [int(p) for p in b.spare_pages.numpy()]
    assert len(spare) * 16 >= len(slots)
    new_slots = [spare[i // 16] * 16 + (15 - i % 16) for i in range(len(slots))]
    before = pool.copy()
    kv_layout.ref_restore_tokens(pool, 0, 1, new_slots, st)
    assert (pool != before).sum() == b.T * 2 * sh.Hkv * sh.D         # the fill never equals a drawn value
    np.testing.assert_array_equal(kv_layout.ref_gather_tokens(pool, 0, 1, new_slots), st)
    # a restored slot reads back through a block table that names its page
    K, V = kv_layout.read_logical(pool, 0, np.array([spare[0]]), 16)
    for i in range(min(16, len(slots))):
        np.testing.assert_array_equal(K[15 - i], k_new[i])
        np.testing.assert_array_equal(V[15 - i], v_new[i])
    # the sixteen slots of one page, gathered token by token, are the page's blob re-ordered:
    # element counts and multiset agree with the page gather
    page = int(b.block_tables[4, 0])
    tok = kv_layout.ref_gather_tokens(pool, 0, 1, [page * 16 + t for t in range(16)])
    blob = kv_layout.ref_gather(pool, 0, 1, [page])
    np.testing.assert_array_equal(np.sort(tok.reshape(-1)), np.sort(blob.reshape(-1)))


def test_token_gather_layer_range():
    sh = synth.Shape(4, 2, 64, L=3)
    g = synth.generator(7)
    pool = bits(synth.randn_bf16((3, 5, 2, sh.Hkv, 16 * sh.D), g)).copy()
    slots = [3 * 16 + 15, 0, 4 * 16 + 7, 3 * 16 + 15]                 # duplicates allowed in a gather
    st = kv_layout.ref_gather_tokens(pool, 1, 3, slots)
    assert st.shape == (2, 4, 2, sh.Hkv, sh.D)
    np.testing.assert_array_equal(st[:, 0], st[:, 3])
    for l in (1, 2):
        K, V = kv_layout.read_logical(pool, l, np.array([4]), 16)
        np.testing.assert_array_equal(st[l - 1, 2, 0], K[7])
        np.testing.assert_array_equal(st[l - 1, 2, 1], V[7])
    with pytest.raises(AssertionError):
        kv_layout.ref_gather_tokens(pool, 0, 1, [5 * 16])


def test_bf16_widening_is_exact():
    x = synth.randn_bf16((1000,), synth.generator(9))
    np.testing.assert_array_equal(kv_layout.bf16_bits_to_f32(bits(x)), x.float().numpy())


# ---- pages of 8 tokens ------------------------------------------------------------------

@pytest.mark.parametrize("D", [64, 128])
def test_page8_format_is_a_bijection_with_the_stated_units(D):
    t, d = np.meshgrid(np.arange(8), np.arange(D), indexing="ij")
    ki = kv_layout.k_index(t, d, D, page_size=8)
    vi = kv_layout.v_index(t, d, D, page_size=8)
    assert sorted(ki.ravel()) == list(range(8 * D))
    assert sorted(vi.ravel()) == list(range(8 * D))
    # K: 8 features of a token adjacent, the 8 tokens of a feature block adjacent, blocks 64 apart
    assert np.all(ki[:, 1:8] - ki[:, 0:7] == 1)
    assert np.all(ki[1:, 0] - ki[:-1, 0] == 8)
    assert np.all(ki[:, 8:] - ki[:, :-8] == 64)
    # V: the 8 tokens of a feature adjacent, features 8 apart: feature d starts at element 8 d
    assert np.all(vi[1:, :] - vi[:-1, :] == 1)
    assert np.all(vi[0, :] == 8 * np.arange(D))


@pytest.mark.parametrize("D", [64, 128])
def test_a_page_of_16_is_two_pages_of_8_interleaved_by_16_byte_units(D):
    """Tokens 0..7 in page A and 8..15 in page B (8 tokens each) against the same 16 tokens in
    one page P: every K feature block of P is A's block followed by B's, every V feature tile of
    P is A's tile followed by B's -- the fact the attention kernels lean on when they put two
    small pages where one page of 16 would be."""
    rng = np.random.default_rng(D)
    k = rng.integers(0, 2 ** 16, size=(16, 1, D), dtype=np.uint16)
    v = rng.integers(0, 2 ** 16, size=(16, 1, D), dtype=np.uint16)
    big = kv_layout.new_pool(1, 1, 1, D, 0)
    kv_layout.ref_append(big, 0, np.array([[0]]), np.array([0]), np.array([0, 16]), k, v)
    small = kv_layout.new_pool(1, 2, 1, D, 0, page_size=8)
    kv_layout.ref_append(small, 0, np.array([[1, 0]]), np.array([0]), np.array([0, 16]), k, v, page_size=8)
    A, B = small[0, 1], small[0, 0]                                  # [2, 1, 8*D]
    Pk = big[0, 0, 0, 0].reshape(D // 8, 2, 64)                      # [feature block][token half][8 tokens x 8]
    np.testing.assert_array_equal(Pk[:, 0], A[0, 0].reshape(D // 8, 64))
    np.testing.assert_array_equal(Pk[:, 1], B[0, 0].reshape(D // 8, 64))
    Pv = big[0, 0, 1, 0].reshape(D // 16, 2, 128)                    # [feature tile][token half][16 x 8 tokens]
    np.testing.assert_array_equal(Pv[:, 0], A[1, 0].reshape(D // 16, 128))
    np.testing.assert_array_equal(Pv[:, 1], B[1, 0].reshape(D // 16, 128))


def test_page8_append_reads_back_and_token_copies_invert():
    sh = synth.Shape(4, 2, 64, page_size=8)
    g = synth.generator(21)
    b = synth.make_batch(sh, [7, 8, 23, 0, 5, 40], [1, 1, 1, 17, 0, 9], g, spare=6)
    assert [int(x) for x in b.blocks_needed()] == [1, 2, 3, 3, 1, 7]
    k_new = bits(synth.randn_bf16((b.T, sh.Hkv, sh.D), g))
    v_new = bits(synth.randn_bf16((b.T, sh.Hkv, sh.D), g))
    pool = kv_layout.new_pool(1, b.num_pages, sh.Hkv, sh.D, 0xDEAD, page_size=8)
    assert pool.shape[-1] == 8 * sh.D and kv_layout.page_elems(sh.Hkv, sh.D, 8) == sh.page_elems
    before = pool.copy()
    bt = b.block_tables.numpy()
    kv_layout.ref_append(pool, 0, bt, b.ctx_lens.numpy(), b.cu_q_lens.numpy(), k_new, v_new, page_size=8)
    assert (pool != before).sum() == b.T * 2 * sh.Hkv * sh.D
    slots = []
    for s in range(b.S):
        c, q = int(b.ctx_lens[s]), int(b.q_lens[s])
        for i in range(q):
            pos, tok = c + i, int(b.cu_q_lens[s]) + i
            page, t = int(bt[s, pos // 8]), pos % 8
            slots.append(page * 8 + t)
            for h in range(sh.Hkv):
                for d in (0, 7, 8, 17, sh.D - 1):
                    assert pool[0, page, 0, h, ((d // 8) * 8 + t) * 8 + d % 8] == k_new[tok, h, d]
                    assert pool[0, page, 1, h, d * 8 + t] == v_new[tok, h, d]
        K, V = kv_layout.read_logical(pool, 0, bt[s], c + q, page_size=8)
        lo = int(b.cu_q_lens[s])
        np.testing.assert_array_equal(K[c:], k_new[lo:lo + q])
        np.testing.assert_array_equal(V[c:], v_new[lo:lo + q])
    # the pages filled this step: a page is full when its 8th slot is written
    assert synth.newly_filled_pages(b) == [int(bt[0, 0]), int(bt[2, 2]), int(bt[3, 0]), int(bt[3, 1]), int(bt[5, 5])]
    st = kv_layout.ref_gather_tokens(pool, 0, 1, slots, page_size=8)
    np.testing.assert_array_equal(st[0, :, 0], k_new)
    np.testing.assert_array_equal(st[0, :, 1], v_new)
    moved = before.copy()
    kv_layout.ref_restore_tokens(moved, 0, 1, slots, st, page_size=8)
    np.testing.assert_array_equal(moved, pool)
