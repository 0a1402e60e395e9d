"""GPU parity of cs_paged_attention_mixed against the fp64 oracle on logical sequences."""
import numpy as np
import pytest
import torch

from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import Step, assert_attention_close, bits, from_bits

pytestmark = pytest.mark.gpu


def run_step(batch, seed, q_gain=1.0, split=0, check_append=True, dtype=torch.bfloat16, fuse=1, ahead=0):
    """append + attention through the C ABI; returns (gpu_out, Step, device pool, cs.Batch)."""
    st = Step(batch, seed, q_gain=q_gain, dtype=dtype)
    sh = batch.shape
    cpu_pool = st.prior_pool()
    pool = cs.Pool(from_bits(cpu_pool, "cuda", dtype), cpu_pool.shape[0], cpu_pool.shape[1], sh.Hkv, sh.D,
                   page_size=sh.page_size)
    attend = cs.cs_paged_attention_mixed if dtype == torch.bfloat16 else cs.cs_paged_attention_mixed_f16
    bb = cs.Batch(batch.block_tables, batch.ctx_lens, batch.cu_q_lens)
    cs.cs_kv_append(pool, 0, bb, st.k_new.cuda(), st.v_new.cuda())
    if check_append:
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits(pool.tensor), st.oracle_append(cpu_pool))
    cs.cs_set_decode_split_tokens(split)
    cs.cs_set_mixed_fusion(fuse)
    cs.cs_set_decode_pages_ahead(ahead)
    try:
        ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
        out = torch.full((batch.T, sh.Hq, sh.D), float("nan"), dtype=dtype, device="cuda")
        attend(pool, 0, bb, st.q.cuda(), out, sh.Hq, sh.scale, ws)
        torch.cuda.synchronize()
    finally:
        cs.cs_set_decode_split_tokens(0)
        cs.cs_set_mixed_fusion(1)
        cs.cs_set_decode_pages_ahead(0)
    return out, st, pool, bb


def decode_batch(sh, ctxs, seed, spare=0):
    return synth.make_batch(sh, ctxs, [1] * len(ctxs), synth.generator(seed), spare=spare)


@pytest.mark.parametrize("split", [0, 16, 64])
def test_decode_small_contexts(split):
    # page boundaries: n = ctx+1 in {1, 2, 15, 16, 17, 32, 33, 101, ...}
    sh = synth.Shape(4, 2, 64)
    b = decode_batch(sh, [0, 1, 14, 15, 16, 31, 32, 100, 63, 40, 17, 255, 256, 300], 21)
    out, st, _, _ = run_step(b, 21, split=split)
    assert_attention_close(out, st.oracle_attention(), "decode small split=%d" % split)


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (28, 4, 128), (64, 8, 128), (40, 8, 128), (16, 1, 64), (6, 6, 128)])
def test_decode_group_sizes(Hq, Hkv, D):
    sh = synth.Shape(Hq, Hkv, D)
    b = decode_batch(sh, [700, 33, 1024, 257, 511], 22)
    out, st, _, _ = run_step(b, 22, split=256)
    assert_attention_close(out, st.oracle_attention(), "decode G=%d D=%d" % (Hq // Hkv, D))


def test_decode_peaked_softmax():
    # queries scaled x6: the softmax is sharp, so a masking or indexing slip moves outputs by O(1)
    sh = synth.Shape(8, 2, 128)
    b = decode_batch(sh, [5, 130, 999, 2047, 77], 23)
    out, st, _, _ = run_step(b, 23, q_gain=6.0, split=128)
    assert_attention_close(out, st.oracle_attention(), "decode peaked")


@pytest.mark.parametrize("S,split", [(880, 0), (881, 0), (1000, 128), (300, 64), (500, 64)])
def test_decode_item_list_sources(S, split):
    """The work-item list travels in the kernel arguments up to 880 items (longest first) and
    is built by the planning kernel beyond that: 880 and 881 uncut sequences sit either side
    of the limit, 1000 sequences cut at 128 keys need the planning kernel and the merge, 300
    sequences cut at 64 keys exceed the limit through their pieces."""
    sh = synth.Shape(4, 2, 64)
    ctxs = synth.uniform_int(0, 300, S, synth.generator(40 + S)).tolist()
    b = decode_batch(sh, ctxs, 41)
    out, st, _, _ = run_step(b, 41, split=split, check_append=False)
    assert_attention_close(out, st.oracle_attention(), "decode S=%d split=%d" % (S, split))


@pytest.mark.parametrize("Hq,Hkv,D,split,dtype", [(4, 2, 64, 0, torch.bfloat16), (32, 8, 128, 64, torch.bfloat16),
                                                   (28, 4, 128, 256, torch.bfloat16), (8, 2, 128, 32, torch.float16)])
def test_decode_pages_ahead(Hq, Hkv, D, split, dtype):
    """The decode kernel exists with one and with two pages in flight per wavefront (the host
    picks by the size of the batch).  A wavefront multiplies its pages in the same order either
    way, so the outputs are bit-identical; contexts chosen so that wavefronts get 0, 1, 2, 3
    and many pages, with and without cutting."""
    sh = synth.Shape(Hq, Hkv, D)
    ctxs = [0, 15, 16, 31, 47, 63, 64, 100, 127, 128, 191, 200, 255, 300, 1000, 2047, 2500]
    b = decode_batch(sh, ctxs, 52)
    o1, st, _, _ = run_step(b, 52, split=split, dtype=dtype, ahead=1)
    o2, _, _, _ = run_step(b, 52, split=split, dtype=dtype, ahead=2)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    check = assert_attention_close if dtype == torch.bfloat16 else assert_close_f16
    check(o2, st.oracle_attention(), "two pages ahead %d/%d/%d split %d" % (Hq, Hkv, D, split))


def test_decode_llama8b_shrunk():
    b = synth.config_llama8b_decode(shrink=8)
    out, st, _, _ = run_step(b, 1)
    assert_attention_close(out, st.oracle_attention(), "llama8b/8")


# ------------------------------------------------------------------------------------
# prefill chunks and mixed batches
# ------------------------------------------------------------------------------------

def test_tiny_config_end_to_end():
    """Workload 0: append + mixed attention, then checkpoint the 5 newly filled pages,
    resume them into fresh pages with rewritten block tables: the attention output must not
    change by a single bit (preempt/resume is invisible to the request)."""
    b = synth.config_tiny()
    sh = b.shape
    out, st, pool, bb = run_step(b, 0)
    assert_attention_close(out, st.oracle_attention(), "tiny mixed")
    dirty = synth.newly_filled_pages(b)
    fresh = [int(x) for x in b.spare_pages[:len(dirty)]]
    staging = torch.empty((1, len(dirty), sh.page_elems), dtype=torch.bfloat16, device="cuda")
    cs.cs_kv_ckpt_gather(pool, 0, 1, torch.tensor(dirty, dtype=torch.int32, device="cuda"), staging)
    torch.cuda.synchronize()
    flat = pool.tensor.view(sh.L, b.num_pages, -1)
    flat[:, dirty] = float("nan")                                   # the old pages are released
    cs.cs_kv_ckpt_restore(pool, 0, 1, torch.tensor(fresh, dtype=torch.int32, device="cuda"), staging)
    bt2 = b.block_tables.clone()
    for old, new in zip(dirty, fresh):
        bt2[b.block_tables == old] = new
    bb2 = cs.Batch(bt2, b.ctx_lens, b.cu_q_lens)
    out2 = torch.full_like(out, float("nan"))
    cs.cs_paged_attention_mixed(pool, 0, bb2, st.q.cuda(), out2, sh.Hq, sh.scale, cs.workspace_for(bb2, sh.Hq, sh.Hkv, sh.D))
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 2, 64), (32, 8, 128), (28, 4, 128), (40, 8, 128), (16, 1, 64), (3, 3, 128), (8, 8, 64)])
def test_prefill_chunks_ragged(Hq, Hkv, D):
    # chunk lengths that are not multiples of the tile, prior contexts on and off page
    # boundaries, a first chunk (context 0), a 2-token chunk
    sh = synth.Shape(Hq, Hkv, D)
    b = synth.make_batch(sh, [0, 48, 17, 255, 5, 100], [32, 32, 50, 77, 2, 129], synth.generator(31))
    out, st, _, _ = run_step(b, 31)
    assert_attention_close(out, st.oracle_attention(), "prefill ragged %d/%d/%d" % (Hq, Hkv, D))


def test_prefill_interleaved_with_decodes_and_idle():
    # chunks, decode tokens and idle sequences in arbitrary order: workgroup slots without a
    # tile sit between the tiles
    sh = synth.Shape(8, 2, 128)
    b = synth.make_batch(sh, [700, 30, 0, 0, 99, 15, 2000, 64], [40, 1, 33, 0, 1, 1, 64, 300], synth.generator(34))
    out, st, _, _ = run_step(b, 34)
    active = [s for s in range(b.S) if int(b.q_lens[s]) > 0]
    assert_attention_close(out, st.oracle_attention(active), "interleaved")


def test_prefill_first_row_is_v0_exactly():
    # the first token of a first chunk sees only itself: out = v0, exact in bf16
    sh = synth.Shape(4, 2, 64)
    b = synth.make_batch(sh, [0], [40], synth.generator(32))
    out, st, _, _ = run_step(b, 32)
    v0 = st.v_new[0]                                               # [Hkv, D]
    for h in range(sh.Hq):
        assert torch.equal(out[0, h].cpu(), v0[h // sh.G])


def test_prefill_peaked_softmax():
    sh = synth.Shape(8, 2, 128)
    b = synth.make_batch(sh, [0, 333, 1000], [96, 64, 40], synth.generator(33))
    out, st, _, _ = run_step(b, 33, q_gain=6.0)
    assert_attention_close(out, st.oracle_attention(), "prefill peaked")


@pytest.mark.parametrize("maker,seed,shrink", [(synth.config_qwen7b_mixed, 2, 8), (synth.config_llama70b_long, 3, 16),
                                               (synth.config_qwen14b_ckpt, 4, 16)])
def test_mixed_shrunk_configs(maker, seed, shrink):
    b = maker(shrink=shrink)
    if b.shape.L > 1:
        b.shape.L = 1
    out, st, _, _ = run_step(b, seed)
    active = [s for s in range(b.S) if int(b.q_lens[s]) > 0]
    assert_attention_close(out, st.oracle_attention(active), b.name)


def test_preemption_drops_offline_tail_without_touching_online_rows():
    """Layer-wise preemption hands the same arrays with a smaller num_seqs: the online rows
    must be bit-identical with and without the offline sequences in the batch."""
    b = synth.config_qwen7b_mixed(shrink=16)
    sh = b.shape
    n_on = b.extra["n_online"]
    out, st, pool, bb = run_step(b, 2)
    bb_on = bb.truncated(n_on)
    out_on = torch.full_like(out, float("nan"))
    ws = cs.workspace_for(bb_on, sh.Hq, sh.Hkv, sh.D)
    cs.cs_paged_attention_mixed(pool, 0, bb_on, st.q.cuda(), out_on, sh.Hq, sh.scale, ws)
    torch.cuda.synchronize()
    T_on = bb_on.num_tokens
    assert T_on == n_on
    if cs.cs_paged_attention_workspace_bytes(bb, sh.Hq, sh.Hkv, sh.D) == cs.cs_paged_attention_workspace_bytes(bb_on, sh.Hq, sh.Hkv, sh.D):
        assert torch.equal(out[:T_on].view(torch.int16), out_on[:T_on].view(torch.int16))
    assert_attention_close(out_on[:T_on], st.oracle_attention(range(n_on))[:T_on], "online only")
    assert torch.isnan(out_on[T_on:].float()).all()                  # offline rows were not written


def test_online_prefill_with_offline_decodes():
    """The other mix the paper describes (Sec. 4.2): an online request in its prefill phase
    batched with offline requests that are decoding.  Online sequences still come first, so
    cutting the batch after them leaves the online rows bit-identical."""
    sh = synth.Shape(28, 4, 128)
    ctx = [0, 300, 1200, 64, 2047, 801, 33, 1500, 500]
    ql = [200, 96, 1, 1, 1, 1, 1, 1, 64]          # 2 online prompts + 2 online decodes | 4 offline decodes + 1 offline chunk
    n_on = 4
    b = synth.make_batch(sh, ctx, ql, synth.generator(35))
    out, st, pool, bb = run_step(b, 35)
    assert_attention_close(out, st.oracle_attention(), "online prefill + offline decode")
    bb_on = bb.truncated(n_on)
    out_on = torch.full_like(out, float("nan"))
    cs.cs_paged_attention_mixed(pool, 0, bb_on, st.q.cuda(), out_on, sh.Hq, sh.scale,
                                cs.workspace_for(bb_on, sh.Hq, sh.Hkv, sh.D))
    torch.cuda.synchronize()
    T_on = int(b.cu_q_lens[n_on])
    assert_attention_close(out_on[:T_on], st.oracle_attention(list(range(n_on)))[:T_on], "online prefix alone")
    assert (out[:T_on].float() - out_on[:T_on].float()).abs().max().item() <= 2e-2
    assert torch.isnan(out_on[T_on:].float()).all()                 # offline rows are not touched


# ------------------------------------------------------------------------------------
# fp16 variant (the paper's serving precision, Sec. 6.1): same kernels on the f16 matrix
# instructions; append and the copies are shared (they move 16-bit words)
# ------------------------------------------------------------------------------------

def assert_close_f16(out, ref, what):
    """fp16 keeps 3 more mantissa bits than bf16: besides the common bar, the error must be
    well inside it (a bf16 rounding slipped into the f16 path would not be)."""
    assert_attention_close(out, ref, what)
    g = out.detach().float().cpu().numpy().astype(np.float64)
    rows = ~np.isnan(ref).any(axis=(1, 2))
    rel = np.linalg.norm(g[rows] - ref[rows]) / np.linalg.norm(ref[rows])
    assert rel <= 2e-3, "%s: relative Frobenius error %.2e, expected fp16-level accuracy" % (what, rel)


@pytest.mark.parametrize("split", [0, 64])
def test_f16_decode(split):
    sh = synth.Shape(28, 4, 128)
    b = decode_batch(sh, [0, 15, 16, 700, 33, 1024, 257, 2047], 51)
    out, st, _, _ = run_step(b, 51, split=split, dtype=torch.float16)
    assert_close_f16(out, st.oracle_attention(), "f16 decode split=%d" % split)


@pytest.mark.parametrize("Hq,Hkv,D,gain", [(32, 8, 128, 1.0), (4, 2, 64, 1.0), (8, 2, 128, 6.0)])
def test_f16_prefill_and_mixed(Hq, Hkv, D, gain):
    sh = synth.Shape(Hq, Hkv, D)
    b = synth.make_batch(sh, [300, 64, 0, 48, 17, 1500, 5], [1, 1, 32, 50, 77, 40, 2], synth.generator(52))
    out, st, _, _ = run_step(b, 52, q_gain=gain, dtype=torch.float16)
    assert_close_f16(out, st.oracle_attention(), "f16 mixed %d/%d/%d" % (Hq, Hkv, D))


def test_f16_key_range_split_and_shrunk_config():
    sh = synth.Shape(8, 2, 128)
    b = synth.make_batch(sh, [3000, 1501, 0, 4100], [40, 17, 33, 1], synth.generator(61))
    out, st, _, _ = run_step(b, 61, dtype=torch.float16)
    assert_close_f16(out, st.oracle_attention(), "f16 prefill key ranges")
    b = synth.config_qwen7b_mixed(shrink=8)
    out, st, _, _ = run_step(b, 2, dtype=torch.float16)
    assert_close_f16(out, st.oracle_attention(), "f16 qwen7b/8")


@pytest.mark.parametrize("seed", list(range(48)))
def test_random_mixed_batches(seed):
    """Seeded random shapes and batches: any group size up to 16, either head_dim, decode
    tokens, chunks and idle sequences in any order, contexts on and off page boundaries, with
    the automatic and with a forced decode split, fused and separate launches, either decode
    prefetch depth."""
    import random
    rnd = random.Random(1000 + seed)
    D = rnd.choice([64, 128])
    Hkv = rnd.choice([1, 2, 3, 4, 8])
    G = rnd.choice([1, 2, 4, 5, 7, 8, 16])
    sh = synth.Shape(Hkv * G, Hkv, D)
    S = rnd.randint(1, 10)
    ctx, ql = [], []
    for _ in range(S):
        kind = rnd.choice(["decode", "decode", "chunk", "chunk", "idle"])
        c = rnd.choice([0, 1, 15, 16, 17, 31, 32, rnd.randint(0, 700), rnd.randint(0, 2500)])
        ctx.append(c)
        ql.append(1 if kind == "decode" else 0 if kind == "idle" else rnd.choice([2, 16, 17, rnd.randint(2, 150)]))
    if sum(ql) == 0:
        ql[0] = 1
    b = synth.make_batch(sh, ctx, ql, synth.generator(2000 + seed), spare=rnd.randint(0, 5))
    split = rnd.choice([0, 0, 64, 256])
    gain = rnd.choice([1.0, 1.0, 4.0])
    dtype = rnd.choice([torch.bfloat16, torch.bfloat16, torch.float16])
    fuse = rnd.choice([2, 1, 0])                           # decode behind the tiles always / the host's choice / two kernels in a row
    ahead = rnd.choice([0, 1, 2])                           # decode prefetch depth: automatic, one, two pages
    if rnd.choice([0, 1, 2]) == 0:
        fuse = 3                                            # a decode workgroup per CU beside the tiles
    out, st, _, _ = run_step(b, 2000 + seed, q_gain=gain, split=split, dtype=dtype, fuse=fuse, ahead=ahead)
    active = [s for s in range(S) if ql[s] > 0]
    assert_attention_close(out, st.oracle_attention(active),
                           "random seed %d: %d/%d/%d ctx %s q %s split %d gain %g %s" % (seed, sh.Hq, Hkv, D, ctx, ql, split, gain, dtype))


@pytest.mark.parametrize("Hq,Hkv,D,split,dtype", [(8, 2, 128, 0, torch.bfloat16), (28, 4, 128, 64, torch.bfloat16),
                                                   (16, 1, 64, 32, torch.bfloat16), (8, 2, 128, 64, torch.float16)])
def test_fused_and_separate_launches_agree(Hq, Hkv, D, split, dtype):
    """A batch with decode tokens and chunks runs as one fused grid, the decode work behind the
    tiles or beside them; with the fusion switched off the same work items run as two kernels in a
    row.  Same arithmetic in the same order: the outputs are bit-identical, and all meet the
    oracle."""
    sh = synth.Shape(Hq, Hkv, D)
    ctx = [700, 33, 0, 1500, 260, 15, 2047, 90, 5, 311]
    ql = [1, 100, 17, 1, 1, 48, 1, 0, 1, 2]
    b = synth.make_batch(sh, ctx, ql, synth.generator(77), spare=3)
    o1, st, _, _ = run_step(b, 77, split=split, dtype=dtype, fuse=2)
    o2, _, _, _ = run_step(b, 77, split=split, dtype=dtype, fuse=0)
    o3, _, _, _ = run_step(b, 77, split=split, dtype=dtype, fuse=3)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    assert torch.equal(o3.view(torch.int16), o2.view(torch.int16))
    active = [s for s in range(len(ql)) if ql[s] > 0]
    check = assert_attention_close if dtype == torch.bfloat16 else assert_close_f16
    check(o1, st.oracle_attention(active), "fused %d/%d/%d split %d" % (Hq, Hkv, D, split))


@pytest.mark.parametrize("Hq,Hkv,D,dtype", [(8, 2, 128, torch.bfloat16), (28, 4, 128, torch.bfloat16), (4, 2, 64, torch.float16)])
def test_fused_grid_with_a_sliver_of_decode_work(Hq, Hkv, D, dtype):
    """Prefill-heavy mix: the host takes the fused kernel whose tiles alternate their issue
    priority (decode side under 0.3 of the prefill side's ideal time).  Priorities change no
    arithmetic: bit-identical to the separate launches, and both meet the oracle."""
    sh = synth.Shape(Hq, Hkv, D)
    ctx = [40, 900, 0, 17, 2000]
    ql = [1, 300, 130, 1, 260]
    b = synth.make_batch(sh, ctx, ql, synth.generator(78), spare=2)
    o1, st, _, _ = run_step(b, 78, dtype=dtype, fuse=1)
    o2, _, _, _ = run_step(b, 78, dtype=dtype, fuse=0)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    check = assert_attention_close if dtype == torch.bfloat16 else assert_close_f16
    check(o1, st.oracle_attention(), "prefill-heavy fused %d/%d/%d" % (Hq, Hkv, D))


@pytest.mark.parametrize("cus,split", [(2, 64), (5, 0), (8, 128), (256, 32)])
def test_decode_workgroups_that_walk_many_pairs(cus, split):
    """Decode beside the tiles: as many decode workgroups as the chip has CUs, each walking the
    (work item, kv head) pairs j, 2W-1-j, 2W+j, ... one after the other through the same merge
    buffers.  With a chip of 2, 5 or 8 CUs every workgroup walks many rounds and the last round
    is ragged; with 256 there are fewer pairs than workgroups.  Bit-identical to two kernels in a
    row, and both meet the oracle."""
    sh = synth.Shape(12, 4, 128)
    ctx = [700, 33, 260, 1500, 15, 0, 2047, 90, 5, 311, 1023, 64, 48]
    ql = [1, 100, 1, 1, 1, 17, 1, 1, 1, 1, 1, 1, 40]
    b = synth.make_batch(sh, ctx, ql, synth.generator(79), spare=3)
    cs.cs_debug_set_cu_count(cus)
    try:
        o1, st, _, bb = run_step(b, 79, split=split, fuse=3)
        assert cs.cs_debug_mixed_arrangement(bb, sh.Hq, sh.Hkv, sh.D) in (0, 1, 2)
        o2, _, _, _ = run_step(b, 79, split=split, fuse=0)
    finally:
        cs.cs_debug_set_cu_count(0)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    assert_attention_close(o1, st.oracle_attention(), "decode beside the tiles, %d CUs, split %d" % (cus, split))


@pytest.mark.parametrize("mode,whole,ranges,backwards_tiles", [(3, 3, 2, False), (3, 5, 3, False), (2, 2, 2, False),
                                                               (3, 0, 2, False), (3, 1000, 4, False), (3, 9, 2, True)])
def test_fused_grid_with_only_its_last_tiles_cut(mode, whole, ranges, backwards_tiles):
    """In the fused grid the host may leave the first tiles of the launch order whole and cut only
    those behind them into key ranges (the last round's, which would otherwise run alone on their
    CUs).  Forced here at every kind of boundary: a cut that starts inside a chunk, after the last
    tile (nothing cut), at the first (all cut), and in a grid walked backwards (more tiles than
    workgroup slots on a small chip).  Whole tiles write their rows themselves, cut tiles through
    their partials and the merge: every row must meet the oracle, whichever way it went."""
    sh = synth.Shape(12, 4, 128)
    ctx = [700, 2300, 1500, 15, 3100, 260, 4000]
    ql = [1, 200, 1, 1, 130, 1, 96]
    b = synth.make_batch(sh, ctx, ql, synth.generator(83), spare=3)
    cs.cs_debug_set_tail_cut(whole, ranges)
    if backwards_tiles:
        cs.cs_debug_set_cu_count(2)
    try:
        out, st, _, bb = run_step(b, 83, fuse=mode)
        n_slots, first_cut, n_ranges = cs.cs_debug_mixed_tail_cut(bb, sh.Hq, sh.Hkv, sh.D)
        assert first_cut == min(whole, n_slots) and n_ranges == (ranges if whole < n_slots else 1)
    finally:
        cs.cs_debug_set_tail_cut(-1, 0)
        cs.cs_debug_set_cu_count(0)
    assert_attention_close(out, st.oracle_attention(), "tail cut: mode %d, whole %d, %d ranges" % (mode, whole, ranges))


def test_prefill_many_short_chunks():
    """More workgroup slots than one grid dimension holds (60 000 sequences: two-token chunks and
    decode tokens interleaved): the slot index rides in grid.x together with the kv head."""
    sh = synth.Shape(2, 1, 64)
    S = 60000
    ql = [2 if s % 3 else 1 for s in range(S)]
    ctx = [s % 5 for s in range(S)]
    b = synth.make_batch(sh, ctx, ql, synth.generator(36))
    out, st, _, _ = run_step(b, 36, check_append=False)
    sample = list(range(0, S, 997)) + [S - 1, S - 2]
    ref = st.oracle_attention(sample)
    assert_attention_close(out, ref, "60000 sequences")
    assert torch.isfinite(out.float()).all()


def test_page_permutation_leaves_output_bit_identical():
    sh = synth.Shape(8, 2, 128)
    ctx, ql = [100, 700, 31, 0, 260], [1, 1, 1, 48, 33]
    b1 = synth.make_batch(sh, ctx, ql, synth.generator(41), spare=5)
    b2 = synth.make_batch(sh, ctx, ql, synth.generator(42), spare=5)
    assert not torch.equal(b1.block_tables, b2.block_tables)
    o1, _, _, _ = run_step(b1, 40)
    o2, _, _, _ = run_step(b2, 40)                                   # same values, other pages
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))


def test_attention_argument_errors():
    sh = synth.Shape(4, 2, 64)
    b = decode_batch(sh, [600, 700], 50)
    pool = cs.Pool.empty(1, b.num_pages, sh.Hkv, sh.D)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    q = torch.zeros((2, 4, 64), dtype=torch.bfloat16, device="cuda")
    cs.cs_set_decode_split_tokens(256)
    try:
        with pytest.raises(cs.CsError) as e:
            cs.cs_paged_attention_mixed(pool, 0, bb, q, q.clone(), 4, 0.125, None)
        assert e.value.status in (cs.CS_ERR_WORKSPACE_TOO_SMALL, cs.CS_ERR_INVALID_ARG)
        with pytest.raises(cs.CsError) as e:
            cs.cs_paged_attention_mixed(pool, 0, bb, q, q.clone(), 3, 0.125, cs.workspace_for(bb, 4, 2, 64))
        assert e.value.status == cs.CS_ERR_INVALID_ARG                # 3 query heads over 2 kv heads
        with pytest.raises(cs.CsError) as e:
            cs.cs_paged_attention_mixed(pool, 1, bb, q, q.clone(), 4, 0.125, cs.workspace_for(bb, 4, 2, 64))
        assert e.value.status == cs.CS_ERR_INVALID_ARG                # layer out of range
    finally:
        cs.cs_set_decode_split_tokens(0)


@pytest.mark.parametrize("Hq,Hkv,D,gain", [(8, 2, 128, 1.0), (28, 4, 128, 1.0), (16, 1, 64, 1.0), (8, 2, 128, 6.0)])
def test_prefill_key_range_split(Hq, Hkv, D, gain):
    # few chunk tokens on long contexts: the tiles are cut into key ranges whose partials a
    # second kernel merges (some ranges lie wholly beyond what the earlier token blocks see)
    sh = synth.Shape(Hq, Hkv, D)
    b = synth.make_batch(sh, [3000, 1501, 0, 4100], [40, 17, 33, 1], synth.generator(61))
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    assert cs.cs_paged_attention_workspace_bytes(bb, Hq, Hkv, D) > 0
    out, st, _, _ = run_step(b, 61, q_gain=gain)
    assert_attention_close(out, st.oracle_attention(), "prefill split %d/%d/%d" % (Hq, Hkv, D))


@pytest.mark.parametrize("page_size", [16, 8])
def test_bad_page_ids_are_skipped_and_harm_no_other_sequence(page_size):
    """Block tables live on the device and are not validated by the host: an entry outside
    [0, num_pages) is skipped by every kernel (append writes nothing for it, attention reads
    nothing through it).  The rows of the sequences with bad entries are unspecified; every
    other sequence and every page they do not own must come out as if nothing were wrong."""
    sh = synth.Shape(8, 2, 128, page_size=page_size)
    ctx, ql = [300, 700, 40, 0, 513, 90], [1, 1, 40, 33, 1, 17]
    b = synth.make_batch(sh, ctx, ql, synth.generator(71), spare=2)
    st = Step(b, 71)
    cpu_pool = st.prior_pool()
    bt = b.block_tables.clone()
    bad_seqs = [1, 2, 4]
    bt[1, 3] = -1                                  # decode: a page in the middle of the context
    bt[1, int(b.blocks_needed()[1]) - 1] = b.num_pages          # ... and the page the new token goes to
    bt[2, 0] = 1 << 30                             # chunk: first context page, and a page the chunk writes
    bt[2, int(b.blocks_needed()[2]) - 1] = -7
    bt[4, :] = b.num_pages + 5                     # decode: every page
    pool = cs.Pool(from_bits(cpu_pool, "cuda"), 1, b.num_pages, sh.Hkv, sh.D, page_size=page_size)
    bb = cs.Batch(bt, b.ctx_lens, b.cu_q_lens)
    cs.cs_kv_append(pool, 0, bb, st.k_new.cuda(), st.v_new.cuda())
    torch.cuda.synchronize()
    # the oracle's append with the bad sequences' bad entries left out: append only what has a page
    want = cpu_pool.copy()
    st.oracle_append(want)
    got = bits(pool.tensor)
    owned_by_bad = set()
    for s in bad_seqs:
        owned_by_bad.update(int(x) for x in b.block_tables[s] if x >= 0)
    keep = np.array([p not in owned_by_bad for p in range(b.num_pages)])
    np.testing.assert_array_equal(got[:, keep], want[:, keep])
    for mode in (2, 0):
        cs.cs_set_mixed_fusion(mode)
        try:
            ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
            out = torch.full((b.T, sh.Hq, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
            cs.cs_paged_attention_mixed(pool, 0, bb, st.q.cuda(), out, sh.Hq, sh.scale, ws)
            torch.cuda.synchronize()
        finally:
            cs.cs_set_mixed_fusion(1)
        good = [s for s in range(b.S) if s not in bad_seqs]
        ref = st.oracle_attention(good)
        assert_attention_close(out, ref, "good sequences beside bad page ids, page size %d" % page_size)
        # a decode with no valid page at all has no key: its row is written as zeros, not 0/0
        t4 = int(b.cu_q_lens[4])
        assert (out[t4].float() == 0).all()


@pytest.mark.parametrize("cus", [64, 128, 304, 512])
def test_plans_for_other_compute_unit_counts_are_still_correct(cus):
    """The launch plans are sized by the device's compute-unit count.  Planned as if the chip had a
    quarter, half, a fifth more or twice the units it has -- other split sizes, other numbers of
    key ranges, other tile orders -- the same batches must still meet the oracle (a plan sized
    for another chip is slower on this one, never wrong)."""
    cs.cs_debug_set_cu_count(cus)
    try:
        # decode sequences that are cut, a chunk cut into key ranges, chunks whose tiles are reordered
        sh = synth.Shape(8, 2, 128)
        b = synth.make_batch(sh, [5000, 300, 2500, 3000, 0, 700], [1, 1, 1, 40, 33, 200], synth.generator(81))
        out, st, _, _ = run_step(b, 81, q_gain=3.0)
        assert_attention_close(out, st.oracle_attention(), "planned for %d CUs, mixed" % cus)
        sh = synth.Shape(32, 8, 128)
        b = synth.make_batch(sh, [900, 100, 400], [320, 256, 290], synth.generator(82))
        out, st, _, _ = run_step(b, 82, fuse=2)
        assert_attention_close(out, st.oracle_attention(), "planned for %d CUs, chunks" % cus)
    finally:
        cs.cs_debug_set_cu_count(0)
