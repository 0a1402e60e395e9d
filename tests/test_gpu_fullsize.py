"""Parity at the stated workload sizes, in the launch configuration bench.py times.

The pools are filled with seeded N(0,1) bf16 directly on the GPU (the logical K/V of a
sequence is then, by definition, what its block table points at).  The oracle cannot redo
whole batches of this size in seconds, so it recomputes SAMPLED sequences / query rows one by
one from logical K/V that the test extracts with the oracle's own format code; append,
gather and restore are compared bit for bit on sampled pages.
"""
import numpy as np
import pytest
import torch

from oracle import attention, kv_layout
from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import ABS_TOL, REL_TOL, bits

pytestmark = pytest.mark.gpu


def fill(t, gen):
    flat = t.view(-1)
    step = 1 << 27
    for o in range(0, flat.numel(), step):
        n = min(step, flat.numel() - o)
        flat[o:o + n] = torch.randn(n, generator=gen, device=t.device, dtype=torch.float32).to(torch.bfloat16)


def logical_from_pool(pool_t, layer, bt_row, n, Hkv, D, ps=16):
    """Logical K, V (float32 [n, Hkv, D]) of one sequence: pull its pages (of ps tokens) to the
    host with plain torch indexing and undo the page format with the oracle's reader."""
    nb = (n + ps - 1) // ps
    ids = bt_row[:nb].to(torch.int64)
    pages = pool_t[layer].index_select(0, ids.to(pool_t.device)).cpu()            # [nb, 2, Hkv, ps*D]
    small = bits(pages).reshape(1, nb, 2, Hkv, ps * D)
    K, V = kv_layout.read_logical(small, 0, np.arange(nb), n, page_size=ps)
    return kv_layout.bf16_bits_to_f32(K), kv_layout.bf16_bits_to_f32(V)


def run_full(index, sample_seqs, rows_per_chunk=6):
    return run_batch(synth.CONFIGS[index](), synth.BASE_SEED + index, sample_seqs, rows_per_chunk)


def run_batch(b, seed, sample_seqs, rows_per_chunk=6):
    sh = b.shape
    ps = sh.page_size
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    L_alloc = 1                                     # attention uses one layer of the pool
    pool = cs.Pool.empty(L_alloc, b.num_pages, sh.Hkv, sh.D, page_size=ps)
    fill(pool.tensor, gen)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    q = synth.randn_bf16((b.T, sh.Hq, sh.D), gen, "cuda")
    k_new = synth.randn_bf16((b.T, sh.Hkv, sh.D), gen, "cuda")
    v_new = synth.randn_bf16((b.T, sh.Hkv, sh.D), gen, "cuda")
    # snapshot the pages the sampled sequences will append into, before the append
    touched = {}
    for s in sample_seqs:
        c, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
        for blk in range(c // ps, (c + ql - 1) // ps + 1):
            pid = int(b.block_tables[s, blk])
            touched[pid] = bits(pool.tensor[0, pid].cpu()).copy()
    cs.cs_kv_append(pool, 0, bb, k_new, v_new)
    out = torch.full((b.T, sh.Hq, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
    cs.cs_paged_attention_mixed(pool, 0, bb, q, out, sh.Hq, sh.scale, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all(), "non-finite output rows"
    kn, vn = bits(k_new), bits(v_new)
    qf = q.float().cpu().numpy()
    worst_abs = worst_rel = 0.0
    for s in sample_seqs:
        c, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
        t0 = int(b.cu_q_lens[s])
        # (1) append, bit exact on every page this sequence wrote: oracle append on the snapshot
        blks = list(range(c // ps, (c + ql - 1) // ps + 1))
        small = np.stack([touched[int(b.block_tables[s, blk])] for blk in blks])[None]   # [1, nb, 2, Hkv, ps*D]
        bt_local = np.full((1, (c + ql + ps - 1) // ps), -1, np.int32)
        for j, blk in enumerate(blks):
            bt_local[0, blk] = j
        kv_layout.ref_append(small, 0, bt_local, np.array([c]), np.array([0, ql]), kn[t0:t0 + ql], vn[t0:t0 + ql],
                             page_size=ps)
        for j, blk in enumerate(blks):
            got = bits(pool.tensor[0, int(b.block_tables[s, blk])].cpu())
            np.testing.assert_array_equal(got, small[0, j], err_msg="append, seq %d block %d" % (s, blk))
        # (2) attention on sampled rows, from logical K/V read back through the block table
        K, V = logical_from_pool(pool.tensor, 0, b.block_tables[s], c + ql, sh.Hkv, sh.D, ps)
        np.testing.assert_array_equal(K[c:], kv_layout.bf16_bits_to_f32(kn[t0:t0 + ql]))
        rows = sorted(set([0, ql - 1] + list(np.random.default_rng(s).integers(0, ql, rows_per_chunk)))) if ql > 1 else [0]
        ref = attention.attention_rows(qf[[t0 + r for r in rows]], np.array([c + r for r in rows]), K, V, sh.scale)
        got = out[[t0 + r for r in rows]].float().cpu().numpy().astype(np.float64)
        err = np.abs(got - ref).max()
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        worst_abs, worst_rel = max(worst_abs, err), max(worst_rel, rel)
        assert err <= ABS_TOL and rel <= REL_TOL, "seq %d: max abs %.3e rel %.3e" % (s, err, rel)
    return worst_abs, worst_rel


def test_llama8b_decode_full_size():
    b = synth.config_llama8b_decode()
    order = np.argsort(b.ctx_lens.numpy())
    run_full(1, [int(order[0]), int(order[-1]), int(order[128]), 0, 255, 17])


def test_qwen7b_mixed_full_size():
    b = synth.config_qwen7b_mixed()
    order = np.argsort(b.ctx_lens[:64].numpy())
    run_full(2, [int(order[0]), int(order[-1]), 5, 64, 65, 66, 67])


def test_llama70b_long_full_size():
    b = synth.config_llama70b_long()
    order = np.argsort(b.ctx_lens[:128].numpy())
    run_full(3, [int(order[0]), int(order[-1]), 77, 128], rows_per_chunk=4)


def test_model_shapes_with_pages_of_8_tokens():
    """The three attention workloads at their stated sizes on pools of 8-token pages."""
    b = synth.config_llama8b_decode(page_size=8)
    order = np.argsort(b.ctx_lens.numpy())
    run_batch(b, synth.BASE_SEED + 11, [int(order[0]), int(order[-1]), 0, 255])
    b = synth.config_qwen7b_mixed(page_size=8)
    order = np.argsort(b.ctx_lens[:64].numpy())
    run_batch(b, synth.BASE_SEED + 12, [int(order[0]), int(order[-1]), 64, 65, 66, 67])
    b = synth.config_llama70b_long(page_size=8)
    order = np.argsort(b.ctx_lens[:128].numpy())
    run_batch(b, synth.BASE_SEED + 13, [int(order[-1]), 77, 128], rows_per_chunk=4)


def test_very_long_contexts():
    """Contexts far beyond the workloads': a decode over 150 001 keys, one over 70 002, and a
    chunk of 48 tokens on 90 000 (few tiles on a very long context: key ranges and their
    merge).  Once with the automatic plan (two sequences alone are cut until every CU has a
    workgroup: some hundred pieces each, still listed in the kernel arguments) and once cut at
    256 keys: more pieces than an item word can say, so the planning kernel lists them."""
    sh = synth.Shape(4, 2, 64)
    b = synth.make_batch(sh, [150000, 70001, 90000], [1, 1, 48], synth.generator(90))
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    items, n_items, split = cs.cs_debug_decode_items(bb, sh.Hkv, sh.D)
    assert items is not None and 128 <= n_items <= 510 and n_items * sh.Hkv >= 256
    assert cs.cs_paged_attention_workspace_bytes(bb, sh.Hq, sh.Hkv, sh.D) > 0
    run_batch(b, 90, [0, 1, 2], rows_per_chunk=5)
    cs.cs_set_decode_split_tokens(256)
    try:
        items, n_items, split = cs.cs_debug_decode_items(bb, sh.Hkv, sh.D)
        assert items is None and n_items > 255 and split == 256      # listed on the device
        run_batch(b, 90, [0, 1, 2], rows_per_chunk=5)
    finally:
        cs.cs_set_decode_split_tokens(0)


@pytest.mark.parametrize("Hq,Hkv,ctx,ql", [
    (32, 8, [8192], [1024]),                 # 256 tile workgroups: cut in two, one full round of pairs
    (28, 4, [16384], [1280]),                # 280: cut in three, two rounds
    (32, 8, [12000, 17000], [1280, 1280]),   # 640 over two sequences of different length
    (64, 8, [33000], [1536]),                # 768: cut in two
    (32, 8, [100, 30000, 500, 60000], [512] * 4),   # 512 of very unequal length: only the long tiles are cut
])
def test_chunks_between_one_and_four_workgroups_per_cu_are_cut_into_key_ranges(Hq, Hkv, ctx, ql):
    """A grid of 256..1024 tile workgroups runs as one or two rounds over the workgroup slots;
    on long contexts the host cuts the tiles into key ranges so that the rounds come out full.
    Full-size parity of exactly those plans (the plan must really cut), plus two decode
    sequences riding along."""
    sh = synth.Shape(Hq, Hkv, 128)
    b = synth.make_batch(sh, [700, 3000] + ctx, [1, 1] + ql, synth.generator(91))
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    only_chunks = cs.Batch(b.block_tables[2:], b.ctx_lens[2:], b.cu_q_lens[2:] - 2)
    assert cs.cs_paged_attention_workspace_bytes(only_chunks, sh.Hq, sh.Hkv, sh.D) > 0    # partials: the tiles are cut
    run_batch(b, 91, list(range(len(ctx) + 2)), rows_per_chunk=4)


@pytest.mark.parametrize("Hq,Hkv,ctx,ql,n_dec", [
    (40, 8, [2048, 1000, 3000, 500], [320] * 4, 0),   # 416 tile workgroups of four lengths: solo + pairs
    (32, 8, [6000], [1536], 0),                       # 384: one chunk, causal lengths
    (28, 4, [200, 800, 1400, 2000], [448] * 4, 0),    # 392, four kv heads
    (32, 8, [0], [4096], 0),                          # 1024: more tiles than slots, longest first
    (32, 8, [0, 3000], [3072, 1024], 9),              # 1024 beside nine decodes: the fused grid walks the tiles backwards
])
def test_prefill_grids_dealt_to_cus_by_tile_length(Hq, Hkv, ctx, ql, n_dec):
    """The host orders uncut tiles for the dispatcher: between one and two tile workgroups per
    CU the longest get a CU of their own and the rest are paired long with short; with more tiles
    than workgroup slots the longest go first.  The plan must really be a permutation of the
    tiles, and every chunk must still meet the oracle."""
    sh = synth.Shape(Hq, Hkv, 128)
    b = synth.make_batch(sh, [900] * n_dec + ctx, [1] * n_dec + ql, synth.generator(93))
    only_chunks = cs.Batch(b.block_tables[n_dec:], b.ctx_lens[n_dec:], b.cu_q_lens[n_dec:] - n_dec)
    import ctypes
    buf = (ctypes.c_int32 * 512)()
    n = cs.lib().cs_debug_prefill_order(ctypes.byref(only_chunks.c), sh.Hq, sh.Hkv, sh.D, buf, 512)
    assert n > 256 // Hkv and len(set(buf[:n])) == n
    cs.cs_set_mixed_fusion(2)
    try:
        run_batch(b, 93, list(range(n_dec + len(ctx))), rows_per_chunk=6)
    finally:
        cs.cs_set_mixed_fusion(1)


@pytest.mark.parametrize("seed", range(16))
def test_random_batches_at_model_shapes(seed):
    """Seeded random mixes at the four model shapes and at sizes where the launch planning
    matters (chunks of up to 2048 tokens on contexts of up to 40 000 keys, decodes of up to
    20 000): whatever the host decides -- work items, prefetch depth, key ranges, fused grid or
    not -- sampled rows must meet the oracle and the appended pages be exact."""
    import random
    rnd = random.Random(9000 + seed)
    Hq, Hkv = rnd.choice([(32, 8), (28, 4), (64, 8), (40, 8)])
    sh = synth.Shape(Hq, Hkv, 128)
    n_dec = rnd.choice([0, 0, 3, 17, 70])
    n_ch = rnd.choice([1, 1, 2, 4, 7])
    ctx = [rnd.choice([rnd.randint(0, 3000), rnd.randint(0, 20000)]) for _ in range(n_dec)]
    ql = [1] * n_dec
    for _ in range(n_ch):
        ctx.append(rnd.choice([0, rnd.randint(0, 4000), rnd.randint(0, 40000)]))
        ql.append(rnd.choice([rnd.randint(2, 400), rnd.randint(200, 1500), rnd.choice([256, 512, 1024, 1280, 2048])]))
    order = list(range(len(ctx)))
    rnd.shuffle(order)
    ctx, ql = [ctx[i] for i in order], [ql[i] for i in order]
    mode, ahead = rnd.choice([1, 1, 2, 0]), rnd.choice([0, 0, 1, 2])
    cs.cs_set_mixed_fusion(mode)
    cs.cs_set_decode_pages_ahead(ahead)
    try:
        b = synth.make_batch(sh, ctx, ql, synth.generator(9500 + seed))
        sample = list(range(len(ctx))) if len(ctx) <= 8 else rnd.sample(range(len(ctx)), 8)
        run_batch(b, 9500 + seed, sample, rows_per_chunk=3)
    finally:
        cs.cs_set_mixed_fusion(1)
        cs.cs_set_decode_pages_ahead(0)


def test_qwen14b_ckpt_full_size():
    """Workload 4 at its stated page counts on a subset of layers: gather all dirty pages of 3
    of the 48 layers (the kernels index layers independently), restore into the spare pages,
    rewrite the block tables, and run the mixed attention pass over the restored requests."""
    b = synth.config_qwen14b_ckpt()
    sh = b.shape
    L = 3
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 4)
    pool = cs.Pool.empty(L, b.num_pages, sh.Hkv, sh.D)
    fill(pool.tensor, gen)
    dirty = b.extra["dirty_pages"]
    fresh = [int(x) for x in b.spare_pages[:len(dirty)]]
    d_ids = torch.tensor(dirty, dtype=torch.int32, device="cuda")
    f_ids = torch.tensor(fresh, dtype=torch.int32, device="cuda")
    staging = torch.empty((L, len(dirty), sh.page_elems), dtype=torch.bfloat16, device="cuda")
    before = pool.tensor[:, dirty].cpu()
    cs.cs_kv_ckpt_gather(pool, 0, L, d_ids, staging)
    torch.cuda.synchronize()
    # gather: bit exact against the oracle on sampled layers/pages (and all pages via torch equality)
    sample = [0, 1, len(dirty) // 2, len(dirty) - 1]
    small_pool = bits(before[:, sample]).reshape(L, len(sample), 2, sh.Hkv, 16 * sh.D)
    want = kv_layout.ref_gather(small_pool, 0, L, list(range(len(sample))))
    np.testing.assert_array_equal(bits(staging[:, sample].cpu()), want)
    assert torch.equal(staging.cpu().view(torch.int16), before.reshape(L, len(dirty), -1).view(torch.int16))
    # preempt: the old pages are given away; resume into fresh pages
    pool.tensor[:, dirty] = float("nan")
    cs.cs_kv_ckpt_restore(pool, 0, L, f_ids, staging)
    torch.cuda.synchronize()
    assert torch.equal(pool.tensor[:, fresh].cpu().view(torch.int16), before.view(torch.int16))
    remap = torch.arange(b.num_pages, dtype=torch.int32)
    remap[torch.tensor(dirty, dtype=torch.int64)] = torch.tensor(fresh, dtype=torch.int32)
    bt2 = b.block_tables.clone()
    bt2[bt2 >= 0] = remap[bt2[bt2 >= 0].to(torch.int64)]
    # attention over the restored requests (layer 1), sampled sequences checked by the oracle
    n_act = b.extra["n_active"]
    bb = cs.Batch(bt2[:n_act], b.ctx_lens[:n_act], b.cu_q_lens[:n_act + 1])
    q = synth.randn_bf16((b.T, sh.Hq, sh.D), gen, "cuda")
    k_new = synth.randn_bf16((b.T, sh.Hkv, sh.D), gen, "cuda")
    v_new = synth.randn_bf16((b.T, sh.Hkv, sh.D), gen, "cuda")
    cs.cs_kv_append(pool, 1, bb, k_new, v_new)
    out = torch.full((b.T, sh.Hq, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    cs.cs_paged_attention_mixed(pool, 1, bb, q, out, sh.Hq, sh.scale, cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D))
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    qf = q.float().cpu().numpy()
    for s in (0, 63, 64, 67):
        c, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
        t0 = int(b.cu_q_lens[s])
        K, V = logical_from_pool(pool.tensor, 1, bt2[s], c + ql, sh.Hkv, sh.D)
        rows = [0, ql - 1] if ql > 1 else [0]
        ref = attention.attention_rows(qf[[t0 + r for r in rows]], np.array([c + r for r in rows]), K, V, sh.scale)
        got = out[[t0 + r for r in rows]].float().cpu().numpy().astype(np.float64)
        assert np.abs(got - ref).max() <= ABS_TOL
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= REL_TOL
