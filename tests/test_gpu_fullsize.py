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
from helpers import (ABS_TOL, PROBE_GAIN, REL_TOL, assert_rows_close, bits, chunk_probe_targets, from_bits,
                     probe_tokens, probe_vectors)

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


def run_full(index, sample_seqs, rows_per_chunk=6, **kw):
    return run_batch(synth.CONFIGS[index](), synth.BASE_SEED + index, sample_seqs, rows_per_chunk, **kw)


def plant_probes(pool, layer, b, s, k_new, seed, max_pages=None):
    """Plant one key per page of sequence s (see helpers: probe data).  Context pages are pulled
    to the host, written with the ORACLE's append and pushed back; pages the step itself fills
    get their key through k_new (the library's append then stores it).  max_pages: probe only
    that many pages, evenly strided from a seeded offset (for sequences whose every page would
    cost the oracle too long).  Returns (pages probed, their planted tokens, their u vectors)."""
    sh = b.shape
    ps = sh.page_size
    C, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
    n = C + ql
    tokens = probe_tokens(seed, n, ps)
    pages = np.arange(len(tokens))
    if max_pages is not None and len(pages) > max_pages:
        stride = -(-len(pages) // max_pages)
        pages = pages[(seed % stride)::stride]
        if pages[-1] != len(tokens) - 1:
            pages = np.append(pages, len(tokens) - 1)          # always the last page
    tokens = tokens[pages]
    u = probe_vectors(seed, len(pages), sh.D)
    planted = (u.float() * PROBE_GAIN).to(torch.bfloat16)       # exact: a power-of-two gain
    in_ctx = tokens < C
    if in_ctx.any():
        ids = b.block_tables[s, torch.from_numpy(pages[in_ctx])].to(torch.int64)
        small = bits(pool.tensor[layer].index_select(0, ids.to(pool.tensor.device)).cpu()).reshape(1, len(ids), 2, sh.Hkv, ps * sh.D).copy()
        m = int(in_ctx.sum())
        rows = bits(planted[torch.from_numpy(in_ctx)])[:, None, :].repeat(sh.Hkv, axis=1)        # [m, Hkv, D]
        # pseudo-sequence i: one token at slot tokens[i] % ps of local page i; V keeps its bits
        _, V = kv_layout.read_logical(small, 0, np.arange(m), m * ps, page_size=ps)
        slots = np.arange(m) * ps + tokens[in_ctx] % ps
        kv_layout.ref_append(small, 0, np.arange(m, dtype=np.int32)[:, None], (tokens[in_ctx] % ps).astype(np.int32),
                             np.arange(m + 1, dtype=np.int32), rows, V[slots], page_size=ps)
        pool.tensor[layer].index_copy_(0, ids.to(pool.tensor.device),
                                       from_bits(small[0], pool.tensor.device).view(len(ids), 2, sh.Hkv, ps * sh.D))
    t0 = int(b.cu_q_lens[s])
    for i in np.nonzero(~in_ctx)[0]:
        k_new[t0 + int(tokens[i]) - C] = planted[i].to(k_new.device)[None, :].expand(sh.Hkv, -1)
    return pages, tokens, u


def run_probes(b, pool, bb, ws, q, k_new, v_new, out, seed, probe_seqs, max_pages=None):
    """Every page (or max_pages of them) of the sequences in probe_seqs gets a planted key and a
    (query row, head) aimed at it; the outputs of those (row, head) pairs must meet the oracle,
    evaluated on the logical K/V read back through the block table.  Decode sequences need
    ceil(pages / Hq) attention calls, chunks one."""
    sh = b.shape
    ps = sh.page_size
    plan = {}
    for s in probe_seqs:
        plan[s] = plant_probes(pool, 0, b, s, k_new, seed * 1000 + s, max_pages)
    cs.cs_kv_append(pool, 0, bb, k_new, v_new)
    n_calls = 1
    for s in probe_seqs:
        if int(b.q_lens[s]) == 1:
            n_calls = max(n_calls, -(-len(plan[s][0]) // sh.Hq))
    logical, targets = {}, {}
    for s in probe_seqs:
        C, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
        logical[s] = logical_from_pool(pool.tensor, 0, b.block_tables[s], C + ql, sh.Hkv, sh.D, ps)
        if ql > 1:
            targets[s] = chunk_probe_targets(C, ql, sh.Hq, plan[s][1])
    worst = [0.0, 0.0, 0]
    probed = 0
    for call in range(n_calls):
        qc = q.clone()
        for s in probe_seqs:
            t0, ql = int(b.cu_q_lens[s]), int(b.q_lens[s])
            pages, tokens, u = plan[s]
            if ql == 1:
                sel = np.arange(call * sh.Hq, min(len(pages), (call + 1) * sh.Hq))
                if len(sel):
                    qc[t0, :len(sel)] = u[torch.from_numpy(sel)].to(qc.device)
            elif call == 0:
                rows, heads = targets[s]
                ok = rows >= 0
                qc[torch.from_numpy(t0 + rows[ok]).to(qc.device), torch.from_numpy(heads[ok]).to(qc.device)] = \
                    u[torch.from_numpy(ok)].to(qc.device)
        out.fill_(float("nan"))
        cs.cs_paged_attention_mixed(pool, 0, bb, qc, out, sh.Hq, sh.scale, ws)
        torch.cuda.synchronize()
        qf = qc.float().cpu().numpy()
        of = out.float().cpu().numpy().astype(np.float64)
        for s in probe_seqs:
            C, t0, ql = int(b.ctx_lens[s]), int(b.cu_q_lens[s]), int(b.q_lens[s])
            K, V = logical[s]
            pages, tokens, u = plan[s]
            if ql == 1:
                n_here = min(len(pages), (call + 1) * sh.Hq) - call * sh.Hq
                if n_here <= 0:
                    continue
                ref = attention.attention_rows(qf[t0:t0 + 1], np.array([C]), K, V, sh.scale)[0, :n_here]
                got = of[t0, :n_here]
                # the aimed head's output is (nearly) the V row of the planted token, read through
                # the oracle's format code: the probe really looks at its page
                sel = np.arange(call * sh.Hq, call * sh.Hq + n_here)
                G = sh.Hq // sh.Hkv
                vrow = np.stack([V[tokens[i], (i - call * sh.Hq) // G] for i in sel])
                assert np.abs(ref - vrow).max() < 1e-2, "seq %d: a decode probe does not dominate its row" % s
                r = assert_rows_close(got, ref, "probes of decode seq %d, call %d (pages %d..%d)" % (s, call, pages[sel[0]], pages[sel[-1]]))
                probed += n_here
            elif call == 0:
                rows, heads = targets[s]
                ok = np.nonzero(rows >= 0)[0]
                G = sh.Hq // sh.Hkv
                got = np.empty((len(ok), sh.D))
                ref = np.empty((len(ok), sh.D))
                for h in range(sh.Hq):                         # one oracle call per head: its kv head only
                    mine = ok[heads[ok] == h]
                    if not len(mine):
                        continue
                    g = h // G
                    r_h = attention.attention_rows(qf[t0 + rows[mine]][:, h:h + 1], (C + rows[mine]).astype(np.int32),
                                                   K[:, g:g + 1], V[:, g:g + 1], sh.scale)[:, 0]
                    where = np.searchsorted(ok, mine)
                    ref[where] = r_h
                    got[where] = of[t0 + rows[mine], h]
                r = assert_rows_close(got, ref, "probes of chunk seq %d (%d pages)" % (s, len(ok)))
                probed += len(ok)
            else:
                continue
            worst = [max(worst[0], r[0]), max(worst[1], r[1]), worst[2] + r[2]]
    print("  probes: %d pages of %d sequences over %d calls, worst abs %.2e rel %.2e, %d elements outside the mixed bound"
          % (probed, len(probe_seqs), n_calls, worst[0], worst[1], worst[2]))
    return probed


def run_batch(b, seed, sample_seqs, rows_per_chunk=6, q_gain=1.0, probe_seqs=None, max_probe_pages=None):
    """q_gain: the queries are scaled (a peaked softmax: a few keys carry each row).
    probe_seqs: after the sampled-row check, these sequences get a planted key in every page and
    aimed queries (run_probes), so that no page of theirs can go missing unseen."""
    sh = b.shape
    ps = sh.page_size
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    L_alloc = 1                                     # attention uses one layer of the pool
    pool = cs.Pool.empty(L_alloc, b.num_pages, sh.Hkv, sh.D, page_size=ps)
    fill(pool.tensor, gen)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    q = synth.randn_bf16((b.T, sh.Hq, sh.D), gen, "cuda")
    if q_gain != 1.0:
        q = (q.float() * q_gain).to(torch.bfloat16)
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
    n_outside = 0
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
        err, rel, nfail = assert_rows_close(got, ref, "seq %d (q_gain %g)" % (s, q_gain))
        worst_abs, worst_rel, n_outside = max(worst_abs, err), max(worst_rel, rel), n_outside + nfail
    print("  sampled rows of %d sequences (q_gain %g): worst abs %.2e rel %.2e, %d elements outside the mixed bound"
          % (len(sample_seqs), q_gain, worst_abs, worst_rel, n_outside))
    if probe_seqs:
        run_probes(b, pool, bb, ws, q, k_new, v_new, out, seed, probe_seqs, max_probe_pages)
    return worst_abs, worst_rel


def test_llama8b_decode_full_size():
    """Stated size; sampled rows on the N(0,1) data, then every page of six sequences probed."""
    b = synth.config_llama8b_decode()
    order = np.argsort(b.ctx_lens.numpy())
    sample = [int(order[0]), int(order[-1]), int(order[128]), 0, 255, 17]
    run_full(1, sample, probe_seqs=sample)


def test_qwen7b_mixed_full_size():
    """Stated size; every page of the shortest and the longest decode and of the chunks on the
    longest and the shortest context probed."""
    b = synth.config_qwen7b_mixed()
    order = np.argsort(b.ctx_lens[:64].numpy())
    chunks = sorted(range(64, 68), key=lambda s: int(b.ctx_lens[s]))
    run_full(2, [int(order[0]), int(order[-1]), 5, 64, 65, 66, 67],
             probe_seqs=[int(order[0]), int(order[-1]), chunks[0], chunks[-1]])


def test_llama70b_long_full_size():
    """Stated size; every page of the longest decode (about 2048 pages, 32 calls), of a middle
    one and of the 1024-token chunk on 30720 keys probed."""
    b = synth.config_llama70b_long()
    order = np.argsort(b.ctx_lens[:128].numpy())
    run_full(3, [int(order[0]), int(order[-1]), 77, 128], rows_per_chunk=4,
             probe_seqs=[int(order[-1]), int(order[64]), 128])


@pytest.mark.parametrize("index,gain", [(1, 5.0), (2, 4.0), (3, 6.0)])
def test_stated_sizes_with_a_peaked_softmax(index, gain):
    """The three attention workloads at their stated sizes with the queries scaled: each row's
    weight sits on a handful of keys somewhere in its context, so a key that is masked, read
    from the wrong page or counted twice moves the output by O(1) instead of O(1/n)."""
    b = synth.CONFIGS[index]()
    n_on = b.extra["n_online"]
    order = np.argsort(b.ctx_lens[:n_on].numpy())
    sample = [int(order[0]), int(order[-1]), int(order[n_on // 2])] + list(range(n_on, b.S))
    run_batch(b, synth.BASE_SEED + 20 + index, sample, rows_per_chunk=4, q_gain=gain)


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
    # probes: 1024 pages of each sequence, evenly strided (every page would cost the oracle minutes)
    run_batch(b, 90, [0, 1, 2], rows_per_chunk=5, probe_seqs=[0, 1, 2], max_probe_pages=1024)
    run_batch(b, 92, [0, 1, 2], rows_per_chunk=3, q_gain=5.0)
    cs.cs_set_decode_split_tokens(256)
    try:
        items, n_items, split = cs.cs_debug_decode_items(bb, sh.Hkv, sh.D)
        assert items is None and n_items > 255 and split == 256      # listed on the device
        run_batch(b, 90, [0, 1, 2], rows_per_chunk=5, probe_seqs=[0, 1], max_probe_pages=1024)
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
    # every page of the longest chunk probed (a key range that starts or ends a page off shows), and
    # the whole batch once more with a peaked softmax
    longest = 2 + int(np.argmax(ctx))
    run_batch(b, 91, list(range(len(ctx) + 2)), rows_per_chunk=4, probe_seqs=[1, longest], max_probe_pages=2048)
    run_batch(b, 95, list(range(len(ctx) + 2)), rows_per_chunk=3, q_gain=4.0)


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
    if rnd.choice([0, 1, 2]) == 0:
        mode = 3
    cs.cs_set_mixed_fusion(mode)
    cs.cs_set_decode_pages_ahead(ahead)
    try:
        b = synth.make_batch(sh, ctx, ql, synth.generator(9500 + seed))
        sample = list(range(len(ctx))) if len(ctx) <= 8 else rnd.sample(range(len(ctx)), 8)
        # probes on the longest decode and the longest chunk (512 pages each at most), and a second
        # pass over other data with a peaked softmax
        dec = [s for s in range(len(ctx)) if ql[s] == 1]
        chk = [s for s in range(len(ctx)) if ql[s] > 1]
        probe = [max(dec, key=lambda s: ctx[s])] if dec else []
        probe.append(max(chk, key=lambda s: ctx[s] + ql[s]))
        run_batch(b, 9500 + seed, sample, rows_per_chunk=3, probe_seqs=probe, max_probe_pages=512)
        run_batch(b, 9700 + seed, sample[:4], rows_per_chunk=2, q_gain=rnd.choice([4.0, 6.0]))
    finally:
        cs.cs_set_mixed_fusion(1)
        cs.cs_set_decode_pages_ahead(0)


def test_qwen14b_ckpt_full_size():
    """Workload 4 at its stated size: the 48-layer pool (about 72 GB), all dirty pages of all 48
    layers gathered in one call (7.25 GB), the old pages given away, everything restored into the
    spare pages, the block tables rewritten, and the mixed attention pass run on the LAST layer,
    whose pages lie some 70 GB into the pool.  Gather and restore are compared with the pool on
    the device for every layer and page, and bit for bit with the oracle's copies on sampled
    (layer, page) pairs pulled to the host before the call (layers 0, 23 and 47 among them)."""
    b = synth.config_qwen14b_ckpt()
    sh = b.shape
    L = sh.L
    assert L == 48
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + 4)
    pool = cs.Pool.empty(L, b.num_pages, sh.Hkv, sh.D)
    assert pool.tensor.numel() * 2 > 60e9
    fill(pool.tensor, gen)
    dirty = b.extra["dirty_pages"]
    fresh = [int(x) for x in b.spare_pages[:len(dirty)]]
    d_ids = torch.tensor(dirty, dtype=torch.int32, device="cuda")
    f_ids = torch.tensor(fresh, dtype=torch.int32, device="cuda")
    d64, f64 = d_ids.to(torch.int64), f_ids.to(torch.int64)
    staging = torch.full((L, len(dirty), sh.page_elems), float("nan"), dtype=torch.bfloat16, device="cuda")
    assert staging.numel() * 2 > 7e9
    # sampled (layer, position in the dirty list) pairs, pulled with plain torch indexing before the call
    layers = [0, 1, 23, 46, 47]
    picks = [0, 1, len(dirty) // 2, len(dirty) - 1]
    before = {l: bits(pool.tensor[l].index_select(0, d64[picks]).cpu()).reshape(1, len(picks), 2, sh.Hkv, 16 * sh.D).copy()
              for l in layers}
    cs.cs_kv_ckpt_gather(pool, 0, L, d_ids, staging)
    torch.cuda.synchronize()
    for l in layers:
        want = kv_layout.ref_gather(before[l], 0, 1, list(range(len(picks))))
        np.testing.assert_array_equal(bits(staging[l, picks].cpu())[None], want, err_msg="gather, layer %d" % l)
    for l in range(L):                                           # every layer and page, on the device
        assert torch.equal(staging[l].view(torch.int16), pool.tensor[l].index_select(0, d64).view(len(dirty), -1).view(torch.int16)), \
            "gather differs from the pool in layer %d" % l
    # preempt: the old pages are given away; resume into fresh pages
    for l in range(L):
        pool.tensor[l].index_fill_(0, d64, float("nan"))
    keep_other = {l: bits(pool.tensor[l, :4].cpu()).copy() for l in (0, 47)}     # pages 0..3 are someone's: must not move
    cs.cs_kv_ckpt_restore(pool, 0, L, f_ids, staging)
    torch.cuda.synchronize()
    for l in range(L):
        assert torch.equal(pool.tensor[l].index_select(0, f64).view(len(dirty), -1).view(torch.int16), staging[l].view(torch.int16)), \
            "restore differs from the staging buffer in layer %d" % l
        assert torch.isnan(pool.tensor[l].index_select(0, d64[:64]).float()).all(), "restore wrote into an old page, layer %d" % l
    untouched = [p for p in range(4) if p not in set(fresh) and p not in set(dirty)]
    for l in (0, 47):
        np.testing.assert_array_equal(bits(pool.tensor[l, untouched].cpu()), keep_other[l][untouched])
        # the oracle's restore of the sampled pages into a small pool of their own
        small = kv_layout.new_pool(1, len(picks), sh.Hkv, sh.D)
        kv_layout.ref_restore(small, 0, 1, list(range(len(picks))), kv_layout.ref_gather(before[l], 0, 1, list(range(len(picks)))))
        np.testing.assert_array_equal(bits(pool.tensor[l].index_select(0, f64[picks]).cpu()).reshape(small.shape), small,
                                      err_msg="restore, layer %d" % l)
    remap = torch.arange(b.num_pages, dtype=torch.int32)
    remap[torch.tensor(dirty, dtype=torch.int64)] = torch.tensor(fresh, dtype=torch.int32)
    bt2 = b.block_tables.clone()
    bt2[bt2 >= 0] = remap[bt2[bt2 >= 0].to(torch.int64)]
    # attention over the restored requests on the last layer, sampled sequences checked by the oracle
    last = L - 1
    n_act = b.extra["n_active"]
    bb = cs.Batch(bt2[:n_act], b.ctx_lens[:n_act], b.cu_q_lens[:n_act + 1])
    q = synth.randn_bf16((b.T, sh.Hq, sh.D), gen, "cuda")
    k_new = synth.randn_bf16((b.T, sh.Hkv, sh.D), gen, "cuda")
    v_new = synth.randn_bf16((b.T, sh.Hkv, sh.D), gen, "cuda")
    page_of_new = int(bt2[0, int(b.ctx_lens[0]) // 16])
    page_before = bits(pool.tensor[last, page_of_new].cpu()).copy()[None, None]
    cs.cs_kv_append(pool, last, bb, k_new, v_new)
    out = torch.full((b.T, sh.Hq, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    cs.cs_paged_attention_mixed(pool, last, bb, q, out, sh.Hq, sh.scale, cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D))
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    # the append on the last layer, bit for bit on the page sequence 0 writes into
    kv_layout.ref_append(page_before, 0, np.zeros((1, int(b.ctx_lens[0]) // 16 + 1), np.int32), np.array([int(b.ctx_lens[0])]),
                         np.array([0, 1]), bits(k_new[:1]), bits(v_new[:1]))
    np.testing.assert_array_equal(bits(pool.tensor[last, page_of_new].cpu()), page_before[0, 0])
    qf = q.float().cpu().numpy()
    for s in (0, 63, 64, 67):
        c, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
        t0 = int(b.cu_q_lens[s])
        K, V = logical_from_pool(pool.tensor, last, bt2[s], c + ql, sh.Hkv, sh.D)
        rows = [0, ql // 2, ql - 1] if ql > 1 else [0]
        ref = attention.attention_rows(qf[[t0 + r for r in rows]], np.array([c + r for r in rows]), K, V, sh.scale)
        got = out[[t0 + r for r in rows]].float().cpu().numpy().astype(np.float64)
        assert_rows_close(got, ref, "layer %d, seq %d" % (last, s))
