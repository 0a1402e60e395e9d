"""The checkpointing flow of the paper end to end (Sec. 4.4, Sec. 5): while requests decode,
every page that fills up is copied to host memory on a side stream (incremental
checkpointing, the GPU-page -> host-slot map kept by the caller); on preemption a request's
pages are simply dropped -- its full pages are already on the host, only the tokens of its
unfinished last page still have to be saved (token-granular gather); on resume everything is
brought back into fresh pages.  The resumed request must decode exactly as if nothing had
happened."""
import numpy as np
import pytest
import torch

from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import assert_attention_close, bits
from oracle import attention

pytestmark = pytest.mark.gpu

L, STEPS, VICTIM = 2, 21, 2


def test_incremental_checkpoint_preempt_resume():
    sh = synth.Shape(8, 2, 128, L=L)
    ctx0 = [5, 30, 47, 100]
    S = len(ctx0)
    final = [c + STEPS + 1 for c in ctx0]
    b = synth.make_batch(sh, final, [0] * S, synth.generator(80), spare=16)     # block tables sized for the whole run
    bt = b.block_tables.clone()
    spare = [int(p) for p in b.spare_pages]
    g = synth.generator(81)
    # logical data: prior context, then one new token per step and sequence, per layer
    prior = [[(synth.randn_bf16((c, sh.Hkv, sh.D), g), synth.randn_bf16((c, sh.Hkv, sh.D), g)) for c in ctx0] for _ in range(L)]
    new_k = synth.randn_bf16((STEPS + 1, L, S, sh.Hkv, sh.D), g)
    new_v = synth.randn_bf16((STEPS + 1, L, S, sh.Hkv, sh.D), g)
    q_last = synth.randn_bf16((L, S, sh.Hq, sh.D), g)

    def build_pool():
        pool = cs.Pool.empty(L, b.num_pages, sh.Hkv, sh.D)
        pool.tensor.view(torch.int16).fill_(0x7FC0)
        cu = torch.zeros(S + 1, dtype=torch.int32)
        cu[1:] = torch.cumsum(torch.tensor(ctx0, dtype=torch.int32), 0)
        bb0 = cs.Batch(bt, torch.zeros(S, dtype=torch.int32), cu)
        for l in range(L):
            cs.cs_kv_append(pool, l, bb0, torch.cat([p[0] for p in prior[l]]).cuda(), torch.cat([p[1] for p in prior[l]]).cuda())
        return pool

    def decode_step(pool, tables, step, out=None, q=None):
        ctx = torch.tensor([c + step for c in ctx0], dtype=torch.int32)
        bb = cs.Batch(tables, ctx, torch.arange(S + 1, dtype=torch.int32))
        for l in range(L):
            cs.cs_kv_append(pool, l, bb, new_k[step, l].cuda(), new_v[step, l].cuda())
            if out is not None:
                cs.cs_paged_attention_mixed(pool, l, bb, q[l].cuda(), out[l], sh.Hq, sh.scale, cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D))
        return ctx

    # ---- reference: an uninterrupted run
    ref_pool = build_pool()
    for step in range(STEPS):
        decode_step(ref_pool, bt, step)
    ref_out = torch.full((L, S, sh.Hq, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    decode_step(ref_pool, bt, STEPS, ref_out, q_last)
    torch.cuda.synchronize()

    # ---- the run with incremental checkpointing
    pool = build_pool()
    side = torch.cuda.Stream()
    cap = 64
    host = torch.empty((L, cap, sh.page_elems), dtype=torch.bfloat16).pin_memory()
    host_slot = {}                                     # GPU page id -> slot of `host` (the page-table extension of Sec. 5)
    def checkpoint(pages):
        """Gather the given pages and copy them to the host on the side stream; remember where."""
        if not pages:
            return
        side.wait_stream(torch.cuda.current_stream())  # the pages were filled on the compute stream
        n, base = len(pages), len(host_slot)
        ids = torch.tensor(pages, dtype=torch.int32, device="cuda")
        staging = torch.empty((L, n, sh.page_elems), dtype=torch.bfloat16, device="cuda")
        tmp = torch.empty((L, n, sh.page_elems), dtype=torch.bfloat16).pin_memory()
        cs.cs_kv_ckpt_save(pool, 0, L, ids, staging, tmp, stream=side)
        side.synchronize()
        host[:, base:base + n] = tmp
        for i, p in enumerate(pages):
            host_slot[p] = base + i

    # pages already full before the first step are checkpointed up front
    checkpoint([int(bt[s, blk]) for s in range(S) for blk in range(ctx0[s] // 16)])
    for step in range(STEPS):
        ctx = decode_step(pool, bt, step)
        filled = [int(bt[s, int(ctx[s]) // 16]) for s in range(S) if int(ctx[s]) % 16 == 15]
        checkpoint(filled)                             # only the pages this step completed
    n_tok = ctx0[VICTIM] + STEPS                        # tokens the victim holds now
    full, tail = n_tok // 16, n_tok % 16
    victim_pages = [int(bt[VICTIM, blk]) for blk in range((n_tok + 15) // 16)]
    assert all(p in host_slot for p in victim_pages[:full])           # every full page is already on the host
    assert tail > 0 and victim_pages[full] not in host_slot           # the unfinished page is not
    # ---- preemption: save the tail tokens (token-granular), drop the pages
    slots = torch.tensor([victim_pages[full] * 16 + t for t in range(tail)], dtype=torch.int32, device="cuda")
    tail_buf = torch.empty((L, tail, 2, sh.Hkv, sh.D), dtype=torch.bfloat16, device="cuda")
    cs.cs_kv_ckpt_gather_tokens(pool, 0, L, slots, tail_buf)
    tail_host = tail_buf.cpu()
    np.testing.assert_array_equal(bits(tail_host[:, -1, 0]), bits(new_k[STEPS - 1, :, VICTIM]))     # the newest token's K rows
    pool.tensor[:, victim_pages] = float("nan")                      # released
    # ---- resume into fresh pages
    fresh = spare[:len(victim_pages)]
    tables = bt.clone()
    tables[VICTIM, :len(fresh)] = torch.tensor(fresh, dtype=torch.int32)
    back = torch.stack([host[:, host_slot[p]] for p in victim_pages[:full]], dim=1).contiguous().pin_memory()
    stage2 = torch.empty((L, full, sh.page_elems), dtype=torch.bfloat16, device="cuda")
    side.wait_stream(torch.cuda.current_stream())
    cs.cs_kv_ckpt_load(pool, 0, L, torch.tensor(fresh[:full], dtype=torch.int32, device="cuda"), stage2, back, stream=side)
    side.synchronize()
    new_slots = torch.tensor([fresh[full] * 16 + t for t in range(tail)], dtype=torch.int32, device="cuda")
    cs.cs_kv_ckpt_restore_tokens(pool, 0, L, new_slots, tail_host.cuda())
    out = torch.full_like(ref_out, float("nan"))
    decode_step(pool, tables, STEPS, out, q_last)
    torch.cuda.synchronize()
    # bit-identical to the uninterrupted run (same logical data, other pages), and right
    assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16))
    for l in range(L):
        want = np.empty((S, sh.Hq, sh.D))
        for s in range(S):
            K = torch.cat([prior[l][s][0], new_k[:STEPS + 1, l, s]]).float().numpy()
            V = torch.cat([prior[l][s][1], new_v[:STEPS + 1, l, s]]).float().numpy()
            want[s] = attention.attention_chunk(q_last[l, s:s + 1].float().numpy(), K, V, ctx0[s] + STEPS, sh.scale)[0]
        assert_attention_close(out[l], want, "layer %d after resume" % l)
