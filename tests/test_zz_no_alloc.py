"""cs_paged_attention_mixed_static -- the attention call for callers that cannot allocate --
against cs_paged_attention_mixed on the same batches, through the C ABI.

Two calls in a row on one stream, the second on a smaller batch: the library's static scratch
still holds the first call's work items and partials when the second starts, and nothing clears
it, so stale contents must not leak into the second result.  Both batches need scratch (decode
sequences cut into pieces, a chunk cut into key ranges).  The bar is bit-identity: the two
entry points run the same kernels in the same order on the same plan."""
import ctypes

import pytest
import torch

from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import Step, assert_attention_close, from_bits

pytestmark = pytest.mark.gpu


def make(ctx, ql, seed, sh):
    b = synth.make_batch(sh, ctx, ql, synth.generator(seed))
    st = Step(b, seed)
    cpu_pool = st.prior_pool()
    pool = cs.Pool(from_bits(cpu_pool, "cuda"), 1, b.num_pages, sh.Hkv, sh.D)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    cs.cs_kv_append(pool, 0, bb, st.k_new.cuda(), st.v_new.cuda())
    return b, st, pool, bb, st.q.cuda()


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    lib = cs.lib()
    sh = synth.Shape(8, 2, 128)
    big = make([9000, 300, 5000, 3000], [1, 1, 1, 40], 301, sh)
    small = make([2500, 1501], [1, 17], 302, sh)
    limit = lib.cs_static_scratch_bytes()
    assert limit == 64 << 20
    for b, st, pool, bb, q in (big, small):
        need = cs.cs_paged_attention_workspace_bytes(bb, sh.Hq, sh.Hkv, sh.D)
        assert 0 < need <= limit, "both batches must use the scratch"
    assert cs.cs_paged_attention_workspace_bytes(small[3], sh.Hq, sh.Hkv, sh.D) < cs.cs_paged_attention_workspace_bytes(big[3], sh.Hq, sh.Hkv, sh.D)
    stream = torch.cuda.current_stream().cuda_stream
    outs = []
    outs_alloc = [torch.full((b.T, sh.Hq, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda") for b, *_ in (big, small)]
    torch.cuda.synchronize()
    count0 = torch.cuda.memory_stats()["allocation.all.allocated"]           # allocations made so far, cumulative
    for (b, st, pool, bb, q), out in zip((big, small), outs_alloc):          # back to back, no synchronisation between
        rc = lib.cs_paged_attention_mixed_static(ctypes.byref(pool.c), 0, ctypes.byref(bb.c), q.data_ptr(), out.data_ptr(),
                                                 sh.Hq, ctypes.c_float(sh.scale), stream)
        assert rc == cs.CS_OK, lib.cs_status_string(rc)
        outs.append(out)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == count0   # the calls allocated nothing through torch
    torch.cuda.synchronize()
    for (b, st, pool, bb, q), out in zip((big, small), outs):
        ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
        want = torch.full_like(out, float("nan"))
        cs.cs_paged_attention_mixed(pool, 0, bb, q, want, sh.Hq, sh.scale, ws)
        torch.cuda.synchronize()
        assert torch.isfinite(out.float()).all()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), "static-scratch result differs"
        assert_attention_close(out, st.oracle_attention(), "static-scratch call")


def test_static_scratch_entry_point_refuses_what_does_not_fit_and_passes_errors_through():
    lib = cs.lib()
    sh = synth.Shape(64, 8, 128)
    # 40 decodes of 20000 keys cut every 256 keys: some 3000 work items of 32 KiB of partials each
    b = synth.make_batch(sh, [20000] * 40, [1] * 40, synth.generator(303))
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    pool = cs.Pool.empty(1, b.num_pages, sh.Hkv, sh.D)
    q = torch.zeros((b.T, sh.Hq, sh.D), dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, float("nan"))
    stream = torch.cuda.current_stream().cuda_stream
    cs.cs_set_decode_split_tokens(256)
    try:
        assert cs.cs_paged_attention_workspace_bytes(bb, sh.Hq, sh.Hkv, sh.D) > lib.cs_static_scratch_bytes()
        rc = lib.cs_paged_attention_mixed_static(ctypes.byref(pool.c), 0, ctypes.byref(bb.c), q.data_ptr(), out.data_ptr(),
                                                 sh.Hq, ctypes.c_float(sh.scale), stream)
    finally:
        cs.cs_set_decode_split_tokens(0)
    torch.cuda.synchronize()
    assert rc == cs.CS_ERR_STATIC_SCRATCH_TOO_SMALL
    assert b"static buffer" in lib.cs_status_string(rc)
    assert torch.isnan(out.float()).all(), "a refused call must not have enqueued anything"
    # argument errors come back as from the workspace entry point; empty batches are fine
    assert lib.cs_paged_attention_mixed_static(None, 0, ctypes.byref(bb.c), q.data_ptr(), out.data_ptr(), sh.Hq,
                                               ctypes.c_float(sh.scale), stream) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_paged_attention_mixed_static(ctypes.byref(pool.c), 0, ctypes.byref(bb.c), q.data_ptr(), out.data_ptr(), 63,
                                               ctypes.c_float(sh.scale), stream) == cs.CS_ERR_INVALID_ARG
    empty = cs.cs_batch(0, 0, None, 0, None, None, None, None)
    assert lib.cs_paged_attention_mixed_static(ctypes.byref(pool.c), 0, ctypes.byref(empty), None, None, sh.Hq,
                                               ctypes.c_float(sh.scale), stream) == cs.CS_OK


def test_static_scratch_entry_point_under_graph_capture():
    """What the entry point is for: a caller that records its layer loop into a HIP graph and so
    cannot allocate a workspace.  The first call on the device runs eagerly (it looks the
    buffer's address up); then append + attention are captured and replayed three times, with
    eager work between the replays, each replay bit-identical to the workspace entry point."""
    lib = cs.lib()
    sh = synth.Shape(8, 2, 128)
    b, st, pool, bb, q = make([7000, 200, 3100, 2000], [1, 1, 1, 24], 304, sh)
    assert cs.cs_paged_attention_workspace_bytes(bb, sh.Hq, sh.Hkv, sh.D) > 0
    want = torch.full((b.T, sh.Hq, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    cs.cs_paged_attention_mixed(pool, 0, bb, q, want, sh.Hq, sh.scale, cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D))
    out = torch.full_like(want, float("nan"))
    k_new, v_new = st.k_new.cuda(), st.v_new.cuda()

    def run():
        cs.cs_kv_append(pool, 0, bb, k_new, v_new)
        cs.cs_paged_attention_mixed_static(pool, 0, bb, q, out, sh.Hq, sh.scale)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                                  # eager first call: address lookup, warm-up
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for replay in range(3):
        out.fill_(float("nan"))
        assert torch.isfinite(torch.randn(1 << 16, device="cuda").sum()).item()      # eager work and a synchronisation
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), "replay %d differs" % replay
