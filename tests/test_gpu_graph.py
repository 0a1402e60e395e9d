"""The calls neither synchronise nor allocate, so a caller may record them into a HIP graph
(the per-layer loop of a small batch is launch-bound; the paper's engine launches its model
as graphs, Sec. 5).  A captured multi-layer step is replayed several times, with eager work
and synchronisations between the replays, and every replay must reproduce the eager result
bit for bit."""
import numpy as np
import pytest
import torch

from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import Step, bits, from_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("maker,shrink", [(synth.config_tiny, None), (synth.config_qwen7b_mixed, 16),
                                          (synth.config_llama70b_long, 32)])
def test_captured_layers_replay_bit_identical(maker, shrink):
    b = maker() if shrink is None else maker(shrink=shrink)
    sh = b.shape
    L = 3
    steps = [Step(b, 70 + l, layer=l) for l in range(L)]
    cpu_pool = steps[0].prior_pool(L=L)
    for l in range(1, L):
        steps[l].layer = l
        cpu_pool[l] = steps[l].prior_pool(L=L)[l]
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
    q = [st.q.cuda() for st in steps]
    kn = [st.k_new.cuda() for st in steps]
    vn = [st.v_new.cuda() for st in steps]

    def fresh_pool():
        return cs.Pool(from_bits(cpu_pool, "cuda"), L, cpu_pool.shape[1], sh.Hkv, sh.D)

    def run(pool, outs):
        for l in range(L):
            cs.cs_kv_append(pool, l, bb, kn[l], vn[l])
            cs.cs_paged_attention_mixed(pool, l, bb, q[l], outs[l], sh.Hq, sh.scale, ws)

    # eager reference
    pool_e = fresh_pool()
    outs_e = [torch.zeros((b.T, sh.Hq, sh.D), dtype=torch.bfloat16, device="cuda") for _ in range(L)]
    run(pool_e, outs_e)
    torch.cuda.synchronize()
    want = [bits(o) for o in outs_e]
    want_pool = bits(pool_e.tensor)

    # captured
    pool_g = fresh_pool()
    outs_g = [torch.zeros_like(o) for o in outs_e]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(pool_g, outs_g)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(pool_g, outs_g)
    for replay in range(3):
        for o in outs_g:
            o.fill_(float("nan"))                             # eager work between replays
        junk = torch.randn(1 << 16, device="cuda").sum().item()   # and a synchronisation
        assert np.isfinite(junk)
        graph.replay()
        torch.cuda.synchronize()
        for l in range(L):
            np.testing.assert_array_equal(bits(outs_g[l]), want[l], err_msg="replay %d layer %d" % (replay, l))
        np.testing.assert_array_equal(bits(pool_g.tensor), want_pool)
