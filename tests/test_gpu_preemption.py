"""Layer-wise preemption loop: safepoints every k layers, the offline tail dropped between
two layers, online rows untouched by the preemption."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import Step, assert_attention_close, from_bits

pytestmark = pytest.mark.gpu

L = 8


def setup(dtype=torch.bfloat16):
    b = synth.config_qwen7b_mixed(shrink=16)
    sh = b.shape
    steps = [Step(b, 20 + l, layer=0, dtype=dtype) for l in range(L)]   # independent data per layer
    pools = np.stack([st.prior_pool()[0] for st in steps])           # [L, P, 2, Hkv, 16D]
    pool = cs.Pool(from_bits(pools, "cuda", dtype), L, b.num_pages, sh.Hkv, sh.D)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    q = torch.stack([st.q for st in steps]).cuda()
    k = torch.stack([st.k_new for st in steps]).cuda()
    v = torch.stack([st.v_new for st in steps]).cuda()
    ws = cs.run_layers_workspace_for(bb, b.extra["n_online"], sh.Hq, sh.Hkv, sh.D)
    return b, sh, steps, pool, bb, q, k, v, ws


def run(pool, bb, q, k, v, ws, sh, sp):
    out = torch.full_like(q, float("nan"))
    first = cs.cs_run_layers(pool, 0, L, bb, q, k, v, out, sh.Hq, sh.scale, ws, sp, f16=q.dtype == torch.float16)
    torch.cuda.synchronize()
    return out, first


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
def test_no_preemption_runs_every_layer_on_the_full_batch(dtype):
    b, sh, steps, pool, bb, q, k, v, ws = setup(dtype)
    flag = ctypes.c_int32(0)
    sp = cs.cs_safepoint(ctypes.addressof(flag), cs.POLL_FN(0), None, 4, b.extra["n_online"], 0)
    out, first = run(pool, bb, q, k, v, ws, sh, sp)
    assert first == -1
    for l in (0, 3, 7):
        assert_attention_close(out[l], steps[l].oracle_attention(), "layer %d" % l)


@pytest.mark.parametrize("sync", [0, 1])
def test_preemption_at_the_second_safepoint(sync):
    b, sh, steps, pool, bb, q, k, v, ws = setup()
    n_on = b.extra["n_online"]
    full, _ = run(pool, bb, q, k, v, ws, sh, None)
    calls = []

    def poll(_):
        calls.append(1)
        return 1 if len(calls) >= 2 else 0                           # the signal arrives during layers 0..3

    cb = cs.POLL_FN(poll)
    sp = cs.cs_safepoint(None, cb, None, 4, n_on, sync)
    # fresh pool (the first run appended already; appending the same values again is idempotent)
    out, first = run(pool, bb, q, k, v, ws, sh, sp)
    assert first == 4 and len(calls) == 2
    T_on = int(b.cu_q_lens[n_on])
    # layers 0..3: whole batch, identical to the unpreempted run
    assert torch.equal(out[:4].view(torch.int16), full[:4].view(torch.int16))
    # layers 4..7: online rows computed (and correct), offline rows never written
    assert torch.isnan(out[4:, T_on:].float()).all()
    for l in (4, 7):
        assert_attention_close(out[l, :T_on], steps[l].oracle_attention(range(n_on))[:T_on], "online layer %d" % l)


def test_flag_raised_before_the_iteration_preempts_at_layer_zero():
    b, sh, steps, pool, bb, q, k, v, ws = setup()
    flag = ctypes.c_int32(1)
    sp = cs.cs_safepoint(ctypes.addressof(flag), cs.POLL_FN(0), None, 4, b.extra["n_online"], 0)
    out, first = run(pool, bb, q, k, v, ws, sh, sp)
    assert first == 0
    T_on = int(b.cu_q_lens[b.extra["n_online"]])
    assert torch.isnan(out[:, T_on:].float()).all() and torch.isfinite(out[:, :T_on].float()).all()


def test_offline_decodes_in_the_tail_and_an_online_prefix_that_needs_more_workspace():
    """The ordinary co-serving batch: a few online decodes on long contexts first, many offline
    decodes behind them.  Whole, no sequence is cut (enough work items as they are) and no
    workspace is needed; the online prefix alone is cut into pieces and needs partials.  The
    loop must ask for the larger workspace up front: with the full batch's (none) it refuses
    before enqueuing anything; with cs_run_layers_workspace_bytes() the preempted iteration
    completes and the online rows of its online-only layers meet the oracle."""
    sh = synth.Shape(4, 2, 64)
    n_on, n_off = 2, 300
    b = synth.make_batch(sh, [3000, 5000] + [200] * n_off, [1] * (n_on + n_off), synth.generator(31))
    steps = [Step(b, 40 + l, layer=0) for l in range(L)]
    pools = np.stack([st.prior_pool()[0] for st in steps])
    pool = cs.Pool(from_bits(pools, "cuda"), L, b.num_pages, sh.Hkv, sh.D)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    q = torch.stack([st.q for st in steps]).cuda()
    k = torch.stack([st.k_new for st in steps]).cuda()
    v = torch.stack([st.v_new for st in steps]).cuda()
    full_need = cs.cs_paged_attention_workspace_bytes(bb, sh.Hq, sh.Hkv, sh.D)
    need = cs.cs_run_layers_workspace_bytes(bb, n_on, sh.Hq, sh.Hkv, sh.D)
    assert full_need == 0 and need > 0
    assert need == cs.cs_paged_attention_workspace_bytes(bb.truncated(n_on), sh.Hq, sh.Hkv, sh.D)

    def poll_twice():
        calls = []

        def poll(_):
            calls.append(1)
            return 1 if len(calls) >= 2 else 0
        return cs.POLL_FN(poll), calls

    cb, calls = poll_twice()
    sp = cs.cs_safepoint(None, cb, None, 4, n_on, 0)
    out = torch.full_like(q, float("nan"))
    with pytest.raises(cs.CsError) as e:
        cs.cs_run_layers(pool, 0, L, bb, q, k, v, out, sh.Hq, sh.scale, torch.empty(16, dtype=torch.uint8, device="cuda"), sp)
    torch.cuda.synchronize()
    assert e.value.status == cs.CS_ERR_WORKSPACE_TOO_SMALL and not calls
    assert torch.isnan(out.float()).all(), "a refused iteration must not have enqueued a layer"

    ws = cs.run_layers_workspace_for(bb, n_on, sh.Hq, sh.Hkv, sh.D)
    out, first = run(pool, bb, q, k, v, ws, sh, sp)
    assert first == 4 and len(calls) == 2
    T_on = int(b.cu_q_lens[n_on])
    assert torch.isnan(out[4:, T_on:].float()).all() and torch.isfinite(out[:4].float()).all()
    for l in (0, 3):
        assert_attention_close(out[l], steps[l].oracle_attention(), "full layer %d" % l)
    for l in (4, 7):
        assert_attention_close(out[l, :T_on], steps[l].oracle_attention(range(n_on))[:T_on], "online layer %d" % l)
