"""GPU parity of cs_paged_attention_mixed against the fp64 oracle on logical sequences."""
import numpy as np
import pytest
import torch

from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import Step, assert_attention_close, bits, from_bits

pytestmark = pytest.mark.gpu


def run_step(batch, seed, q_gain=1.0, split=0, check_append=True):
    """append + attention through the C ABI; returns (gpu_out, Step, device pool, cs.Batch)."""
    st = Step(batch, seed, q_gain=q_gain)
    sh = batch.shape
    cpu_pool = st.prior_pool()
    pool = cs.Pool(from_bits(cpu_pool, "cuda"), cpu_pool.shape[0], cpu_pool.shape[1], sh.Hkv, sh.D)
    bb = cs.Batch(batch.block_tables, batch.ctx_lens, batch.cu_q_lens)
    cs.cs_kv_append(pool, 0, bb, st.k_new.cuda(), st.v_new.cuda())
    if check_append:
        torch.cuda.synchronize()
        np.testing.assert_array_equal(bits(pool.tensor), st.oracle_append(cpu_pool))
    cs.cs_set_decode_split_tokens(split)
    try:
        ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
        out = torch.full((batch.T, sh.Hq, sh.D), float("nan"), dtype=torch.bfloat16, device="cuda")
        cs.cs_paged_attention_mixed(pool, 0, bb, st.q.cuda(), out, sh.Hq, sh.scale, ws)
        torch.cuda.synchronize()
    finally:
        cs.cs_set_decode_split_tokens(0)
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


def test_decode_llama8b_shrunk():
    b = synth.config_llama8b_decode(shrink=8)
    out, st, _, _ = run_step(b, 1)
    assert_attention_close(out, st.oracle_attention(), "llama8b/8")
