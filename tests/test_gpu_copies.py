"""GPU parity of the copy kernels (append, checkpoint gather, restore) -- bit exact."""
import numpy as np
import pytest
import torch

from oracle import kv_layout
from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import NAN_BITS, Step, bits, from_bits

pytestmark = pytest.mark.gpu


def _dev_pool(np_pool, sh, L=None):
    t = from_bits(np_pool, "cuda")
    return cs.Pool(t, L or np_pool.shape[0], np_pool.shape[1], sh.Hkv, sh.D, page_size=sh.page_size)


def _run_append_case(batch, seed):
    st = Step(batch, seed)
    sh = batch.shape
    cpu_pool = st.prior_pool()
    pool = _dev_pool(cpu_pool, sh)
    bb = cs.Batch(batch.block_tables, batch.ctx_lens, batch.cu_q_lens)
    cs.cs_kv_append(pool, 0, bb, st.k_new.cuda(), st.v_new.cuda())
    torch.cuda.synchronize()
    st.oracle_append(cpu_pool)
    np.testing.assert_array_equal(bits(pool.tensor), cpu_pool)


def test_append_tiny_config():
    _run_append_case(synth.config_tiny(), 0)


@pytest.mark.parametrize("maker,seed", [(synth.config_llama8b_decode, 1), (synth.config_qwen7b_mixed, 2),
                                        (synth.config_llama70b_long, 3)])
def test_append_shrunk_configs(maker, seed):
    _run_append_case(maker(shrink=16), seed)


def test_append_page_boundaries_and_idle_sequences():
    # contexts that complete a page (15 mod 16), open one (0 mod 16), an idle sequence (q=0)
    # and head dim 64 with 3 kv heads
    sh = synth.Shape(6, 3, 64)
    g = synth.generator(11)
    b = synth.make_batch(sh, [15, 16, 31, 0, 5, 47, 1], [1, 1, 1, 17, 0, 33, 15], g, spare=3)
    _run_append_case(b, 11)


@pytest.mark.parametrize("Hkv,D,ps,S,qmax", [(4, 64, 16, 40, 1200), (8, 128, 8, 16, 1500), (8, 128, 16, 12, 2048)])
def test_append_of_tens_of_thousands_of_chunk_tokens(Hkv, D, ps, S, qmax):
    """Chunk appends of 18-35 thousand tokens (some nine thousand (page, kv head) workgroups):
    ragged chunk lengths and contexts, so that first and last pages are partly filled; every
    element of the pool is compared with the oracle's append."""
    import random
    rnd = random.Random(S * 1000 + D)
    sh = synth.Shape(2 * Hkv, Hkv, D, page_size=ps)
    ctx = [rnd.randint(0, 40) for _ in range(S)]
    ql = [rnd.randint(qmax // 2, qmax) for _ in range(S)]
    b = synth.make_batch(sh, ctx, ql, synth.generator(12), spare=5)
    assert b.T >= 17000
    _run_append_case(b, 12)


def test_append_empty_batch_is_a_noop():
    sh = synth.Shape(4, 2, 64)
    pool = cs.Pool.empty(1, 4, sh.Hkv, sh.D)
    pool.tensor.zero_()
    b = cs.Batch(torch.zeros((0, 1), dtype=torch.int32), torch.zeros(0, dtype=torch.int32),
                 torch.zeros(1, dtype=torch.int32))
    cs.cs_kv_append(pool, 0, b, None, None)
    torch.cuda.synchronize()
    assert int(pool.tensor.view(torch.int16).ne(0).sum()) == 0


def test_gather_restore_tiny_config():
    b = synth.config_tiny()
    sh = b.shape
    st = Step(b, 0)
    cpu_pool = st.oracle_append(st.prior_pool())
    pool = _dev_pool(cpu_pool, sh)
    dirty = synth.newly_filled_pages(b)
    ids = torch.tensor(dirty, dtype=torch.int32, device="cuda")
    staging = torch.empty((1, len(dirty), sh.page_elems), dtype=torch.bfloat16, device="cuda")
    cs.cs_kv_ckpt_gather(pool, 0, 1, ids, staging)
    torch.cuda.synchronize()
    want = kv_layout.ref_gather(cpu_pool, 0, 1, dirty)
    np.testing.assert_array_equal(bits(staging), want)
    fresh = [int(x) for x in b.spare_pages[:len(dirty)]]
    cs.cs_kv_ckpt_restore(pool, 0, 1, torch.tensor(fresh, dtype=torch.int32, device="cuda"), staging)
    torch.cuda.synchronize()
    kv_layout.ref_restore(cpu_pool, 0, 1, fresh, want)
    np.testing.assert_array_equal(bits(pool.tensor), cpu_pool)


@pytest.mark.parametrize("L,P,Hkv,D,n,lrange,strided", [
    (3, 40, 8, 128, 17, (0, 3), False),      # 64 KiB pages, all layers
    (4, 33, 4, 128, 9, (1, 3), False),       # 32 KiB pages, inner layer range
    (2, 21, 3, 64, 21, (0, 2), True),        # 12 KiB pages (ragged last chunk), padded strides
    (2, 9, 2, 64, 1, (1, 2), False),
])
def test_gather_restore_multilayer(L, P, Hkv, D, n, lrange, strided):
    rng = np.random.default_rng(L * 1000 + P)
    pe = kv_layout.page_elems(Hkv, D)
    ps = pe + 64 if strided else pe
    ls = P * ps + (128 if strided else 0)
    flat = rng.integers(0, 2 ** 16, size=L * ls, dtype=np.uint16)
    dev = from_bits(flat, "cuda")
    pool = cs.Pool(dev, L, P, Hkv, D, layer_stride=ls, page_stride=ps)

    def view(a):      # [L, P, pe] view of the strided flat array
        return np.lib.stride_tricks.as_strided(a, (L, P, pe), (ls * 2, ps * 2, 2))

    ids = rng.permutation(P)[:n].astype(np.int32)
    l0, l1 = lrange
    staging = torch.full(((l1 - l0), n, pe), -1.0, dtype=torch.bfloat16, device="cuda")
    cs.cs_kv_ckpt_gather(pool, l0, l1, torch.from_numpy(ids).cuda(), staging)
    torch.cuda.synchronize()
    cpu = view(flat).reshape(L, P, 2, Hkv, 16 * D).copy()
    want = kv_layout.ref_gather(cpu, l0, l1, ids)
    np.testing.assert_array_equal(bits(staging), want)
    np.testing.assert_array_equal(bits(dev), flat)                    # the pool is only read
    # restore into other pages; everything else (padding included) stays bit-identical
    dst = rng.permutation(P)[:n].astype(np.int32)
    cs.cs_kv_ckpt_restore(pool, l0, l1, torch.from_numpy(dst).cuda(), staging)
    torch.cuda.synchronize()
    after = bits(dev)
    kv_layout.ref_restore(cpu, l0, l1, dst, want)
    np.testing.assert_array_equal(view(after).reshape(cpu.shape), cpu)
    expect_flat = flat.copy()
    view(expect_flat)[...] = cpu.reshape(L, P, pe)
    np.testing.assert_array_equal(after, expect_flat)


@pytest.mark.parametrize("L,P,Hkv,D,n,lrange,strided", [
    (3, 40, 8, 128, 300, (0, 3), False),
    (4, 33, 4, 128, 77, (1, 3), False),
    (2, 21, 3, 64, 21 * 16, (0, 2), True),    # every slot of the pool, padded strides
    (2, 9, 2, 64, 1, (1, 2), False),
])
def test_token_gather_restore(L, P, Hkv, D, n, lrange, strided):
    """Token-granular checkpoint: bit-exact against the oracle, pool untouched by the gather,
    restore writes the named slots and nothing else (padding included)."""
    rng = np.random.default_rng(L * 1000 + P + n)
    pe = kv_layout.page_elems(Hkv, D)
    ps = pe + 64 if strided else pe
    ls = P * ps + (128 if strided else 0)
    flat = rng.integers(0, 2 ** 16, size=L * ls, dtype=np.uint16)
    dev = from_bits(flat, "cuda")
    pool = cs.Pool(dev, L, P, Hkv, D, layer_stride=ls, page_stride=ps)

    def view(a):
        return np.lib.stride_tricks.as_strided(a, (L, P, pe), (ls * 2, ps * 2, 2))

    slots = rng.permutation(P * 16)[:n].astype(np.int32)
    l0, l1 = lrange
    staging = torch.full(((l1 - l0), n, 2, Hkv, D), -1.0, dtype=torch.bfloat16, device="cuda")
    cs.cs_kv_ckpt_gather_tokens(pool, l0, l1, torch.from_numpy(slots).cuda(), staging)
    torch.cuda.synchronize()
    cpu = view(flat).reshape(L, P, 2, Hkv, 16 * D).copy()
    want = kv_layout.ref_gather_tokens(cpu, l0, l1, slots)
    np.testing.assert_array_equal(bits(staging), want)
    np.testing.assert_array_equal(bits(dev), flat)
    dst = rng.permutation(P * 16)[:n].astype(np.int32)
    cs.cs_kv_ckpt_restore_tokens(pool, l0, l1, torch.from_numpy(dst).cuda(), staging)
    torch.cuda.synchronize()
    after = bits(dev)
    kv_layout.ref_restore_tokens(cpu, l0, l1, dst, want)
    expect_flat = flat.copy()
    view(expect_flat)[...] = cpu.reshape(L, P, pe)
    np.testing.assert_array_equal(after, expect_flat)


def test_token_checkpoint_of_a_decode_step_restores_attention():
    """The paper's per-step use: checkpoint the tokens a decode step has just appended, drop
    them, bring them back into fresh pages, and the next attention call is bit-identical."""
    b = synth.config_llama8b_decode(shrink=16)
    sh = b.shape
    st = Step(b, 5)
    cpu_pool = st.prior_pool()
    pool = _dev_pool(cpu_pool, sh)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    cs.cs_kv_append(pool, 0, bb, st.k_new.cuda(), st.v_new.cuda())
    q = st.q.cuda()
    out = torch.empty_like(q)
    cs.cs_paged_attention_mixed(pool, 0, bb, q, out, sh.Hq, sh.scale, cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D))
    pos = b.ctx_lens.long()
    pages = b.block_tables[torch.arange(b.S), pos // 16].long()
    slots = (pages * 16 + pos % 16).to(torch.int32).cuda()
    staging = torch.empty((1, b.S, 2, sh.Hkv, sh.D), dtype=torch.bfloat16, device="cuda")
    cs.cs_kv_ckpt_gather_tokens(pool, 0, 1, slots, staging)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(bits(staging[0, :, 0]), bits(st.k_new))
    np.testing.assert_array_equal(bits(staging[0, :, 1]), bits(st.v_new))
    # overwrite the new tokens' slots with NaN bits, then restore them from the buffer
    junk = torch.full_like(staging, float("nan"))
    cs.cs_kv_ckpt_restore_tokens(pool, 0, 1, slots, junk)
    cs.cs_kv_ckpt_restore_tokens(pool, 0, 1, slots, staging)
    out2 = torch.empty_like(q)
    cs.cs_paged_attention_mixed(pool, 0, bb, q, out2, sh.Hq, sh.scale, cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D))
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))


def test_token_gather_bad_slots_and_errors():
    pool = cs.Pool.empty(2, 8, 2, 64)
    pool.tensor.view(torch.int16).fill_(0x1234)
    staging = torch.zeros((2, 3, 2, 2, 64), dtype=torch.bfloat16, device="cuda")
    cs.cs_kv_ckpt_gather_tokens(pool, 0, 2, torch.zeros(0, dtype=torch.int32, device="cuda"), staging)
    slots = torch.tensor([5 * 16 + 3, -1, 8 * 16], dtype=torch.int32, device="cuda")   # -1 and page 8 are outside
    cs.cs_kv_ckpt_gather_tokens(pool, 0, 2, slots, staging)
    torch.cuda.synchronize()
    s = staging.view(torch.int16).cpu()
    assert s[:, 0].eq(0x1234).all() and s[:, 1:].eq(0).all()
    with pytest.raises(cs.CsError) as e:
        cs.cs_kv_ckpt_gather_tokens(pool, 0, 2, slots, staging[:1])
    assert e.value.status == cs.CS_ERR_STAGING_TOO_SMALL
    with pytest.raises(cs.CsError) as e:
        cs.cs_kv_ckpt_restore_tokens(pool, 1, 3, slots, staging)
    assert e.value.status == cs.CS_ERR_INVALID_ARG


def test_gather_zero_pages_and_bad_ids_are_harmless():
    pool = cs.Pool.empty(2, 8, 2, 64)
    pool.tensor.view(torch.int16).fill_(0x1234)
    staging = torch.zeros((2, 3, pool.page_elems), dtype=torch.bfloat16, device="cuda")
    cs.cs_kv_ckpt_gather(pool, 0, 2, torch.zeros(0, dtype=torch.int32, device="cuda"), staging)
    ids = torch.tensor([5, -1, 8], dtype=torch.int32, device="cuda")   # -1 and 8 are outside the pool
    cs.cs_kv_ckpt_gather(pool, 0, 2, ids, staging)
    torch.cuda.synchronize()
    s = staging.view(torch.int16).cpu()
    assert s[:, 0].eq(0x1234).all() and s[:, 1:].eq(0).all()


def test_error_codes_need_no_device_work():
    pool = cs.Pool.empty(1, 4, 2, 64)
    staging = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    ids = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(cs.CsError) as e:
        cs.cs_kv_ckpt_gather(pool, 0, 1, ids, staging)
    assert e.value.status == cs.CS_ERR_STAGING_TOO_SMALL
    with pytest.raises(cs.CsError) as e:
        cs.cs_kv_ckpt_gather(pool, 0, 2, ids, staging)
    assert e.value.status == cs.CS_ERR_INVALID_ARG


def test_plain_copy():
    src = torch.randint(0, 255, (3 * 16384 + 4096 + 16,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    cs.cs_debug_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
