"""Asynchronous checkpoint pipeline: gather + one device-to-host copy on a stream of its own,
host-to-device + restore on resume, concurrent with attention on the compute stream."""
import numpy as np
import pytest
import torch

from oracle import kv_layout
from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from helpers import Step, assert_attention_close, bits, from_bits

pytestmark = pytest.mark.gpu


def test_save_to_host_and_load_into_fresh_pages_matches_the_oracle():
    b = synth.config_qwen14b_ckpt(shrink=16, layers=3)
    sh = b.shape
    st = Step(b, 4, layer=1)
    cpu_pool = st.oracle_append(st.prior_pool(L=3))
    rng = np.random.default_rng(0)
    cpu_pool[0] = rng.integers(0, 0x7F00, size=cpu_pool[0].shape, dtype=np.uint16)   # other layers hold data too
    cpu_pool[2] = rng.integers(0, 0x7F00, size=cpu_pool[2].shape, dtype=np.uint16)
    pool = cs.Pool(from_bits(cpu_pool, "cuda"), 3, b.num_pages, sh.Hkv, sh.D)
    dirty = b.extra["dirty_pages"]
    fresh = [int(x) for x in b.spare_pages[:len(dirty)]]
    ids = torch.tensor(dirty, dtype=torch.int32, device="cuda")
    staging = torch.empty((3, len(dirty), sh.page_elems), dtype=torch.bfloat16, device="cuda")
    host = torch.empty((3, len(dirty), sh.page_elems), dtype=torch.bfloat16).pin_memory()
    side = torch.cuda.Stream()
    cs.cs_kv_ckpt_save(pool, 0, 3, ids, staging, host, stream=side)
    side.synchronize()
    want = kv_layout.ref_gather(cpu_pool, 0, 3, dirty)
    np.testing.assert_array_equal(bits(host), want)
    # preemption: the pages are released (overwritten); resume into fresh pages from the host copy
    pool.tensor[:, dirty] = float("nan")
    staging.fill_(0)
    cs.cs_kv_ckpt_load(pool, 0, 3, torch.tensor(fresh, dtype=torch.int32, device="cuda"), staging, host, stream=side)
    side.synchronize()
    for p in dirty:
        cpu_pool[:, p] = 0x7FC0
    kv_layout.ref_restore(cpu_pool, 0, 3, fresh, want)
    got = bits(pool.tensor)
    keep = np.ones(b.num_pages, bool)
    keep[dirty] = False                                   # NaN payloads differ; compare all other pages
    np.testing.assert_array_equal(got[:, keep], cpu_pool[:, keep])


def test_checkpoint_on_a_side_stream_does_not_change_attention():
    """The gathered pages have no data dependency with the running step: attention on the
    compute stream gives bit-identical output with and without a concurrent save."""
    b = synth.config_qwen7b_mixed(shrink=4)
    sh = b.shape
    st = Step(b, 2)
    cpu_pool = st.oracle_append(st.prior_pool())
    pool = cs.Pool(from_bits(cpu_pool, "cuda"), 1, b.num_pages, sh.Hkv, sh.D)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    q = st.q.cuda()
    ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
    out0 = torch.empty((b.T, sh.Hq, sh.D), dtype=torch.bfloat16, device="cuda")
    cs.cs_paged_attention_mixed(pool, 0, bb, q, out0, sh.Hq, sh.scale, ws)
    torch.cuda.synchronize()
    assert_attention_close(out0, st.oracle_attention(), "mixed/4")
    # all full pages of the offline requests are checkpointed while attention runs again
    pages = []
    for s in range(b.extra["n_online"], b.S):
        pages += [int(x) for x in b.block_tables[s, : int(b.ctx_lens[s] + b.q_lens[s]) // 16]]
    ids = torch.tensor(pages, dtype=torch.int32, device="cuda")
    staging = torch.empty((1, len(pages), sh.page_elems), dtype=torch.bfloat16, device="cuda")
    host = torch.empty((1, len(pages), sh.page_elems), dtype=torch.bfloat16).pin_memory()
    side = torch.cuda.Stream()
    out1 = torch.empty_like(out0)
    for _ in range(3):
        cs.cs_kv_ckpt_save(pool, 0, 1, ids, staging, host, stream=side)
        cs.cs_paged_attention_mixed(pool, 0, bb, q, out1, sh.Hq, sh.scale, ws)
    torch.cuda.synchronize()
    assert torch.equal(out0.view(torch.int16), out1.view(torch.int16))
    np.testing.assert_array_equal(bits(host), kv_layout.ref_gather(cpu_pool, 0, 1, pages))


def test_incremental_rounds_through_the_page_map_and_the_host_page_store():
    """Three offline requests fill pages over three steps; after every step the pages that
    have no host copy yet are saved as one run of the host page store (one contiguous
    device-to-host copy each).  Two requests are then preempted (their GPU pages overwritten)
    and resumed into fresh pages, run by run.  Every byte on the host and in the restored
    pages must be what the oracle's gather / restore give."""
    sh = synth.Shape(8, 2, 64)
    L, P, H = 3, 48, 40
    rng = np.random.default_rng(7)
    cpu_pool = rng.integers(0, 0x7F00, size=(L, P, 2, sh.Hkv, 16 * sh.D), dtype=np.uint16)
    pool = cs.Pool(from_bits(cpu_pool, "cuda"), L, P, sh.Hkv, sh.D)
    store_t = torch.zeros((H, L, sh.page_elems), dtype=torch.bfloat16).pin_memory()
    store = cs.HostStore(store_t)
    pmap = cs.PageMap(P, H)
    side = torch.cuda.Stream()
    staging = torch.empty((P, L, sh.page_elems), dtype=torch.bfloat16, device="cuda")
    perm = rng.permutation(P).tolist()
    req = {"a": perm[0:7], "b": perm[7:12], "c": perm[12:21]}            # their GPU pages, in order
    filled = {"a": [2, 5, 7], "b": [1, 3, 5], "c": [4, 4, 9]}            # full pages after steps 1..3
    host_img = np.zeros((H, L, sh.page_elems), np.uint16)                # what the store must hold

    def checkpoint_round(step, who):
        pages = [g for r in who for g in req[r][:filled[r][step]]]
        dirty, first = pmap.checkpoint(pages)
        if dirty:
            ids = torch.tensor(dirty, dtype=torch.int32, device="cuda")
            cs.cs_kv_ckpt_save_run(pool, 0, L, ids, staging, store, first, stream=side)
            side.synchronize()
            want = kv_layout.ref_gather(cpu_pool, 0, L, dirty)           # [L][n][...]
            host_img[first:first + len(dirty)] = np.transpose(want, (1, 0, 2))
        return dirty

    assert sorted(checkpoint_round(0, "abc")) == sorted(req["a"][:2] + req["b"][:1] + req["c"][:4])
    assert sorted(checkpoint_round(1, "abc")) == sorted(req["a"][2:5] + req["b"][1:3])   # c filled nothing new
    np.testing.assert_array_equal(bits(store_t), host_img)

    # preemption of a and b: pages released and reused by someone else
    host_a = pmap.evict(req["a"])
    host_b = pmap.evict(req["b"])
    assert host_a[5:] == [-1, -1] and all(h >= 0 for h in host_a[:5])   # pages 5, 6 never were full
    assert host_b[3:] == [-1, -1]
    gone = req["a"] + req["b"]
    pool.tensor[:, gone] = float("nan")
    assert sorted(checkpoint_round(2, "c")) == sorted(req["c"][4:9])
    np.testing.assert_array_equal(bits(store_t), host_img)

    # resume a and b into fresh pages, one host-to-device copy per ascending run
    fresh = perm[21:]
    expect = bits(pool.tensor).copy().reshape(cpu_pool.shape)
    for host_pages in (host_a[:5], host_b[:3]):
        gpu_new = [fresh.pop() for _ in host_pages]
        for i, n in cs.ascending_runs(host_pages):
            ids = torch.tensor(gpu_new[i:i + n], dtype=torch.int32, device="cuda")
            cs.cs_kv_ckpt_load_run(pool, 0, L, ids, staging, store, host_pages[i], stream=side)
            run_img = np.transpose(host_img[host_pages[i]:host_pages[i] + n], (1, 0, 2))
            kv_layout.ref_restore(expect, 0, L, gpu_new[i:i + n], np.ascontiguousarray(run_img))
        pmap.bind(host_pages, gpu_new)
        assert [pmap.host_of(g) for g in gpu_new] == host_pages
    side.synchronize()
    got = bits(pool.tensor).reshape(cpu_pool.shape)
    keep = np.ones(P, bool)
    keep[gone] = False                                                   # NaN payloads: not compared
    np.testing.assert_array_equal(got[:, keep], expect[:, keep])
    # and the restored pages hold what the evicted pages held
    old_a = req["a"][:5]
    new_a = [g for g in range(P) if pmap.host_of(g) in host_a[:5]]
    for h in host_a[:5]:
        g_new = pmap.gpu_of(h)
        g_old = old_a[host_a.index(h)]
        np.testing.assert_array_equal(got[:, g_new], cpu_pool[:, g_old])
    assert len(new_a) == 5


def test_run_entry_points_reject_a_mismatched_store():
    sh = synth.Shape(4, 2, 64)
    pool = cs.Pool.empty(2, 8, sh.Hkv, sh.D)
    ids = torch.zeros(2, dtype=torch.int32, device="cuda")
    staging = torch.empty((2, 2, sh.page_elems), dtype=torch.bfloat16, device="cuda")
    store = cs.HostStore(torch.zeros((4, 2, sh.page_elems), dtype=torch.bfloat16).pin_memory())
    with pytest.raises(cs.CsError):
        cs.cs_kv_ckpt_save_run(pool, 0, 1, ids, staging, store, 0)        # one layer, store holds two
    with pytest.raises(cs.CsError):
        cs.cs_kv_ckpt_save_run(pool, 0, 2, ids, staging, store, 3)        # run 3..4 leaves the store
    with pytest.raises(cs.CsError):
        cs.cs_kv_ckpt_load_run(pool, 0, 2, ids, staging[:1], store, 0)    # staging too small
    cs.cs_kv_ckpt_save_run(pool, 0, 2, ids, staging, store, 2)
    torch.cuda.synchronize()
