"""The C ABI without a GPU: the library loads, exports what the header declares, and its
host-side checks answer with error codes before anything would be enqueued."""
import ctypes
import os
import re

import pytest
import torch

from paper_2410_01228_amd import binding as cs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "conserve_kv.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cs_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"cs_kv_append", "cs_paged_attention_mixed", "cs_kv_ckpt_gather", "cs_kv_ckpt_restore"} <= set(names)
    lib = cs.lib()
    for n in names:
        assert hasattr(lib, n), "missing export: " + n
    assert sorted(cs.EXPORTS) == names


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(cs, "_lib", None)
    monkeypatch.setattr(cs, "LIB_PATH", "/nonexistent/libconserve_kv.so")
    with pytest.raises(RuntimeError):
        cs.lib()


def test_page_bytes_and_status_strings():
    assert cs.cs_page_bytes(8, 128) == 65536 and cs.cs_page_bytes(4, 128) == 32768 and cs.cs_page_bytes(2, 64) == 8192
    assert cs.cs_page_bytes(8, 96) == 0
    lib = cs.lib()
    assert lib.cs_status_string(0) == b"ok"
    assert lib.cs_status_string(cs.CS_ERR_WORKSPACE_TOO_SMALL) == b"workspace too small"


def _pool(base=0x1000, L=2, P=8, Hkv=2, D=64, page=16, ls=None, ps=None):
    pe = 2 * Hkv * page * D
    ps = pe if ps is None else ps
    return cs.cs_kv_pool(base, L, P, page, Hkv, D, P * ps if ls is None else ls, ps)


def _batch(ctx, ql, max_blocks=64, fake_dev=0x2000):
    h_ctx = torch.tensor(ctx, dtype=torch.int32)
    cu = torch.zeros(len(ql) + 1, dtype=torch.int32)
    cu[1:] = torch.cumsum(torch.tensor(ql, dtype=torch.int32), 0)
    b = cs.cs_batch(len(ctx), int(cu[-1]), fake_dev, max_blocks, fake_dev, fake_dev, h_ctx.data_ptr(), cu.data_ptr())
    return b, (h_ctx, cu)


def test_checkpoint_argument_checks_happen_on_the_host():
    lib = cs.lib()
    ids, st = 0x3000, 0x4000
    page = cs.cs_page_bytes(2, 64)
    p = _pool()
    assert lib.cs_kv_ckpt_gather(ctypes.byref(p), 0, 2, ids, 3, st, 2 * 3 * page - 1, None) == cs.CS_ERR_STAGING_TOO_SMALL
    assert lib.cs_kv_ckpt_gather(ctypes.byref(p), 0, 3, ids, 3, st, 1 << 30, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_kv_ckpt_gather(ctypes.byref(p), 1, 0, ids, 3, st, 1 << 30, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_kv_ckpt_gather(ctypes.byref(p), 0, 2, None, 3, st, 1 << 30, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_kv_ckpt_restore(ctypes.byref(p), 0, 2, ids, -1, st, 1 << 30, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_kv_ckpt_restore(ctypes.byref(p), 0, 2, ids, 3, st + 4, 1 << 30, None) == cs.CS_ERR_INVALID_ARG
    # empty work is legal and launches nothing
    assert lib.cs_kv_ckpt_gather(ctypes.byref(p), 0, 2, None, 0, None, 0, None) == cs.CS_OK
    assert lib.cs_kv_ckpt_restore(ctypes.byref(p), 1, 1, ids, 3, st, 0, None) == cs.CS_OK
    # pages of 8 tokens: half the bytes per page
    p8 = _pool(page=8)
    assert lib.cs_pool_page_bytes(ctypes.byref(p8)) == page // 2 and lib.cs_pool_page_bytes(ctypes.byref(p)) == page
    assert lib.cs_kv_ckpt_gather(ctypes.byref(p8), 0, 2, ids, 3, st, 2 * 3 * (page // 2) - 1, None) == cs.CS_ERR_STAGING_TOO_SMALL
    assert lib.cs_kv_ckpt_gather(ctypes.byref(p8), 0, 2, None, 0, None, 0, None) == cs.CS_OK
    assert lib.cs_kv_ckpt_gather(ctypes.byref(_pool(page=8, ps=2 * 2 * 8 * 64 - 8)), 0, 1, ids, 1, st, 1 << 30, None) == cs.CS_ERR_INVALID_ARG
    # unsupported / malformed pools
    assert lib.cs_pool_page_bytes(ctypes.byref(_pool(page=32))) == 0 and lib.cs_pool_page_bytes(None) == 0
    assert lib.cs_kv_ckpt_gather(ctypes.byref(_pool(page=4)), 0, 1, ids, 1, st, 1 << 30, None) == cs.CS_ERR_UNSUPPORTED
    assert lib.cs_kv_ckpt_gather(ctypes.byref(_pool(page=32)), 0, 1, ids, 1, st, 1 << 30, None) == cs.CS_ERR_UNSUPPORTED
    assert lib.cs_kv_ckpt_gather(ctypes.byref(_pool(D=96)), 0, 1, ids, 1, st, 1 << 30, None) == cs.CS_ERR_UNSUPPORTED
    assert lib.cs_kv_ckpt_gather(ctypes.byref(_pool(ps=100)), 0, 1, ids, 1, st, 1 << 30, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_kv_ckpt_gather(ctypes.byref(_pool(base=0)), 0, 1, ids, 1, st, 1 << 30, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_kv_ckpt_gather(None, 0, 1, ids, 1, st, 1 << 30, None) == cs.CS_ERR_INVALID_ARG


def test_batch_checks_and_empty_batches():
    lib = cs.lib()
    p = _pool()
    q = 0x5000
    b, keep = _batch([5, 40], [1, 3])
    assert lib.cs_kv_append(ctypes.byref(p), 2, ctypes.byref(b), q, q, None) == cs.CS_ERR_INVALID_ARG      # layer
    assert lib.cs_kv_append(ctypes.byref(p), 0, ctypes.byref(b), None, q, None) == cs.CS_ERR_INVALID_ARG
    b2, keep2 = _batch([5, 40], [1, 3], max_blocks=2)                       # 43 tokens need 3 blocks
    assert lib.cs_kv_append(ctypes.byref(p), 0, ctypes.byref(b2), q, q, None) == cs.CS_ERR_INVALID_ARG
    b3, keep3 = _batch([5, 40], [1, 3], max_blocks=5)                       # ... and 6 blocks of 8 tokens
    assert lib.cs_kv_append(ctypes.byref(_pool(page=8)), 0, ctypes.byref(b3), q, q, None) == cs.CS_ERR_INVALID_ARG
    b3, keep3 = _batch([5, -1], [1, 1])
    assert lib.cs_kv_append(ctypes.byref(p), 0, ctypes.byref(b3), q, q, None) == cs.CS_ERR_INVALID_ARG
    b4, keep4 = _batch([5, 6], [1, 1])
    b4.num_tokens = 3                                                       # disagrees with cu_q_lens
    assert lib.cs_kv_append(ctypes.byref(p), 0, ctypes.byref(b4), q, q, None) == cs.CS_ERR_INVALID_ARG
    empty = cs.cs_batch(0, 0, None, 0, None, None, None, None)
    assert lib.cs_kv_append(ctypes.byref(p), 0, ctypes.byref(empty), None, None, None) == cs.CS_OK
    assert lib.cs_paged_attention_mixed(ctypes.byref(p), 0, ctypes.byref(empty), None, None, 4, 0.125, None, 0, None) == cs.CS_OK
    idle, keep5 = _batch([5, 6], [0, 0])
    assert lib.cs_paged_attention_mixed(ctypes.byref(p), 0, ctypes.byref(idle), None, None, 4, 0.125, None, 0, None) == cs.CS_OK


def test_attention_shape_and_workspace_checks():
    lib = cs.lib()
    p = _pool()
    q = 0x5000
    b, keep = _batch([5000, 40000], [1, 1], max_blocks=4096)
    assert lib.cs_paged_attention_mixed(ctypes.byref(p), 0, ctypes.byref(b), q, q, 3, 0.125, None, 0, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_paged_attention_mixed(ctypes.byref(p), 0, ctypes.byref(b), q, q, 64, 0.125, None, 0, None) == cs.CS_ERR_UNSUPPORTED
    assert lib.cs_paged_attention_mixed(ctypes.byref(p), 0, ctypes.byref(b), q, q, 4, 0.0, None, 0, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_paged_attention_mixed(ctypes.byref(p), 0, ctypes.byref(b), q, q, 4, float("nan"), None, 0, None) == cs.CS_ERR_INVALID_ARG
    # these two sequences are cut into several items, so a workspace is needed
    need = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 4, 2, 64)
    assert need > 0
    assert lib.cs_paged_attention_mixed(ctypes.byref(p), 0, ctypes.byref(b), q, q, 4, 0.125, 0x6000, need - 16, None) == cs.CS_ERR_WORKSPACE_TOO_SMALL
    assert lib.cs_paged_attention_mixed(ctypes.byref(p), 0, ctypes.byref(b), q, q, 4, 0.125, None, need, None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 3, 2, 64) == 0
    # the split knob changes the plan and therefore the workspace
    try:
        lib.cs_set_decode_split_tokens(256)
        more = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 4, 2, 64)
        lib.cs_set_decode_split_tokens(1 << 20)
        none_cut = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 4, 2, 64)
    finally:
        lib.cs_set_decode_split_tokens(0)
    assert more >= need > none_cut == 0


def _plan(ctx, ql, Hkv, D, max_blocks=1 << 16):
    """Host-only launch plan of the decode path as (seq, piece, pieces) tuples."""
    lib = cs.lib()
    b, keep = _batch(ctx, ql, max_blocks=max_blocks)
    buf = (ctypes.c_uint32 * 1024)()
    split = ctypes.c_int32(0)
    n = lib.cs_debug_decode_items(ctypes.byref(b), Hkv, D, buf, 1024, ctypes.byref(split))
    items = None if n < 0 else [(w & 0xffff, (w >> 16) & 0xff, w >> 24) for w in buf[:n]]
    return items, n, split.value


def test_decode_plan_lists_every_piece_once_longest_first():
    import random
    rnd = random.Random(7)
    ctx = [rnd.randint(0, 40000) for _ in range(90)]
    ql = [1] * 90
    for s in (3, 17, 50):
        ql[s] = rnd.choice([0, 5, 300])                     # not decode sequences: never listed
    items, n, split = _plan(ctx, ql, 8, 128)
    assert items is not None and n == len(items) and split % 16 == 0 and split >= 256
    decode = [s for s in range(90) if ql[s] == 1]
    by_seq = {}
    for pos, (s, piece, k) in enumerate(items):
        by_seq.setdefault(s, []).append((pos, piece, k))
    assert sorted(by_seq) == decode
    length = []
    for s, lst in by_seq.items():
        k = lst[0][2]
        assert [p for _, p, _ in lst] == list(range(k)) and all(kk == k for _, _, kk in lst)     # each piece once
        assert [pos for pos, _, _ in lst] == list(range(lst[0][0], lst[0][0] + k))              # adjacent
        nkeys = ctx[s] + 1
        assert k == max(1, (nkeys + split // 2) // split)                                       # round(n / split)
        piece_keys = nkeys if k == 1 else (-(-nkeys // k) + 15) // 16 * 16
        assert k * piece_keys >= nkeys                                                          # the pieces cover the keys
        length.append((lst[0][0], piece_keys))
    length.sort()
    assert all(a[1] >= b[1] for a, b in zip(length, length[1:]))                                # longest first


def test_decode_plan_sizes_the_grid_by_the_batch():
    """Workgroups = items x kv heads.  Equal lengths: the fewest pieces that give every CU (256)
    a workgroup.  Uneven lengths: one and a half per CU for small launches, three per CU from about
    0.4 GB of K/V on.  A handful of very long sequences is cut past the sixteen-pieces limit
    until every CU has a workgroup."""
    def wgs(ctx, Hkv, D=128):
        items, n, split = _plan(ctx, [1] * len(ctx), Hkv, D)
        return n * Hkv, split
    assert wgs([4095] * 32, 8) == (256, 4096)                 # 32 x 8 = 256 uncut
    assert wgs([4095] * 48, 8) == (384, 4096)
    assert wgs([2047] * 8, 8) == (256, 512)                   # 8 x 8 x 4 pieces
    assert wgs([4095] * 24, 4) == (384, 1024)                 # 96 workgroups uncut, 192 in halves: quarters
    import random
    rnd = random.Random(11)
    small = [rnd.randint(1024, 8192) for _ in range(24)]      # 0.24 GB at 4 heads
    w, split = wgs(small, 4)
    assert 384 <= w < 768 and split == 1024
    large = [rnd.randint(1024, 8192) for _ in range(64)]      # 0.6 GB
    w, split = wgs(large, 4)
    assert 768 <= w < 1536 and split == 1024
    w, split = wgs([30000, 9000, 25000, 2100], 8)             # a sixteenth of the longest is 2048: 264 workgroups there
    assert split == 2048 and w >= 256
    w, split = wgs([30000, 9000], 8)                          # 152 at 2048: cut finer although that makes 29 pieces
    assert split == 1024 and w >= 256


def test_decode_plan_falls_back_to_the_planning_kernel_beyond_the_argument_block():
    ctx = [100] * 880
    items, n, _ = _plan(ctx, [1] * 880, 2, 64)
    assert n == 880 and [s for s, _, _ in items] == list(range(880))       # equal lengths: stable order
    items, n, _ = _plan(ctx + [100], [1] * 881, 2, 64)
    assert items is None and n == -1000000 - 881
    lib = cs.lib()
    try:
        lib.cs_set_decode_split_tokens(256)
        items, n, split = _plan([70000, 10], [1, 1], 2, 64)                # round(70001/256) = 273 pieces: a word holds 255
        assert items is None and split == 256
        items, n, split = _plan([60000, 10], [1, 1], 2, 64)
        assert n == 234 + 1 and items[-1] == (1, 0, 1) and items[0][2] == 234   # round(60001/256) = 234
    finally:
        lib.cs_set_decode_split_tokens(0)


def test_decode_prefetch_depth_follows_the_launch_volume():
    """Two pages in flight per wavefront from about 0.65 GB of K/V per launch on, one below;
    the knob overrides either way."""
    lib = cs.lib()

    def ahead(ctx, Hkv, D):
        b, keep = _batch(ctx, [1] * len(ctx), max_blocks=1 << 16)
        return lib.cs_debug_decode_pages_ahead(ctypes.byref(b), Hkv, D)

    # 256 sequences x 2304 keys x 8 heads x 128 x 4 bytes = 2.4 GB
    assert ahead([2303] * 256, 8, 128) == 2
    # 64 x 4600 keys x 4 heads: 0.6 GB
    assert ahead([4599] * 64, 4, 128) == 1
    # either side of the threshold: keys * 2 * Hkv * D * 2 bytes against 650e6
    keys_at = -(-650000000 // (2 * 8 * 128 * 2))            # the first key count at or over it
    assert ahead([keys_at - 1], 8, 128) == 2                # ctx + 1 keys = keys_at
    assert ahead([keys_at - 2], 8, 128) == 1
    try:
        lib.cs_set_decode_pages_ahead(1)
        assert ahead([2303] * 256, 8, 128) == 1
        lib.cs_set_decode_pages_ahead(2)
        assert ahead([10], 8, 128) == 2
        lib.cs_set_decode_pages_ahead(7)                    # not a depth: back to automatic
        assert ahead([10], 8, 128) == 1
    finally:
        lib.cs_set_decode_pages_ahead(0)
    b, keep = _batch([5, 5], [3, 4], max_blocks=16)
    assert lib.cs_debug_decode_pages_ahead(ctypes.byref(b), 8, 128) == 1      # no decode sequence
    assert lib.cs_debug_decode_pages_ahead(ctypes.byref(b), 8, 100) == cs.CS_ERR_INVALID_ARG


def test_prefill_key_range_plan_follows_the_rounds():
    """Workspace bytes show the prefill plan: partial results exist only when tiles are cut into
    key ranges.  Few tiles on a long context are cut; a grid of exactly one workgroup per CU
    is cut in two on a long context and left alone on a short one; two workgroups per CU
    (a full round) are never cut; 640 workgroups are cut only when the tiles are long."""
    lib = cs.lib()

    def ranges(Hq, Hkv, P, C):
        b, keep = _batch([C], [P], max_blocks=1 << 16)
        by = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), Hq, Hkv, 128)
        slots = (P * (Hq // Hkv) + 127) // 128 + 1
        return by / (slots * Hkv * 8 * 16 * 132 * 4)

    assert ranges(32, 8, 128, 32768) > 4                 # 32 tile workgroups
    assert 1.9 < ranges(32, 8, 1024, 32768) < 2.1        # 256
    assert 1.9 < ranges(32, 8, 1024, 4096) < 2.1
    assert ranges(32, 8, 1024, 2048) == 0                # ranges would be shorter than 64 steps
    assert ranges(28, 4, 1280, 32768) >= 3               # 280: three or more ranges fill the rounds
    assert ranges(28, 4, 1280, 4096) == 0
    assert ranges(32, 8, 2048, 32768) == 0               # 512: one full round
    assert ranges(28, 4, 2048, 65536) == 0               # 448
    assert 3.9 < ranges(32, 8, 2560, 32768) < 4.1        # 640 -> 2560 = five rounds
    assert ranges(32, 8, 2560, 4096) == 0
    assert ranges(32, 8, 4608, 65536) == 0               # beyond 1024: rounds blur, never cut


def test_prefill_tile_order_gives_the_longest_tiles_a_cu_of_their_own():
    """Four 320-token chunks of very different context at the Qwen-14B shape: 52 tiles per kv
    head on 32 first-round positions.  The order must be a permutation of the tiles, the 12
    positions that keep a CU to themselves must hold the 12 longest, and each shared CU a long
    tile (first round) and a short one (second round) -- the longest of the rest with the
    shortest."""
    lib = cs.lib()
    Hq, Hkv, G = 40, 8, 5
    ctx, ql = [2048, 1000, 3000, 500], [320] * 4
    b, keep = _batch(ctx, ql, max_blocks=1 << 12)
    buf = (ctypes.c_int32 * 512)()
    n = lib.cs_debug_prefill_order(ctypes.byref(b), Hq, Hkv, 128, buf, 512)
    order = list(buf[:n])
    # the tiles and their lengths, as the kernel numbers them: slot start of sequence s is (cu*G/128 + s) ...
    steps = {}
    cu = 0
    for s, (c, q) in enumerate(zip(ctx, ql)):
        start = (cu + 16 * s) * G // 128 + s
        n_ct = (q + 15) // 16 * G
        for j, ct0 in enumerate(range(0, n_ct, 8)):
            tb_max = (min(ct0 + 8, n_ct) - 1) // G
            steps[start + j] = (c + min(q, (tb_max + 1) * 16) + 31) // 32
        cu += q
    assert n == len(steps) == 52 and sorted(order) == sorted(steps)
    first_round = 256 // Hkv
    n_pair = n - first_round
    assert n_pair == 20
    solo = [steps[t] for t in order[n_pair:first_round]]
    rest = sorted((steps[t] for t in order[:n_pair] + order[first_round:]), reverse=True)
    assert min(solo) >= rest[0]
    for k in range(n_pair):
        assert steps[order[k]] == rest[k] and steps[order[first_round + k]] == rest[2 * n_pair - 1 - k]
    # more tiles than workgroup slots: longest first
    b3, keep3 = _batch([0], [4096], max_blocks=1 << 12)
    n3 = lib.cs_debug_prefill_order(ctypes.byref(b3), 32, 8, 128, buf, 512)
    assert n3 == 128 and list(buf[:n3]) == list(range(127, -1, -1))       # one causal chunk: its tiles backwards
    # natural order where no rule applies: tiles cut into key ranges, one workgroup per CU or fewer
    for ctx2, ql2 in (([30000], [1024]), ([100], [256])):
        b2, keep2 = _batch(ctx2, ql2, max_blocks=1 << 12)
        assert lib.cs_debug_prefill_order(ctypes.byref(b2), 32, 8, 128, buf, 512) == 0


def test_debug_copy_argument_checks():
    lib = cs.lib()
    assert lib.cs_debug_copy(0x1000, 0x2000, 24, None) == cs.CS_ERR_INVALID_ARG          # not a multiple of 16
    assert lib.cs_debug_copy(0x1008, 0x2000, 32, None) == cs.CS_ERR_INVALID_ARG          # misaligned
    assert lib.cs_debug_copy(None, None, 0, None) == cs.CS_OK


def test_run_layers_checks_the_workspace_of_both_plans_before_anything_is_enqueued():
    """A preempted iteration runs its remaining layers on the online prefix, whose plan can need
    MORE workspace than the full batch's: fewer decode sequences are cut finer, and a lone long
    chunk is cut into key ranges where many chunks fill the chip uncut.  cs_run_layers must ask
    for the larger of the two and refuse up front, not at the safepoint (host-side checks only:
    the device pointers here are never dereferenced)."""
    lib = cs.lib()
    Hq, Hkv, D = 32, 8, 128
    p = _pool(L=8, P=1 << 20, Hkv=Hkv, D=D)
    x = 0x5000
    first = ctypes.c_int32(7)
    # 512 equal decodes: nothing is cut.  Their first 16 alone: cut into pieces, partials needed.
    b, keep = _batch([4096] * 512, [1] * 512, max_blocks=512)
    full = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), Hq, Hkv, D)
    assert full == 0
    assert lib.cs_run_layers_workspace_bytes(ctypes.byref(b), 0, Hq, Hkv, D) == 0
    assert lib.cs_run_layers_workspace_bytes(ctypes.byref(b), 512, Hq, Hkv, D) == 0
    need = lib.cs_run_layers_workspace_bytes(ctypes.byref(b), 16, Hq, Hkv, D)
    assert need > 0
    sp = cs.cs_safepoint(None, cs.POLL_FN(0), None, 4, 16, 0)
    args = (ctypes.byref(p), 0, 8, ctypes.byref(b), x, x, x, x, 0, 0, Hq, ctypes.c_float(0.1))
    assert lib.cs_run_layers(*args, 0x6000, need - 16, ctypes.byref(sp), ctypes.byref(first), None) == cs.CS_ERR_WORKSPACE_TOO_SMALL
    assert first.value == -1
    assert lib.cs_run_layers(*args, None, 0, ctypes.byref(sp), ctypes.byref(first), None) == cs.CS_ERR_INVALID_ARG
    # one long chunk online-first, 64 short chunks behind it: the prefix alone is cut into key ranges
    b2, keep2 = _batch([8192] + [2048] * 64, [256] + [256] * 64, max_blocks=1024)
    full2 = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b2), Hq, Hkv, D)
    need2 = lib.cs_run_layers_workspace_bytes(ctypes.byref(b2), 1, Hq, Hkv, D)
    assert need2 > full2
    sp2 = cs.cs_safepoint(None, cs.POLL_FN(0), None, 4, 1, 0)
    args2 = (ctypes.byref(p), 0, 8, ctypes.byref(b2), x, x, x, x, 0, 0, Hq, ctypes.c_float(0.1))
    assert lib.cs_run_layers(*args2, 0x6000, need2 - 16, ctypes.byref(sp2), ctypes.byref(first), None) == cs.CS_ERR_WORKSPACE_TOO_SMALL
    # shape and scale are refused before the first layer too
    assert lib.cs_run_layers(ctypes.byref(p), 0, 8, ctypes.byref(b), x, x, x, x, 0, 0, 33, ctypes.c_float(0.1), 0x6000, need,
                             ctypes.byref(sp), ctypes.byref(first), None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_run_layers(*args[:-1], ctypes.c_float(0.0), 0x6000, need, ctypes.byref(sp), ctypes.byref(first), None) == cs.CS_ERR_INVALID_ARG
    assert lib.cs_run_layers_workspace_bytes(ctypes.byref(b), 16, 33, Hkv, D) == 0


def test_plans_scale_with_the_compute_unit_count():
    """The launch plans size their grids by the device's compute-unit count (256 where no device
    answers).  With the count faked, the same batches are planned for a chip half and twice as
    wide: equal decodes are cut until every CU has a workgroup, and a chunk that gives a 256-CU
    chip exactly one tile workgroup per CU (cut in two there) fills a 128-CU chip's slots (left
    alone) and is only half a round on 512 CUs (cut finer)."""
    lib = cs.lib()

    def decode_wgs(ctx, Hkv):
        items, n, split = _plan(ctx, [1] * len(ctx), Hkv, 128)
        return n * Hkv

    def ranges(Hq, Hkv, P, C):
        b, keep = _batch([C], [P], max_blocks=1 << 16)
        by = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), Hq, Hkv, 128)
        slots = (P * (Hq // Hkv) + 127) // 128 + 1
        return by / (slots * Hkv * 8 * 16 * 132 * 4)

    try:
        seen = {}
        for cus in (128, 256, 512):
            lib.cs_debug_set_cu_count(cus)
            seen[cus] = (decode_wgs([4095] * 16, 8), ranges(32, 8, 1024, 32768))
            assert seen[cus][0] >= cus and seen[cus][0] < 2 * cus           # the fewest pieces that give every CU one
        assert seen[128][1] == 0                                            # 256 tiles = both slots of 128 CUs
        assert 1.9 < seen[256][1] < 2.1
        assert seen[512][1] > 2.1
        # the memo of the last plans is keyed by the count too: asking again after a change re-plans
        lib.cs_debug_set_cu_count(128)
        assert ranges(32, 8, 1024, 32768) == 0
    finally:
        lib.cs_debug_set_cu_count(0)
    assert 1.9 < ranges(32, 8, 1024, 32768) < 2.1


def test_workspace_query_is_remembered_but_never_stale():
    """The plan of the last batches is memoised per thread; the key is the VALUES of the host
    length arrays, so reusing a buffer with other lengths re-plans."""
    lib = cs.lib()
    b, keep = _batch([5000, 40000], [1, 1], max_blocks=4096)
    a1 = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 4, 2, 64)
    a2 = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 4, 2, 64)
    assert a1 == a2 > 0
    keep[0][0] = 10
    keep[0][1] = 20                                        # same arrays, other lengths: two short decodes, nothing cut
    assert lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 4, 2, 64) == 0
    keep[0][0] = 5000
    keep[0][1] = 40000
    assert lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 4, 2, 64) == a1
    assert lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 8, 2, 64) > a1     # other shape, other plan


def test_mixed_batches_choose_where_the_decode_work_runs():
    """A batch with both kinds of work runs as one grid with the decode work behind the tiles or
    with a decode workgroup per CU beside them, or as two kernels (Sec. 4.2: online decode tokens
    and offline chunks share an iteration).  The host's choice follows the two sides' weights: a
    decode side as heavy as the chunks goes beside them, a few short decodes stay behind them; one
    kind of work alone is never fused; the knob forces each arrangement."""
    lib = cs.lib()
    import random
    rnd = random.Random(5)

    def arrangement(ctx, ql, Hq, Hkv):
        b, keep = _batch(ctx, ql, max_blocks=1 << 16)
        return lib.cs_debug_mixed_arrangement(ctypes.byref(b), Hq, Hkv, 128)

    long_decodes = [rnd.randint(2048, 32768) for _ in range(128)]
    heavy = (long_decodes + [30720], [1] * 128 + [1024])             # 5 GB of K/V beside a 1024-token chunk on 30K keys
    light = ([rnd.randint(512, 2048) for _ in range(8)] + [5000] * 4, [1] * 8 + [512] * 4)
    try:
        lib.cs_debug_set_cu_count(256)
        assert arrangement(*heavy, 64, 8) == 2
        assert arrangement(*light, 64, 8) == 1
        assert arrangement(long_decodes, [1] * 128, 64, 8) == 0
        assert arrangement([30720], [1024], 64, 8) == 0
        for mode, want in ((0, 0), (2, 1), (3, 2)):
            lib.cs_set_mixed_fusion(mode)
            assert arrangement(*heavy, 64, 8) == want and arrangement(*light, 64, 8) == want
        lib.cs_set_mixed_fusion(1)
        # the choice is part of the remembered plan and follows the knob and the lengths
        assert arrangement(*heavy, 64, 8) == 2
    finally:
        lib.cs_set_mixed_fusion(1)
        lib.cs_debug_set_cu_count(0)
    b, keep = _batch([5], [1])
    assert lib.cs_debug_mixed_arrangement(ctypes.byref(b), 6, 4, 128) == cs.CS_ERR_INVALID_ARG


def test_tile_wavefronts_take_their_issue_priorities_from_the_two_sides_weights():
    """Tiles beside a decode workgroup per CU alternate their issue priority between the halves of
    an iteration; where the host's model has them outlast the decode stream by less than its
    own length, both levels lie above the decode wavefronts' (Sec. 4.2: the two kinds of work of
    an iteration finish together at best).  Behind the tiles the priorities alternate only when the
    decode side is small, and a call that is not fused has none."""
    lib = cs.lib()
    import random
    rnd = random.Random(5)

    def priority(ctx, ql, Hq=64, Hkv=8):
        b, keep = _batch(ctx, ql, max_blocks=1 << 16)
        return lib.cs_debug_mixed_tile_priority(ctypes.byref(b), Hq, Hkv, 128)

    long_decodes = [rnd.randint(2048, 32768) for _ in range(128)]
    try:
        lib.cs_debug_set_cu_count(256)
        # 5 GB of K/V beside a 1024-token chunk on 30K keys: the tiles end about 0.7 of the stream's length after it
        assert priority(long_decodes + [30720], [1] * 128 + [1024]) == 2
        # the same stream beside a small chunk: the stream ends last and is not held up
        assert priority(long_decodes + [4096], [1] * 128 + [256]) == 1
        # a short stream beside long tiles, forced beside them: the tiles mostly share CUs with each other
        lib.cs_set_mixed_fusion(3)
        assert priority([rnd.randint(512, 2048) for _ in range(16)] + [30000], [1] * 16 + [2048]) == 1
        lib.cs_set_mixed_fusion(1)
        # behind the tiles: alternating when the decode side is small, none when the two weigh the same
        assert priority([rnd.randint(512, 2048) for _ in range(8)] + [5000] * 4, [1] * 8 + [512] * 4) == 1
        lib.cs_set_mixed_fusion(2)
        assert priority(long_decodes + [30720], [1] * 128 + [1024]) == 0
        lib.cs_set_mixed_fusion(0)
        assert priority(long_decodes + [30720], [1] * 128 + [1024]) == 0
    finally:
        lib.cs_set_mixed_fusion(1)
        lib.cs_debug_set_cu_count(0)
    b, keep = _batch([5], [1])
    assert lib.cs_debug_mixed_tile_priority(ctypes.byref(b), 6, 4, 128) == cs.CS_ERR_INVALID_ARG


def test_tiles_of_the_last_round_are_cut_beside_a_decode_load():
    """Beside the decode workgroups a CU has one slot for tiles, so 512 equal tile workgroups run
    as two rounds of 256, and the second round starts when the decode side is about done: the host
    cuts exactly those tiles (launch positions 32..63 of 64 at 8 kv heads) in three, and the
    workspace holds partials for the cut tiles only.  The knob forces other cuts or none."""
    lib = cs.lib()
    from paper_2410_01228_amd import synth
    w = synth.config_llama70b_long()          # 128 decodes of 2K..32K keys beside a 1024-token chunk on 30K keys
    b, keep = _batch(w.ctx_lens.tolist(), w.q_lens.tolist(), max_blocks=1 << 16)
    first, ranges = ctypes.c_int32(-1), ctypes.c_int32(-1)

    def cut():
        n = lib.cs_debug_mixed_tail_cut(ctypes.byref(b), 64, 8, 128, ctypes.byref(first), ctypes.byref(ranges))
        return n, first.value, ranges.value

    block = 8 * 16 * 132 * 4                                   # one partial: 128 query rows of 128 + 4 floats
    try:
        lib.cs_debug_set_cu_count(256)
        assert lib.cs_debug_mixed_arrangement(ctypes.byref(b), 64, 8, 128) == 2
        n, f, r = cut()
        assert 64 <= n <= 66 and f == 32 and r == 3
        ws_cut = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 64, 8, 128)
        lib.cs_debug_set_tail_cut(-2, 0)                       # no cut by the model
        assert cut()[1:] == (0, 1)
        ws_whole = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 64, 8, 128)
        assert ws_cut - ws_whole == (n - 32) * 8 * 3 * block
        lib.cs_debug_set_tail_cut(10, 2)
        assert cut()[1:] == (10, 2)
        assert lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), 64, 8, 128) - ws_whole == (n - 10) * 8 * 2 * block
        lib.cs_debug_set_tail_cut(1000, 3)                     # behind the last tile: nothing is cut
        assert cut()[1:] == (n, 1)
        lib.cs_debug_set_tail_cut(-1, 0)
        assert cut()[1:] == (32, 3)
        # behind the tiles nothing of the kind happens
        lib.cs_set_mixed_fusion(2)
        assert cut()[1:] == (0, 1)
    finally:
        lib.cs_set_mixed_fusion(1)
        lib.cs_debug_set_tail_cut(-1, 0)
        lib.cs_debug_set_cu_count(0)


def test_every_cut_the_host_plans_fits_the_workspace_it_asks_for():
    """The tile workgroups trust the launch plan: a cut tile in launch position p writes its range's
    partial into block ((p - first_cut) * kv heads + kv head) * ranges + range of the workspace.
    Over random mixed batches, model shapes, CU counts, arrangements and forced cuts, the positions
    that are cut lie inside the launch and the workspace the host asks for holds every such block
    (Sec. 4.2: chunks of any length beside decode tokens)."""
    lib = cs.lib()
    import random
    rnd = random.Random(20)
    first, ranges = ctypes.c_int32(-1), ctypes.c_int32(-1)
    checked = cuts = 0
    try:
        for trial in range(60):
            Hq, Hkv = rnd.choice(((64, 8), (28, 4), (40, 8), (32, 8)))
            n_pre, n_dec = rnd.randint(1, 6), rnd.randint(1, 200)
            ctx = [rnd.randint(0, 40000) for _ in range(n_pre)] + [rnd.randint(1, 33000) for _ in range(n_dec)]
            ql = [rnd.choice((17, 256, 512, 1024, 2048)) for _ in range(n_pre)] + [1] * n_dec
            order = list(range(len(ctx)))
            rnd.shuffle(order)
            b, keep = _batch([ctx[i] for i in order], [ql[i] for i in order], max_blocks=1 << 16)
            lib.cs_debug_set_cu_count(rnd.choice((8, 64, 256, 304)))
            for mode in (1, 2, 3):
                lib.cs_set_mixed_fusion(mode)
                for knob in ((-1, 0), (rnd.randint(0, 40), rnd.randint(2, 3)), (0, 2), (10 ** 6, 3)):
                    lib.cs_debug_set_tail_cut(*knob)
                    n = lib.cs_debug_mixed_tail_cut(ctypes.byref(b), Hq, Hkv, 128, ctypes.byref(first), ctypes.byref(ranges))
                    ws = lib.cs_paged_attention_workspace_bytes(ctypes.byref(b), Hq, Hkv, 128)
                    assert n >= 1 and 0 <= first.value <= n and 1 <= ranges.value, (trial, mode, knob, n, first.value, ranges.value)
                    assert ws >= 0
                    if ranges.value > 1:
                        blocks = (n - first.value) * Hkv * ranges.value
                        assert blocks > 0 and ws >= blocks * 8 * 16 * 132 * 4, (trial, mode, knob, n, first.value, ranges.value, ws)
                        cuts += 1
                    checked += 1
    finally:
        lib.cs_set_mixed_fusion(1)
        lib.cs_debug_set_tail_cut(-1, 0)
        lib.cs_debug_set_cu_count(0)
    assert checked == 60 * 12 and cuts > 100, (checked, cuts)


def test_slot_model_of_the_fused_grid():
    """The model the host chooses a mixed batch's arrangement by, on cases worked out by hand
    (times in microseconds; a tile alone on its CU takes 0.78 of its paired time, beside a decode
    workgroup 1.1 of it)."""
    play = cs.cs_debug_play_tiles
    close = lambda a, b: abs(a - b) <= 1e-3 * max(1.0, abs(b))
    assert play([], 4) == 0.0
    assert close(play([100.0], 4), 78.0)                              # one tile, a CU to itself
    assert close(play([100.0] * 4, 4), 78.0)                          # one per CU
    assert close(play([100.0] * 8, 4), 100.0)                         # two per CU, paired all the way
    # five tiles on four CUs: CU 0 holds two (paired, 100), the others one each (78)
    assert close(play([100.0] * 5, 4), 100.0)
    # a short partner: 40 us paired, then the long tile is alone: 40 + 60 * 0.78
    assert close(play([100.0, 40.0], 1), 40.0 + 60.0 * 0.78)
    # three tiles on one CU: 100 and 40 paired for 40, then 100' moves in beside the first (60 left, paired):
    # the first ends at 100, the third has 40 left and is alone: 100 + 40 * 0.78
    assert close(play([100.0, 40.0, 100.0], 1), 100.0 + 40.0 * 0.78)
    # beside a decode workgroup that stays 50 us: 50 / 1.1 done, the rest alone at 0.78
    assert close(play([100.0], 1, 50.0), 50.0 + (100.0 - 50.0 / 1.1) * 0.78)
    # ... that outlasts the tile: 110
    assert close(play([100.0], 1, 500.0), 110.0)
    # two tiles, one slot until the decode side leaves at 110: the first ends at 110, the second runs alone
    assert close(play([100.0, 100.0], 1, 110.0), 110.0 + 78.0)
    # the decode side leaves while the first tile runs: the second moves in beside it
    t = play([100.0, 100.0], 1, 55.0)                                   # first: 50 done at 55, 50 left paired -> 105
    assert close(t, 105.0 + 50.0 * 0.78)                                # second: 50 done at 105, 50 left alone
    # work is conserved: never faster than every slot busy at the best rate, never slower than one slot at the worst
    import random
    rnd = random.Random(3)
    for _ in range(50):
        cus = rnd.choice([1, 2, 7, 32])
        work = [rnd.uniform(5, 300) for _ in range(rnd.randint(1, 200))]
        dec = rnd.choice([0.0, rnd.uniform(1, 2000)])
        t = play(work, cus, dec)
        assert t >= max(work) * 0.78 * (1 - 1e-5) and t >= sum(work) / (2 * cus) * 0.78 * (1 - 1e-5)
        assert t <= (dec + sum(work) * 1.1 / cus + max(work) * 1.1) * (1 + 1e-5)
    assert play([1.0], 0) == -1.0 and cs.lib().cs_debug_play_tiles(None, 1, 4, 0.0) == -1.0
