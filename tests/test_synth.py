"""The synthetic workloads have the stated shapes and are reproducible."""
import torch

from paper_2410_01228_amd import synth


def _check_tables(b):
    need = b.blocks_needed()
    used = []
    for s in range(b.S):
        row = b.block_tables[s]
        assert (row[:int(need[s])] >= 0).all() and (row[int(need[s]):] == -1).all()
        used += row[:int(need[s])].tolist()
    assert len(used) == len(set(used)), "a page belongs to one request"
    assert set(used).isdisjoint(set(b.spare_pages.tolist()))
    assert len(used) + b.spare_pages.numel() == b.num_pages
    assert b.cu_q_lens[-1] == b.q_lens.sum()


def test_tiny():
    b = synth.config_tiny()
    assert (b.shape.Hq, b.shape.Hkv, b.shape.D, b.num_pages, b.T, b.S) == (4, 2, 64, 64, 68, 6)
    assert b.ctx_lens.tolist() == [17, 40, 63, 100, 0, 48] and b.q_lens.tolist() == [1, 1, 1, 1, 32, 32]
    _check_tables(b)
    assert torch.equal(b.block_tables, synth.config_tiny().block_tables)


def test_full_size_recipes():
    b = synth.config_llama8b_decode()
    assert b.S == 256 and b.T == 256 and 512 <= int(b.ctx_lens.min()) and int(b.ctx_lens.max()) <= 4096
    _check_tables(b)
    b = synth.config_qwen7b_mixed()
    assert b.T == 64 + 2048 and b.q_lens[:64].eq(1).all() and b.q_lens[64:].tolist() == [512] * 4
    assert int(b.ctx_lens[:64].min()) >= 1024 and int(b.ctx_lens[:64].max()) <= 8192
    assert int(b.ctx_lens[64:].max()) <= 16384 and b.T <= 4096
    b = synth.config_llama70b_long()
    assert b.T == 128 + 1024 and int(b.ctx_lens[-1]) == 30720
    assert int(b.ctx_lens[:128].min()) >= 2048 and int(b.ctx_lens[:128].max()) <= 32768
    b = synth.config_qwen14b_ckpt()
    assert b.S == 512 and b.shape.L == 48 and b.T == 64 + 1024
    d = b.extra["dirty_pages"]
    assert 512 <= len(d) <= 8 * 512 and len(set(d)) == len(d) and b.spare_pages.numel() >= len(d)
    assert b.ctx_lens[:64].eq(4096).all()


def test_shrunk_variants_keep_structure():
    for f in synth.CONFIGS[1:]:
        b = f(shrink=16)
        _check_tables(b)
        assert b.T > 0
