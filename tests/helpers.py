"""Shared test plumbing: build a paged pool on the CPU with the ORACLE's format code, run a
step through the HIP library, and compare with the oracle on the logical sequences."""
import numpy as np
import torch

from oracle import attention, kv_layout
from paper_2410_01228_amd import synth

NAN_BITS = 0x7FC0          # bf16 quiet NaN: what never-written slots hold in these tests
ABS_TOL = 2e-2             # max |gpu - oracle| per element (bf16 attention output)
REL_TOL = 1e-2             # ||gpu - oracle||_F / ||oracle||_F per output tensor


def bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def from_bits(a: np.ndarray, device="cpu", dtype=torch.bfloat16) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(dtype).to(device)


class Step:
    """Logical data of one step of a synth.Batch: prior context K/V per sequence, this
    step's new K/V and queries (all bf16 bit patterns / float32 views)."""

    def __init__(self, batch: synth.Batch, seed_index: int, q_gain: float = 1.0, layer: int = 0,
                 dtype=torch.bfloat16):
        self.b = batch
        self.dtype = dtype
        sh = batch.shape
        g = synth.generator(seed_index)
        C = int(batch.ctx_lens.sum())
        draw = synth.randn_bf16 if dtype == torch.bfloat16 else synth.randn_f16
        self.k_prior = draw((C, sh.Hkv, sh.D), g)
        self.v_prior = draw((C, sh.Hkv, sh.D), g)
        self.k_new = draw((batch.T, sh.Hkv, sh.D), g)
        self.v_new = draw((batch.T, sh.Hkv, sh.D), g)
        self.q = (draw((batch.T, sh.Hq, sh.D), g).float() * q_gain).to(dtype)
        self.layer = layer
        self.cu_ctx = torch.zeros(batch.S + 1, dtype=torch.int32)
        self.cu_ctx[1:] = torch.cumsum(batch.ctx_lens, 0)

    def prior_pool(self, L=None, fill=NAN_BITS) -> np.ndarray:
        """CPU pool holding only the prior context (written with the oracle's append)."""
        b, sh = self.b, self.b.shape
        pool = kv_layout.new_pool(L or sh.L, b.num_pages, sh.Hkv, sh.D, fill, page_size=sh.page_size)
        kv_layout.ref_append(pool, self.layer, b.block_tables.numpy(), np.zeros(b.S, np.int32),
                             self.cu_ctx.numpy(), bits(self.k_prior), bits(self.v_prior), page_size=sh.page_size)
        return pool

    def oracle_append(self, pool: np.ndarray) -> np.ndarray:
        b = self.b
        return kv_layout.ref_append(pool, self.layer, b.block_tables.numpy(), b.ctx_lens.numpy(),
                                    b.cu_q_lens.numpy(), bits(self.k_new), bits(self.v_new),
                                    page_size=b.shape.page_size)

    def logical(self, s: int):
        """float32 logical K, V of sequence s including this step's tokens."""
        b = self.b
        c0, c1 = int(self.cu_ctx[s]), int(self.cu_ctx[s + 1])
        t0, t1 = int(b.cu_q_lens[s]), int(b.cu_q_lens[s + 1])
        K = torch.cat([self.k_prior[c0:c1], self.k_new[t0:t1]]).float().numpy()
        V = torch.cat([self.v_prior[c0:c1], self.v_new[t0:t1]]).float().numpy()
        return K, V

    def oracle_attention(self, seqs=None) -> np.ndarray:
        """float64 [T, Hq, D]; rows of sequences not in `seqs` are NaN."""
        b, sh = self.b, self.b.shape
        out = np.full((b.T, sh.Hq, sh.D), np.nan)
        qf = self.q.float().numpy()
        for s in (range(b.S) if seqs is None else seqs):
            t0, t1 = int(b.cu_q_lens[s]), int(b.cu_q_lens[s + 1])
            if t1 > t0:
                K, V = self.logical(s)
                out[t0:t1] = attention.attention_chunk(qf[t0:t1], K, V, int(b.ctx_lens[s]), sh.scale)
        return out


def assert_attention_close(gpu_out: torch.Tensor, ref: np.ndarray, what=""):
    """The parity bar: max abs error <= 2e-2 AND relative Frobenius error <= 1e-2."""
    g = gpu_out.detach().float().cpu().numpy().astype(np.float64)
    rows = ~np.isnan(ref).any(axis=(1, 2))
    assert rows.any()
    g, r = g[rows], ref[rows]
    assert np.isfinite(g).all(), what + ": non-finite output"
    err = np.abs(g - r).max()
    rel = np.linalg.norm(g - r) / np.linalg.norm(r)
    assert err <= ABS_TOL and rel <= REL_TOL, "%s: max abs err %.3e, rel Frobenius err %.3e" % (what, err, rel)
    return err, rel
