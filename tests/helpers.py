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


# ---------------------------------------------------------------------------------------
# Probe data: inputs on which NO page of a sequence can go missing unseen.
#
# With N(0,1) keys and thousands of them the softmax is flat: one dropped, duplicated or
# swapped 16-key page moves an output by well under the 1e-2 bar.  So a probed sequence gets
# one planted key in EVERY page -- token `probe_token(p)` of page p carries PROBE_GAIN * u_p
# in every kv head, u_p a seeded N(0,1) bf16 vector of its own -- and the queries are aimed:
# a (query row, head) that holds u_p puts (almost) all of its weight on that one key, so its
# output is the V row of that token.  Lose page p, read another page in its place, mask one
# key too many or shift a key range by a page, and that output changes by O(1).
# A decode token has one row of Hq heads, so its pages are probed Hq at a time over several
# attention calls (same pool, same lengths, same launch plan; only q differs).  A chunk has
# q_len * Hq (row, head) pairs, enough to aim at all of its pages in one call.
# ---------------------------------------------------------------------------------------
PROBE_GAIN = 4.0      # a power of two: the planted key is exact in bf16


def probe_vectors(seed: int, n_pages: int, D: int) -> torch.Tensor:
    """u_p for p < n_pages: bf16 [n_pages, D], random directions of squared length D (so that
    every probe's own score, PROBE_GAIN * sqrt(D), stands the same distance above the others')."""
    g = torch.Generator()
    g.manual_seed(77000 + seed)
    u = torch.randn((n_pages, D), generator=g, dtype=torch.float32)
    u = u * (D ** 0.5) / u.norm(dim=1, keepdim=True)
    return u.to(torch.bfloat16)


def probe_tokens(seed: int, n_keys: int, page_size: int = 16) -> np.ndarray:
    """The planted token of every page of a sequence of n_keys keys: int64 [pages]."""
    n_pages = (n_keys + page_size - 1) // page_size
    r = np.random.default_rng(88000 + seed).integers(0, page_size, n_pages)
    first = np.arange(n_pages, dtype=np.int64) * page_size
    room = np.minimum(page_size, n_keys - first)          # the last page may be partly filled
    return first + r % room


def chunk_probe_targets(C: int, q_len: int, Hq: int, tokens: np.ndarray):
    """(row, head) of a chunk that probes each page: distinct pairs, and the row can see the
    planted token (its position C + row is not before it).  Returns int arrays [pages] (row -1:
    more pages than pairs, this page is not probed)."""
    rows = np.full(len(tokens), -1, np.int64)
    heads = np.zeros(len(tokens), np.int64)
    used = set()
    nxt = 0                                               # next (row, head) pair in row-major order
    for p, j in enumerate(tokens):
        lo = max(0, int(j) - C)                           # first row that sees token j
        if nxt < lo * Hq:
            nxt = lo * Hq
        while nxt < q_len * Hq and nxt in used:
            nxt += 1
        if nxt >= q_len * Hq:
            continue
        used.add(nxt)
        rows[p], heads[p] = nxt // Hq, nxt % Hq
        nxt += 1
    return rows, heads


def parity_counts(got: np.ndarray, ref: np.ndarray):
    """(max abs error, relative Frobenius error, number of elements outside
    |g - o| <= ABS_TOL + REL_TOL * |o|); the last is reported for information."""
    d = np.abs(got - ref)
    return float(d.max()), float(np.linalg.norm(got - ref) / np.linalg.norm(ref)), int((d > ABS_TOL + REL_TOL * np.abs(ref)).sum())


def assert_rows_close(got: np.ndarray, ref: np.ndarray, what=""):
    """The parity bar on already-selected rows (float64 arrays of equal shape)."""
    assert np.isfinite(got).all(), what + ": non-finite output"
    err, rel, nfail = parity_counts(got, ref)
    assert err <= ABS_TOL and rel <= REL_TOL, "%s: max abs err %.3e, rel Frobenius err %.3e, %d elements outside the mixed bound" % (what, err, rel, nfail)
    return err, rel, nfail
