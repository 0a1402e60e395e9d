"""Seeded synthetic workloads for the co-serving attention / KV-cache path.

This module only draws numbers and does bookkeeping: sequence lengths, page permutations,
block tables, lists of pages, and N(0,1) values rounded to bf16.  It contains none of the
method's arithmetic and knows nothing about the byte format inside a page, so both the
GPU path and the CPU oracle can be fed from it.

The five workloads stand in for the paper's serving workloads: model shapes of the served
models (Sec. 6.1), 16-token pages (Sec. 5), context lengths in the span of Table 1, a mix
of online decode tokens and offline chunked-prefill tokens (Sec. 4.2).  Sequences are
ordered online (decode) first, offline after, so that dropping the offline tail of the
arrays is what layer-wise preemption does to a batch (Sec. 4.3).
"""
from dataclasses import dataclass, field
import math
from typing import List, Optional

import torch

PAGE = 16
BASE_SEED = 241001228


@dataclass
class Shape:
    Hq: int
    Hkv: int
    D: int
    L: int = 1
    page_size: int = PAGE          # tokens per page: 16 (the paper's) or 8

    @property
    def G(self):
        return self.Hq // self.Hkv

    @property
    def scale(self):
        return 1.0 / math.sqrt(self.D)

    @property
    def page_elems(self):
        return 2 * self.Hkv * self.page_size * self.D


@dataclass
class Batch:
    """One step's batch description (all CPU int32 tensors)."""
    shape: Shape
    ctx_lens: torch.Tensor          # [S] prior context C_s (tokens already cached)
    q_lens: torch.Tensor            # [S] new tokens this step (1 = decode)
    cu_q_lens: torch.Tensor         # [S+1] prefix sums of q_lens
    block_tables: torch.Tensor      # [S, max_blocks] page ids, -1 where unused
    num_pages: int                  # pages in the pool
    spare_pages: torch.Tensor       # page ids not referenced by any block table
    name: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def S(self):
        return int(self.ctx_lens.numel())

    @property
    def T(self):
        return int(self.cu_q_lens[-1])

    def blocks_needed(self):
        ps = self.shape.page_size
        return (self.ctx_lens + self.q_lens + ps - 1) // ps


def generator(index: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + index)
    return g


def randn_bf16(shape, gen: torch.Generator, device="cpu") -> torch.Tensor:
    """N(0,1) in fp32, rounded to nearest-even bf16."""
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)


def randn_f16(shape, gen: torch.Generator, device="cpu") -> torch.Tensor:
    """N(0,1) in fp32, rounded to nearest-even IEEE half (for the fp16 variant of the path)."""
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.float16)


def uniform_int(lo: int, hi: int, n: int, gen) -> torch.Tensor:
    """Integers uniform in [lo, hi], both ends inclusive."""
    return torch.randint(lo, hi + 1, (n,), generator=gen, dtype=torch.int64).to(torch.int32)


def log_uniform_int(lo: int, hi: int, n: int, gen) -> torch.Tensor:
    """floor(exp(U(ln lo, ln hi))) clipped to [lo, hi]."""
    u = torch.rand((n,), generator=gen, dtype=torch.float64)
    x = torch.exp(math.log(lo) + u * (math.log(hi) - math.log(lo))).floor().to(torch.int64)
    return x.clamp(lo, hi).to(torch.int32)


def make_batch(shape: Shape, ctx_lens, q_lens, gen, num_pages: Optional[int] = None,
               spare: int = 0, name: str = "") -> Batch:
    """Deal one random permutation of the pool's page ids out to the sequences in order."""
    ctx_lens = torch.as_tensor(ctx_lens, dtype=torch.int32)
    q_lens = torch.as_tensor(q_lens, dtype=torch.int32)
    S = ctx_lens.numel()
    ps = shape.page_size
    need = ((ctx_lens + q_lens + ps - 1) // ps).to(torch.int64)
    total = int(need.sum())
    if num_pages is None:
        num_pages = total + spare
    assert num_pages >= total + spare, "pool too small for this batch"
    perm = torch.randperm(num_pages, generator=gen).to(torch.int32)
    max_blocks = max(1, int(need.max()) if S else 1)
    bt = torch.full((max(S, 1), max_blocks), -1, dtype=torch.int32)
    o = 0
    for s in range(S):
        nb = int(need[s])
        bt[s, :nb] = perm[o:o + nb]
        o += nb
    cu = torch.zeros(S + 1, dtype=torch.int32)
    cu[1:] = torch.cumsum(q_lens, 0)
    return Batch(shape, ctx_lens, q_lens, cu, bt[:S] if S else bt[:0], num_pages, perm[o:].clone(), name)


def newly_filled_pages(batch: Batch) -> List[int]:
    """Page ids whose last slot is written this step (a page is checkpointed once it is
    full and therefore immutable; Sec. 4.4 and Sec. 5), in sequence then block order."""
    out = []
    ps = batch.shape.page_size
    for s in range(batch.S):
        c, q = int(batch.ctx_lens[s]), int(batch.q_lens[s])
        for b in range((c + q) // ps):
            last_slot = b * ps + ps - 1
            if c <= last_slot < c + q:
                out.append(int(batch.block_tables[s, b]))
    return out


# --------------------------------------------------------------------------------------
# The five workloads.  `shrink` divides sequence counts and context lengths so the CPU
# oracle can check a whole batch in seconds; shrink=1 is the stated size.
# --------------------------------------------------------------------------------------

def config_tiny(gen=None) -> Batch:
    """Workload 0: 4/2 heads, D 64, pool of 64 pages; 4 decodes (context 17, 40, 63, 100)
    then 2 prefill chunks of 32 tokens (prior context 0 and 48)."""
    gen = gen or generator(0)
    b = make_batch(Shape(4, 2, 64), [17, 40, 63, 100, 0, 48], [1, 1, 1, 1, 32, 32], gen,
                   num_pages=64, name="tiny-mixed")
    b.extra["n_online"] = 4
    return b


def config_llama8b_decode(gen=None, shrink: int = 1, page_size: int = PAGE) -> Batch:
    """Workload 1: 32/8 heads, D 128; 256 decodes, context uniform in [512, 4096]."""
    gen = gen or generator(1)
    S = max(1, 256 // shrink)
    ctx = uniform_int(512 // shrink, 4096 // shrink, S, gen)
    b = make_batch(Shape(32, 8, 128, page_size=page_size), ctx, torch.ones(S, dtype=torch.int32), gen,
                   name="llama3.1-8b-decode256")
    b.extra["n_online"] = S
    return b


def config_qwen7b_mixed(gen=None, shrink: int = 1, page_size: int = PAGE) -> Batch:
    """Workload 2: 28/4 heads, D 128; 64 decodes with context uniform in [1024, 8192] plus
    4 prefill chunks of 512 tokens with prior context uniform in [0, 16384]."""
    gen = gen or generator(2)
    S = max(1, 64 // shrink)
    ctx_d = uniform_int(1024 // shrink, 8192 // shrink, S, gen)
    ctx_p = uniform_int(0, 16384 // shrink, 4, gen)
    chunk = max(16, 512 // shrink)
    b = make_batch(Shape(28, 4, 128, page_size=page_size), torch.cat([ctx_d, ctx_p]),
                   [1] * S + [chunk] * 4, gen, name="qwen2.5-7b-mixed")
    b.extra["n_online"] = S
    return b


def config_llama70b_long(gen=None, shrink: int = 1, page_size: int = PAGE) -> Batch:
    """Workload 3: 64/8 heads, D 128; 128 decodes with context log-uniform in
    [2048, 32768] plus one prefill chunk of 1024 tokens at prior context 30720."""
    gen = gen or generator(3)
    S = max(1, 128 // shrink)
    ctx_d = log_uniform_int(2048 // shrink, 32768 // shrink, S, gen)
    b = make_batch(Shape(64, 8, 128, page_size=page_size), torch.cat([ctx_d, torch.tensor([30720 // shrink], dtype=torch.int32)]),
                   [1] * S + [max(16, 1024 // shrink)], gen, name="llama3.1-70b-long-mixed")
    b.extra["n_online"] = S
    return b


def config_qwen14b_ckpt(gen=None, shrink: int = 1, layers: int = 48) -> Batch:
    """Workload 4: 40/8 heads, D 128, 48 layers; 512 offline requests, each with 1..8 dirty
    pages (its last full pages; the same page ids in every layer, as a page is allocated
    across all layers at once).  64 of them then decode at context 4096 and 4 take a
    256-token prefill chunk at prior context 2048; the remaining requests hold 128 tokens.
    Spare pages for the restore targets are left in the pool."""
    gen = gen or generator(4)
    R = max(8, 512 // shrink)
    n_dec = max(2, 64 // shrink)
    n_pre = 4 if shrink == 1 else 2
    ctx_dec = 4096 // shrink
    ctx_pre = 2048 // shrink
    chunk = max(16, 256 // shrink)
    ctx = [ctx_dec] * n_dec + [ctx_pre] * n_pre + [128] * (R - n_dec - n_pre)
    # the attention pass touches only the first n_dec + n_pre requests; the rest are idle
    # (q_len 0) but own pages, some of which are dirty
    q = [1] * n_dec + [chunk] * n_pre + [0] * (R - n_dec - n_pre)
    dirty_counts = uniform_int(1, 8, R, gen)
    b = make_batch(Shape(40, 8, 128, layers), ctx, q, gen, spare=int(dirty_counts.sum()),
                   name="qwen2.5-14b-ckpt")
    dirty = []
    for s in range(R):
        full = int(b.ctx_lens[s]) // PAGE
        d = min(int(dirty_counts[s]), full)
        dirty.extend(int(x) for x in b.block_tables[s, full - d:full])
    b.extra.update(n_online=n_dec, dirty_pages=dirty, n_active=n_dec + n_pre)
    return b


CONFIGS = [config_tiny, config_llama8b_decode, config_qwen7b_mixed, config_llama70b_long,
           config_qwen14b_ckpt]
