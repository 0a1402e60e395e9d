"""The latency model of Sec. 4.2 fitted to timings of this path on the GPU: fit on half of a
(compute tokens, context) grid, judge on the other half.

The paper reports under 4% relative error for whole iterations.  Asked of this path alone:
non-negative coefficients, a held-out error on batches of 150 us and more that stays small
(measured 3.9-4.9% mean and about 14% max; the assertion allows 10% and 35% so that a noisy box does not
fail the suite), and a can_schedule that admits fewer tokens as the context grows."""
import numpy as np
import pytest
import torch

from paper_2410_01228_amd import binding as cs
from paper_2410_01228_amd import synth
from paper_2410_01228_amd.latency_model import fit

pytestmark = pytest.mark.gpu


def time_batches(sh, grid, reps=6):
    pages = max(sum((p + c + 15) // 16 for p, c in batch) for batch in grid)
    pool = cs.Pool.empty(1, pages, sh.Hkv, sh.D)
    pool.tensor.view(-1)[:] = 0.5
    samples = []
    for batch in grid:
        b = synth.make_batch(sh, [c for _, c in batch], [p for p, _ in batch], synth.generator(6), num_pages=pages)
        bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
        q = torch.ones((b.T, sh.Hq, sh.D), dtype=torch.bfloat16, device="cuda")
        kn = torch.ones((b.T, sh.Hkv, sh.D), dtype=torch.bfloat16, device="cuda")
        out = torch.empty_like(q)
        ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)

        def step():
            cs.cs_kv_append(pool, 0, bb, kn, kn)
            cs.cs_paged_attention_mixed(pool, 0, bb, q, out, sh.Hq, sh.scale, ws)

        for _ in range(2):
            step()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(2):                                           # the quieter of two timings
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                step()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) / reps * 1e-3)
        samples.append((batch, best))
    return samples


def test_fit_on_half_the_grid_predicts_the_other_half():
    sh = synth.Shape(32, 8, 128)
    grid = []
    for S in (64, 128, 256):                                         # decode batches
        for C in (2048, 4096, 8192, 16384):
            grid.append([(1, C)] * S)
    for P in (512, 1024, 2048):                                      # one prefill chunk
        for C in (4096, 8192, 16384, 32768):
            grid.append([(P, C)])
    for P, C, S, Cd in ((512, 8192, 64, 4096), (1024, 16384, 128, 4096), (2048, 8192, 32, 8192), (1024, 4096, 256, 2048)):
        grid.append([(1, Cd)] * S + [(P, C)])                        # mixed
    samples = time_batches(sh, grid)
    train, held = samples[0::2], samples[1::2]
    m, rel_train = fit(train)
    assert m.coef.min() >= 0, "negative coefficient: %r" % (m,)
    assert m.k2 > 0 and m.k4 > 0, "the attention and memory terms must both be identified: %r" % (m,)
    rel = np.array([abs(m.predict(b) - t) / t for b, t in held])
    big = np.array([t >= 150e-6 for _, t in held])
    assert big.sum() >= 8
    print("  latency model: k_token %.2e k2 %.2e k4 %.2e k5 %.2e; held-out batches of 150 us and more: mean %.1f%% max %.1f%%; "
          "all held-out: mean %.1f%% max %.1f%%" % (m.k_p, m.k2, m.k4, m.k5, 100 * rel[big].mean(), 100 * rel[big].max(),
                                                    100 * rel.mean(), 100 * rel.max()))
    assert rel[big].mean() <= 0.10 and rel[big].max() <= 0.35, (rel[big].mean(), rel[big].max())
    # what the model says in hardware terms: a (query, key) pair of this shape is 4*Hq*D flop, a cached token 2*Hkv*D*2 bytes
    tflops = 4 * sh.Hq * sh.D / m.k2 / 1e12
    tbps = 2 * sh.Hkv * sh.D * 2 / (m.k2 + m.k4) / 1e12
    assert 500 < tflops < 2500 and 3.0 < tbps < 8.0, (tflops, tbps)
    # can_schedule: more context, fewer tokens; nothing fits a budget below the constant
    batch = [(1, 4096)] * 64
    fits = [m.can_schedule(batch, 2048, ctx, 6e-4) for ctx in (0, 8192, 32768)]
    assert fits[0] >= fits[1] >= fits[2] and fits[0] > fits[2] > 0, fits
    assert m.can_schedule(batch, 2048, 0, 1e-6) == 0
