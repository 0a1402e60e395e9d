#!/usr/bin/env python3
"""Benchmark of the co-serving attention / KV hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--only] [--detail]

One "step" is one pass of the per-layer hot path over one synthetic batch: cs_kv_append of
the step's new K/V followed by cs_paged_attention_mixed (for the checkpoint workload also
cs_kv_ckpt_gather + cs_kv_ckpt_restore over all layers).  Inputs are resident in HBM before
the timed region.  Prints ONE JSON line on stdout; everything else goes to stderr.

The default workload is the largest single-GPU mixed batch: the Llama-3.1-70B long-context
step (128 decodes on contexts log-uniform in [2048, 32768] plus one 1024-token chunk on
30720 keys; 64/8 heads, head dim 128, 16-token pages).  Its decode-only and prefill-only
sub-batches are timed as legs of their own, so the line carries the decode path's HBM
fraction and the prefill path's matrix-core fraction beside the whole call; the key
`workloads` holds the legs of the other four workloads from the same run.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12            # B/s, MI355X HBM3E
MFMA_BF16_PEAK = 2.5e15      # FLOP/s, dense bf16

WORKLOADS = ["tiny", "llama8b_decode", "qwen7b_mixed", "llama70b_long", "qwen14b_ckpt"]
# the kernel behind the call a roofline line is quoted for: the start of its name as the profiler
# prints it (the remaining template arguments -- prefetch depth, issue priorities, page size --
# follow from the launch plan) and a note
_ONE_GRID = "prefill tiles and decode work items in one grid"
KERNEL_OF = {("llama8b_decode", "paged_attention_mixed"): ("cs::decode_split_kernel<128, cs::ItemsInArgs, cs::Bf16,", "the call's only kernel here"),
             ("qwen14b_ckpt", "ckpt_gather"): ("cs::page_copy_kernel<true>", ""),
             ("qwen14b_ckpt", "ckpt_restore"): ("cs::page_copy_kernel<false>", ""),
             ("qwen7b_mixed", "decode_only"): ("cs::decode_split_kernel<128, cs::ItemsInArgs, cs::Bf16,", ""),
             ("llama70b_long", "decode_only"): ("cs::decode_split_kernel<128, cs::ItemsInArgs, cs::Bf16,", ""),
             ("qwen7b_mixed", "paged_attention_mixed"): ("cs::mixed_kernel<128, cs::Bf16,", _ONE_GRID),
             ("llama70b_long", "paged_attention_mixed"): ("cs::mixed_kernel<128, cs::Bf16,", _ONE_GRID),
             ("qwen14b_ckpt", "paged_attention_mixed"): ("cs::mixed_kernel<128, cs::Bf16,", _ONE_GRID),
             ("tiny", "paged_attention_mixed"): ("cs::mixed_kernel<64, cs::Bf16,", _ONE_GRID),
             ("qwen7b_mixed", "prefill_only"): ("cs::prefill_kernel<128, cs::Bf16,", ""),
             ("llama70b_long", "prefill_only"): ("cs::prefill_kernel<128, cs::Bf16,", "")}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def fill_randn_bf16(t, gen, dtype=None):
    """N(0,1) rounded to bf16 (or to `dtype`, stored bit for bit), written in place in chunks
    (t is a flat bf16 device tensor)."""
    import torch
    step = 1 << 27
    for o in range(0, t.numel(), step):
        n = min(step, t.numel() - o)
        r = torch.randn(n, generator=gen, device=t.device, dtype=torch.float32)
        t[o:o + n] = r.to(torch.bfloat16) if dtype in (None, torch.bfloat16) else r.to(dtype).view(torch.bfloat16)


class Leg:
    """One timed call of the step with its algorithmic work."""

    def __init__(self, name, fn, bound, work, also=None):
        """bound / work: the roofline the call is priced against and its algorithmic work (bytes
        for "hbm", flops for "mfma").  also: (bound, work) of the other kind of work the same
        launch does (the fused grid of a mixed batch reads the decode sequences' K/V AND multiplies
        the chunks' tiles); it is reported beside the main figure."""
        self.name, self.fn, self.bound, self.work, self.also = name, fn, bound, work, also
        self.us = self.us_median = self.us_min = None

    def also_record(self):
        bound, work = self.also
        peak = HBM_PEAK if bound == "hbm" else MFMA_BF16_PEAK
        ach = work / (self.us * 1e-6)
        return {"bound": bound, "achieved": round(ach / (1e9 if bound == "hbm" else 1e12), 2),
                "unit": "GB/s" if bound == "hbm" else "TFLOP/s", "frac": round(ach / peak, 4), "work": work}

    def roofline(self, traffic=None):
        peak = HBM_PEAK if self.bound == "hbm" else MFMA_BF16_PEAK
        ach = self.work / (self.us * 1e-6)
        if self.bound == "hbm":
            return {"bound": "hbm", "achieved": round(ach / 1e9, 1), "peak": peak / 1e9, "unit": "GB/s",
                    "frac": round(ach / peak, 4), "traffic": traffic}
        return {"bound": "mfma", "achieved": round(ach / 1e12, 2), "peak": peak / 1e12, "unit": "TFLOP/s",
                "frac": round(ach / peak, 4), "traffic": traffic}


def attention_work(b, seqs=None):
    """Algorithmic bytes of the decode sequences and flops of the prefill chunks."""
    sh = b.shape
    dec_bytes = pre_flops = pre_bytes = 0
    for s in (range(b.S) if seqs is None else seqs):
        c, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
        if ql == 1:
            n = c + 1
            dec_bytes += n * 2 * sh.Hkv * sh.D * 2 + 2 * sh.Hq * sh.D * 2 + 4 * ((n + sh.page_size - 1) // sh.page_size)
        elif ql > 1:
            pre_flops += 4 * sh.Hq * sh.D * (ql * c + ql * (ql + 1) // 2)
            pre_bytes += (c + ql) * 2 * sh.Hkv * sh.D * 2 + 2 * ql * sh.Hq * sh.D * 2
    return dec_bytes, pre_flops, pre_bytes


def build(name, f16=False, page_size=16):
    """Allocate and fill the workload on the GPU; returns (batch, legs, dominant leg name, info).
    f16: the pool and the queries hold IEEE half and the fp16 attention entry point is timed.
    page_size: tokens per page of the pool (8: the three model-shaped attention workloads only)."""
    import torch
    from paper_2410_01228_amd import binding as cs
    from paper_2410_01228_amd import synth
    edt = torch.float16 if f16 else torch.bfloat16
    attend = cs.cs_paged_attention_mixed_f16 if f16 else cs.cs_paged_attention_mixed

    idx = WORKLOADS.index(name)
    b = synth.CONFIGS[idx]() if page_size == 16 else synth.CONFIGS[idx](page_size=page_size)
    sh = b.shape
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + idx)
    pool = cs.Pool.empty(sh.L, b.num_pages, sh.Hkv, sh.D, page_size=sh.page_size)
    fill_randn_bf16(pool.tensor.view(-1), gen, edt)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    T = b.T
    draw = synth.randn_f16 if f16 else synth.randn_bf16
    q = draw((T, sh.Hq, sh.D), gen, "cuda")
    k_new = draw((T, sh.Hkv, sh.D), gen, "cuda")
    v_new = draw((T, sh.Hkv, sh.D), gen, "cuda")
    out = torch.empty_like(q)
    ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
    keep = [pool, bb, q, k_new, v_new, out, ws]
    dec_bytes, pre_flops, pre_bytes = attention_work(b)
    append_bytes = 2 * T * 2 * sh.Hkv * sh.D * 2
    layer = [0]

    legs = []
    if name == "qwen14b_ckpt":
        dirty = torch.tensor(b.extra["dirty_pages"], dtype=torch.int32, device="cuda")
        fresh = b.spare_pages[:dirty.numel()].to("cuda")
        staging = torch.empty((sh.L, dirty.numel(), sh.page_elems), dtype=torch.bfloat16, device="cuda")
        keep += [dirty, fresh, staging]
        cp_bytes = 2 * sh.L * dirty.numel() * sh.page_elems * 2
        legs.append(Leg("ckpt_gather", lambda: cs.cs_kv_ckpt_gather(pool, 0, sh.L, dirty, staging), "hbm", cp_bytes))
        legs.append(Leg("ckpt_restore", lambda: cs.cs_kv_ckpt_restore(pool, 0, sh.L, fresh, staging), "hbm", cp_bytes))
    legs.append(Leg("kv_append", lambda: cs.cs_kv_append(pool, layer[0], bb, k_new, v_new), "hbm", append_bytes))
    # the attention call is priced against the roofline its larger ideal time belongs to; in a mixed
    # batch the bytes of the decode side also include the K/V the chunks must read once
    att_bound = "hbm" if pre_flops / MFMA_BF16_PEAK < dec_bytes / HBM_PEAK else "mfma"
    att_bytes = dec_bytes + pre_bytes
    also = None
    if dec_bytes and pre_flops:
        also = ("mfma", pre_flops) if att_bound == "hbm" else ("hbm", att_bytes)
    legs.append(Leg("paged_attention_mixed",
                    lambda: attend(pool, layer[0], bb, q, out, sh.Hq, sh.scale, ws),
                    att_bound, att_bytes if att_bound == "hbm" else pre_flops, also))

    detail = []
    n_on = b.extra.get("n_online", 0)
    n_act = b.extra.get("n_active", b.S)
    if 0 < n_on < n_act:
        # the two paths on their own sub-batches (for per-path roofline fractions)
        bb_dec = bb.truncated(n_on)
        ws_dec = cs.workspace_for(bb_dec, sh.Hq, sh.Hkv, sh.D)
        cu = b.cu_q_lens[n_on:n_act + 1] - b.cu_q_lens[n_on]
        bb_pre = cs.Batch(b.block_tables[n_on:n_act], b.ctx_lens[n_on:n_act], cu)
        T_on = int(b.cu_q_lens[n_on])
        q_pre, out_pre = q[T_on:], out[T_on:]
        ws_pre = cs.workspace_for(bb_pre, sh.Hq, sh.Hkv, sh.D)
        keep += [bb_dec, ws_dec, bb_pre, q_pre, out_pre, ws_pre]
        detail.append(Leg("decode_only", lambda: attend(pool, layer[0], bb_dec, q, out, sh.Hq, sh.scale, ws_dec),
                          "hbm", dec_bytes))
        detail.append(Leg("prefill_only", lambda: attend(pool, layer[0], bb_pre, q_pre, out_pre, sh.Hq, sh.scale, ws_pre),
                          "mfma", pre_flops))
    info = {"T": T, "S": b.S, "dec_bytes": dec_bytes, "pre_flops": pre_flops, "pre_bytes": pre_bytes,
            "append_bytes": append_bytes, "pool_gb": pool.tensor.numel() * 2 / 1e9, "name": b.name,
            "keep": keep, "layer": layer, "L": sh.L,
            # how the host launches this batch's attention call (only a batch with both kinds of work is fused)
            "arrangement": ("two kernels (one kind of work, or fusion off)", "one grid, decode work behind the tiles",
                            "one grid, a decode workgroup per CU beside the tiles")[
                                cs.cs_debug_mixed_arrangement(bb, sh.Hq, sh.Hkv, sh.D)]}
    return b, legs, detail, info


def time_legs(legs, steps, warmup):
    """W untimed steps, then K timed steps bracketed by synchronisation; HIP events on the
    launch stream around every call give the per-call durations."""
    import torch
    for _ in range(warmup):
        for leg in legs:
            leg.fn()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(legs) + 1)] for _ in range(steps)]
    t0 = time.perf_counter()
    for k in range(steps):
        for i, leg in enumerate(legs):
            ev[k][i].record()
            leg.fn()
        ev[k][len(legs)].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for i, leg in enumerate(legs):
        per_call = sorted(ev[k][i].elapsed_time(ev[k][i + 1]) * 1e3 for k in range(steps))
        leg.us = sum(per_call) / steps
        leg.us_median = per_call[steps // 2]
        leg.us_min = per_call[0]
    return wall / steps


def cpu_baseline(b, min_seconds=10.0, max_seconds=30.0):
    """The oracle as it stands, timed on this host on a bounded sample of the workload's
    sequences (inputs regenerated on the CPU with the same recipe; generation is not timed).
    The sample is swept repeatedly until about 10 s of oracle time has accumulated."""
    import torch
    from oracle import attention
    from paper_2410_01228_amd import synth
    sh = b.shape
    order = [s for s in range(b.S) if int(b.q_lens[s]) > 0]
    threads = attention.num_threads()
    # bound the sample by memory (fp32 K and V of the picked sequences <= ~1.5 GB) and by a
    # rough cost model of the plain loops (4*Hq*D flop per (query, key) pair, ~0.5 GFLOP/s/thread)
    budget_flop = max_seconds * 0.5e9 * threads
    budget_bytes = 1.5e9
    stride = max(1, len(order) // 32)
    pick, cost, mem = [], 0.0, 0.0
    for s in order[::stride]:
        c, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
        w = 4.0 * sh.Hq * sh.D * (ql * c + ql * (ql + 1) / 2)
        m = 2.0 * (c + ql) * sh.Hkv * sh.D * 4
        if pick and (cost + w > budget_flop or mem + m > budget_bytes):
            continue
        pick.append(s)
        cost += w
        mem += m
    g = synth.generator(99)
    data = []
    for s in pick:
        c, ql = int(b.ctx_lens[s]), int(b.q_lens[s])
        K = synth.randn_bf16((c + ql, sh.Hkv, sh.D), g).float().numpy()
        V = synth.randn_bf16((c + ql, sh.Hkv, sh.D), g).float().numpy()
        Q = synth.randn_bf16((ql, sh.Hq, sh.D), g).float().numpy()
        data.append((Q, K, V, c, ql))
    tokens, secs, sweeps = 0, 0.0, 0
    while secs < min_seconds and sweeps < 1000:
        for Q, K, V, c, ql in data:
            t0 = time.perf_counter()
            attention.attention_chunk(Q, K, V, c, sh.scale)
            secs += time.perf_counter() - t0
            tokens += ql
        sweeps += 1
    return {"value": round(tokens / secs, 1), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d sequences (%d tokens a sweep) of the same workload, fp64 logical attention, "
                      "%d sweeps, %.1f s" % (len(pick), len(order), sum(d[4] for d in data), sweeps, secs)}


def cpu_copy_baseline(b, layers=2, max_pages=256, min_seconds=3.0):
    """The oracle's checkpoint gather and restore (plain bit copies over its own pool format) on a
    bounded sample of the workload's dirty pages, in GB/s read+write."""
    import numpy as np
    from oracle import kv_layout
    sh = b.shape
    ids = np.asarray(b.extra["dirty_pages"][:max_pages], dtype=np.int64)
    uniq = {int(p): i for i, p in enumerate(sorted(set(int(p) for p in ids)))}
    pool = np.random.default_rng(5).integers(0, 2 ** 16, size=(layers, len(uniq), 2, sh.Hkv, 16 * sh.D), dtype=np.uint16)
    local = [uniq[int(p)] for p in ids]
    nbytes = 2 * layers * len(local) * kv_layout.page_elems(sh.Hkv, sh.D) * 2
    out = {}
    for name, fn in (("gather", lambda st: kv_layout.ref_gather(pool, 0, layers, local)),
                     ("restore", lambda st: kv_layout.ref_restore(pool, 0, layers, sorted(set(local)), st))):
        st = kv_layout.ref_gather(pool, 0, layers, sorted(set(local))) if name == "restore" else None
        if name == "restore":
            nb = 2 * layers * len(set(local)) * kv_layout.page_elems(sh.Hkv, sh.D) * 2
        else:
            nb = nbytes
        secs, reps = 0.0, 0
        while secs < min_seconds and reps < 1000:
            t0 = time.perf_counter()
            fn(st)
            secs += time.perf_counter() - t0
            reps += 1
        out[name] = round(nb * reps / secs / 1e9, 2)
    return {"gather_GBps": out["gather"], "restore_GBps": out["restore"], "cores": 1, "kind": "oracle",
            "sample": "%d of %d dirty pages x %d of %d layers, read+write bytes" % (len(local), len(b.extra["dirty_pages"]), layers, sh.L)}


def checkpoint_pipeline(info, layers=8, reps=5):
    """The asynchronous checkpoint pipeline (gather + one device-to-host copy on its own
    stream) alone and concurrent with the attention call: host-link rate and interference."""
    import torch
    from paper_2410_01228_amd import binding as cs
    pool, bb, q, k_new, v_new, out, ws = info["keep"][:7]
    dirty, fresh, staging = info["keep"][7:10]
    sh_Hq, scale = q.shape[1], 1.0 / (q.shape[2] ** 0.5)
    n = dirty.numel()
    stage = staging[:layers]
    host = torch.empty((layers, n, staging.shape[2]), dtype=torch.bfloat16).pin_memory()
    nbytes = host.numel() * 2
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()

    def attn():
        cs.cs_paged_attention_mixed(pool, 0, bb, q, out, sh_Hq, scale, ws)

    def timed(stream, fn, n_rep):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n_rep):
            fn()
        e1.record(stream)
        return e0, e1

    for _ in range(2):
        cs.cs_kv_ckpt_save(pool, 0, layers, dirty, stage, host, stream=side)
        attn()
    torch.cuda.synchronize()
    a0, a1 = timed(main, attn, 50)
    torch.cuda.synchronize()
    attn_alone = a0.elapsed_time(a1) / 50 * 1e3
    s0, s1 = timed(side, lambda: cs.cs_kv_ckpt_save(pool, 0, layers, dirty, stage, host, stream=side), reps)
    torch.cuda.synchronize()
    save_alone = s0.elapsed_time(s1) / reps * 1e3
    # concurrent: keep attention running on the compute stream for as long as the saves take
    n_attn = max(50, int(reps * save_alone / attn_alone * 1.2))
    s0, s1 = timed(side, lambda: cs.cs_kv_ckpt_save(pool, 0, layers, dirty, stage, host, stream=side), reps)
    a0, a1 = timed(main, attn, n_attn)
    torch.cuda.synchronize()
    save_busy = s0.elapsed_time(s1) / reps * 1e3
    attn_busy = a0.elapsed_time(a1) / n_attn * 1e3
    l0, l1 = timed(side, lambda: cs.cs_kv_ckpt_load(pool, 0, layers, fresh, stage, host, stream=side), reps)
    torch.cuda.synchronize()
    load_alone = l0.elapsed_time(l1) / reps * 1e3
    # the paper's own example (Sec. 4.4): one whole 2048-token chunk = 128 pages of every layer
    L_all = staging.shape[0]
    chunk_pages = min(128, n)
    chunk_ids = dirty[:chunk_pages].contiguous()
    chunk_stage = staging.view(-1)[:L_all * chunk_pages * staging.shape[2]].view(L_all, chunk_pages, staging.shape[2])
    chunk_host = torch.empty((L_all, chunk_pages, staging.shape[2]), dtype=torch.bfloat16).pin_memory()
    cs.cs_kv_ckpt_save(pool, 0, L_all, chunk_ids, chunk_stage, chunk_host, stream=side)
    c0, c1 = timed(side, lambda: cs.cs_kv_ckpt_save(pool, 0, L_all, chunk_ids, chunk_stage, chunk_host, stream=side), reps)
    torch.cuda.synchronize()
    chunk_ms = c0.elapsed_time(c1) / reps
    chunk_bytes = chunk_host.numel() * 2
    # the same chunk into the host page store ([host page][layer][page bytes], page-major staging)
    store_t = torch.empty((chunk_pages, L_all, staging.shape[2]), dtype=torch.bfloat16).pin_memory()
    store = cs.HostStore(store_t)
    cs.cs_kv_ckpt_save_run(pool, 0, L_all, chunk_ids, chunk_stage, store, 0, stream=side)
    p0, p1 = timed(side, lambda: cs.cs_kv_ckpt_save_run(pool, 0, L_all, chunk_ids, chunk_stage, store, 0, stream=side), reps)
    torch.cuda.synchronize()
    store_ms = p0.elapsed_time(p1) / reps
    r = {"layers": layers, "pages": n, "bytes": nbytes,
         "chunk_2048_tokens_page_store": {"save_ms": round(store_ms, 2), "GBps": round(chunk_bytes / store_ms / 1e6, 1)},
         "chunk_2048_tokens": {"layers": L_all, "pages": chunk_pages, "bytes": chunk_bytes, "save_ms": round(chunk_ms, 2),
                               "GBps": round(chunk_bytes / chunk_ms / 1e6, 1)},
         "save_us": round(save_alone, 1), "save_GBps": round(nbytes / save_alone / 1e3, 1),
         "load_us": round(load_alone, 1), "load_GBps": round(nbytes / load_alone / 1e3, 1),
         "save_us_during_attention": round(save_busy, 1), "save_GBps_during_attention": round(nbytes / save_busy / 1e3, 1),
         "attention_us_alone": round(attn_alone, 1), "attention_us_during_save": round(attn_busy, 1)}
    log("  checkpoint pipeline (%d layers, %d pages, %.2f GB): save %.0f us = %.1f GB/s host link, load %.0f us = %.1f GB/s; "
        "with attention running: save %.1f GB/s, attention %.1f -> %.1f us"
        % (layers, n, nbytes / 1e9, save_alone, r["save_GBps"], load_alone, r["load_GBps"],
           r["save_GBps_during_attention"], attn_alone, attn_busy))
    log("  one 2048-token chunk of all %d layers (%d pages, %.0f MB): saved to the host in %.2f ms (%.2f ms as a run of the host page store)"
        % (L_all, chunk_pages, chunk_bytes / 1e6, chunk_ms, store_ms))
    return r


def graph_replay(b, layers=32, iters=20):
    """A launch-bound batch: `layers` layers of append + attention issued call by call, and the
    same calls recorded once into a HIP graph and replayed."""
    import torch
    from paper_2410_01228_amd import binding as cs
    from paper_2410_01228_amd import synth
    sh = b.shape
    gen = torch.Generator(device="cuda")
    gen.manual_seed(78)
    pool = cs.Pool.empty(layers, b.num_pages, sh.Hkv, sh.D)
    fill_randn_bf16(pool.tensor.view(-1), gen)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
    q = synth.randn_bf16((layers, b.T, sh.Hq, sh.D), gen, "cuda")
    kn = synth.randn_bf16((layers, b.T, sh.Hkv, sh.D), gen, "cuda")
    vn = synth.randn_bf16((layers, b.T, sh.Hkv, sh.D), gen, "cuda")
    out = torch.empty_like(q)

    def run():
        for l in range(layers):
            cs.cs_kv_append(pool, l, bb, kn[l], vn[l])
            cs.cs_paged_attention_mixed(pool, l, bb, q[l], out[l], sh.Hq, sh.scale, ws)

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / iters * 1e6

    eager_us = timed(run)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    graph_us = timed(graph.replay)
    log("  %d layers of append + attention: %.0f us call by call, %.0f us as one HIP graph replay"
        % (layers, eager_us, graph_us))
    return {"layers": layers, "eager_us": round(eager_us, 1), "graph_us": round(graph_us, 1)}


def preemption_loop(b, layers=32, iters=10):
    """Layer-wise preemption driver (cs_run_layers) over `layers` layers of this batch: cost
    of the safepoints (every 4 layers) with and without waiting for the stream, and the time
    of an iteration that is preempted at its second safepoint."""
    import ctypes
    import torch
    from paper_2410_01228_amd import binding as cs
    from paper_2410_01228_amd import synth
    sh = b.shape
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    pool = cs.Pool.empty(layers, b.num_pages, sh.Hkv, sh.D)
    fill_randn_bf16(pool.tensor.view(-1), gen)
    bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
    q = synth.randn_bf16((layers, b.T, sh.Hq, sh.D), gen, "cuda")
    k = synth.randn_bf16((layers, b.T, sh.Hkv, sh.D), gen, "cuda")
    v = synth.randn_bf16((layers, b.T, sh.Hkv, sh.D), gen, "cuda")
    out = torch.empty_like(q)
    ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)
    n_on = b.extra["n_online"]
    flag = ctypes.c_int32(0)

    count = [0]

    def run(sp):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iters):
            count[0] = 0
            cs.cs_run_layers(pool, 0, layers, bb, q, k, v, out, sh.Hq, sh.scale, ws, sp)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / iters * 1e3

    run(None)
    t_none = run(None)
    t_nosync = run(cs.cs_safepoint(ctypes.addressof(flag), cs.POLL_FN(0), None, 4, n_on, 0))
    t_sync = run(cs.cs_safepoint(ctypes.addressof(flag), cs.POLL_FN(0), None, 4, n_on, 1))

    def poll(_):
        count[0] += 1
        return 1 if count[0] == 2 else 0                             # second safepoint of every iteration

    cb = cs.POLL_FN(poll)
    t_pre = run(cs.cs_safepoint(None, cb, None, 4, n_on, 1))
    n_sp = layers // 4
    r = {"layers": layers, "safepoints": n_sp, "iteration_ms": round(t_none, 3),
         "iteration_ms_safepoints_nosync": round(t_nosync, 3), "iteration_ms_safepoints_sync": round(t_sync, 3),
         "safepoint_us_nosync": round((t_nosync - t_none) / n_sp * 1e3, 2),
         "safepoint_us_sync": round((t_sync - t_none) / n_sp * 1e3, 2),
         "iteration_ms_preempted_at_layer_4": round(t_pre, 3)}
    log("  preemption loop (%d layers, safepoint every 4): iteration %.3f ms; with safepoints %.3f ms (no wait, %.2f us each) / "
        "%.3f ms (waiting, %.2f us each); preempted at layer 4: %.3f ms"
        % (layers, t_none, t_nosync, r["safepoint_us_nosync"], t_sync, r["safepoint_us_sync"], t_pre))
    return r


def fit_latency_model(reps=8, dump=""):
    """Offline profiler of the paper's latency model, restricted to this path: time
    append + attention on a grid of (compute tokens, context) batches at the Llama-3.1-8B
    shape, least-squares fit of the per-token, attention, memory-access and constant terms,
    relative error of the fit (the paper reports < 4% for whole iterations)."""
    import torch
    from paper_2410_01228_amd import binding as cs
    from paper_2410_01228_amd import synth
    from paper_2410_01228_amd.latency_model import fit
    sh = synth.Shape(32, 8, 128)
    grid = []
    for P in (128, 256, 512, 1024, 2048):                        # one prefill chunk
        for C in (0, 2048, 8192, 16384, 32768):
            grid.append([(P, C)])
    for S in (32, 128, 256):                                     # decode batches
        for C in (1024, 4096, 16384):
            grid.append([(1, C)] * S)
    for P, C, S, Cd in ((512, 4096, 64, 2048), (1024, 16384, 128, 4096), (2048, 8192, 32, 8192)):   # mixed
        grid.append([(1, Cd)] * S + [(P, C)])
    pages = max(sum((p + c + 15) // 16 for p, c in batch) for batch in grid)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    pool = cs.Pool.empty(1, pages, sh.Hkv, sh.D)
    fill_randn_bf16(pool.tensor.view(-1), gen)
    samples = []
    for batch in grid:
        g = synth.generator(6)
        b = synth.make_batch(sh, [c for _, c in batch], [p for p, _ in batch], g, num_pages=pages)
        bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
        q = synth.randn_bf16((b.T, sh.Hq, sh.D), gen, "cuda")
        kn = synth.randn_bf16((b.T, sh.Hkv, sh.D), gen, "cuda")
        out = torch.empty_like(q)
        ws = cs.workspace_for(bb, sh.Hq, sh.Hkv, sh.D)

        def step():
            cs.cs_kv_append(pool, 0, bb, kn, kn)
            cs.cs_paged_attention_mixed(pool, 0, bb, q, out, sh.Hq, sh.scale, ws)

        for _ in range(2):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            step()
        e1.record()
        torch.cuda.synchronize()
        samples.append((batch, e0.elapsed_time(e1) / reps * 1e-3))
    if dump:
        with open(dump, "w") as f:
            json.dump([{"batch": bt, "seconds": t} for bt, t in samples], f)
    m, rel = fit(samples)
    import numpy as np
    big = np.array([t >= 150e-6 for _, t in samples])           # batches long enough to matter to an SLO
    r = {"shape": "32/8/128", "samples": len(samples), "k_token_s": m.k_p, "k2_attention_s": m.k2,
         "k4_memory_s": m.k4, "k5_constant_s": m.k5,
         "mean_rel_err": round(float(rel.mean()), 4), "max_rel_err": round(float(rel.max()), 4),
         "mean_rel_err_150us_up": round(float(rel[big].mean()), 4), "max_rel_err_150us_up": round(float(rel[big].max()), 4),
         "can_schedule_2048_tokens_ctx0_vs_ctx32768_at_1ms": [
             m.can_schedule([(1, 4096)] * 64, 2048, 0, 1e-3), m.can_schedule([(1, 4096)] * 64, 2048, 32768, 1e-3)]}
    log("  latency model over %d batches: k_token %.3e s, k2 %.3e s/pair, k4 %.3e s/token, k5 %.3e s; "
        "relative error mean %.1f%% max %.1f%% (batches of 150 us and more: mean %.1f%% max %.1f%%)"
        % (len(samples), m.k_p, m.k2, m.k4, m.k5, 100 * rel.mean(), 100 * rel.max(), 100 * rel[big].mean(), 100 * rel[big].max()))
    for (batch, t), e in zip(samples, rel):
        log("    %-34s %9.1f us  err %5.1f%%" % ("%d req, P=%d, C<=%d" % (len(batch), sum(p for p, _ in batch), max(c for _, c in batch)), t * 1e6, 100 * e))
    return r


def append_sweep():
    """cs_kv_append away from the launch-bound sizes of the stated workloads: prefill chunks of
    2048 tokens (page-ordered writer) and single decode tokens (per-token kernel), growing T."""
    import torch
    from paper_2410_01228_amd import binding as cs
    from paper_2410_01228_amd import synth
    sh = synth.Shape(32, 8, 128)
    rows = []
    for T, chunk in ((256, 1), (4096, 1), (32768, 1), (4096, 512), (65536, 2048), (262144, 2048), (1048576, 4096)):
        S = T // chunk
        g = synth.generator(5)
        ctx = synth.uniform_int(0, 64, S, g) if chunk > 1 else synth.uniform_int(16, 256, S, g)
        b = synth.make_batch(sh, ctx, [chunk] * S, g)
        pool = cs.Pool.empty(1, b.num_pages, sh.Hkv, sh.D)
        bb = cs.Batch(b.block_tables, b.ctx_lens, b.cu_q_lens)
        k = torch.randn((T, sh.Hkv, sh.D), device="cuda").to(torch.bfloat16)
        v = torch.randn_like(k)
        for _ in range(3):
            cs.cs_kv_append(pool, 0, bb, k, v)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            cs.cs_kv_append(pool, 0, bb, k, v)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 10 * 1e3
        nbytes = 2 * T * 2 * sh.Hkv * sh.D * 2
        rows.append({"tokens": T, "tokens_per_seq": chunk, "us": round(us, 1), "GBps": round(nbytes / us / 1e3, 1),
                     "frac_hbm": round(nbytes / (us * 1e-6) / HBM_PEAK, 4)})
        log("  append T=%-8d %4d tokens/seq: %9.1f us  %7.1f GB/s (read+write)  %.1f%% of hbm peak"
            % (T, chunk, us, rows[-1]["GBps"], 100 * rows[-1]["frac_hbm"]))
        del pool, k, v
    return rows


def read_traffic(name, kernel):
    """(full kernel name, HBM bytes per launch) of the kernel whose name, as the profiler prints
    it, starts with `kernel`, from the committed counter summary of the workload; of several
    such rows the one with the most launches.  (None, None) if there is no such row."""
    p = os.path.join(ROOT, "profiles", "%s_hbm_traffic.txt" % name)
    if not os.path.exists(p):
        return None, None
    in_table, best = False, (None, None, -1)
    for line in open(p):
        in_table = in_table or line.startswith("## HBM traffic")
        if in_table and line.startswith(kernel):
            f = line.split()                      # name ..., launches, FETCH, WRITE, HBM bytes
            if int(f[-4]) > best[2]:
                best = (line[:line.rfind(">") + 1] if ">" in line else f[0], float(f[-1]), int(f[-4]))
    return best[0], best[1]


def leg_record(leg, workload, dtype="bf16", page_size=16, fused=True):
    """One leg of the JSON line: times, roofline fraction against the leg's own bound and, where a
    committed counter summary covers the leg's kernel, that kernel's measured HBM bytes per launch."""
    r = leg.roofline()
    rec = {"us": round(leg.us, 2), "us_median": round(leg.us_median, 2), "us_min": round(leg.us_min, 2),
           "bound": leg.bound, "frac": r["frac"], "achieved": r["achieved"], "unit": r["unit"], "work": leg.work}
    if getattr(leg, "also", None):
        rec["also"] = leg.also_record()
    prefix, note = KERNEL_OF.get((workload, leg.name), (None, ""))
    if prefix and dtype == "f16":
        prefix = prefix.replace("cs::Bf16", "cs::F16")
    if prefix and page_size == 16 and (fused or "mixed_kernel" not in prefix):
        full, traffic = read_traffic(workload, prefix)
        if full is None:
            log("ERROR: profiles/%s_hbm_traffic.txt has no row for kernel '%s...' (leg %s): the committed counter summary "
                "is stale -- regenerate it from this binary" % (workload, prefix, leg.name))
            rec["traffic_error"] = "no row for %s in profiles/%s_hbm_traffic.txt" % (prefix, workload)
        rec["kernel"] = (full or prefix + " ...>") + (" (%s)" % note if note else "")
        rec["traffic"] = traffic
        rec["traffic_source"] = ("profiles/%s_hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this kernel on this "
                                 "workload, scaled by the plain copy kernel's readings; a committed summary, not measured in this run"
                                 % workload)
    return rec


def measure(name, steps, warmup, args, sub_batches=True):
    """Build one workload, time its step (and, for a mixed one, its decode-only and prefill-only
    sub-batches), and return (batch, info, legs, detail legs, seconds per step)."""
    b, legs, detail, info = build(name, f16=args.dtype == "f16", page_size=args.page_size)
    log("workload %s: S=%d T=%d pool %.2f GB, decode bytes %.3f GB, prefill %.3f TFLOP"
        % (info["name"], info["S"], info["T"], info["pool_gb"], info["dec_bytes"] / 1e9, info["pre_flops"] / 1e12))
    log("  attention call: " + info["arrangement"])
    sec_per_step = time_legs(legs, steps, warmup)
    if sub_batches and detail:
        time_legs(detail, steps, warmup)
    else:
        detail = []
    for leg in legs + detail:
        r = leg.roofline()
        extra = ""
        if getattr(leg, "also", None):
            a = leg.also_record()
            extra = "  + %.1f %s (%.1f%% of %s peak) in the same launch" % (a["achieved"], a["unit"], 100 * a["frac"], a["bound"])
        log("  %-24s %9.1f us  %10.1f %s  (%.1f%% of %s peak)%s" % (leg.name, leg.us, r["achieved"], r["unit"], 100 * r["frac"], r["bound"], extra))
    return b, info, legs, detail, sec_per_step


def dominant_leg(name, legs, detail):
    """The leg whose kernel the roofline object is quoted for: the checkpoint gather for the
    checkpoint workload, otherwise the attention call (whose one grid holds both kinds of work in
    a mixed batch; its decode bytes and prefill flops are then both reported)."""
    by_name = {l.name: l for l in legs}
    return by_name["ckpt_gather"] if name == "qwen14b_ckpt" else by_name["paged_attention_mixed"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama70b_long", choices=WORKLOADS,
                    help="the workload the headline value is quoted on (default: the largest single-GPU mixed batch)")
    ap.add_argument("--only", action="store_true", help="time only --workload (no `workloads` key with the other four)")
    ap.add_argument("--detail", action="store_true",
                    help="also run the workload's extra experiments (preemption loop, graph replay, checkpoint pipeline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--page-size", type=int, default=16, choices=[16, 8],
                    help="tokens per page of the pool (16: the paper's; 8: the smaller variant)")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16"],
                    help="element type of the pool and the queries (f16: the fp16 attention entry point)")
    ap.add_argument("--split-tokens", type=int, default=0, help="force the decode split (0 = automatic)")
    ap.add_argument("--mixed-arrangement", default="auto", choices=["auto", "separate", "behind", "beside"],
                    help="how a batch with decode tokens and chunks is launched: the host's choice (auto), two kernels "
                         "in a row, one grid with the decode work behind the tiles, or one grid with a decode "
                         "workgroup per CU beside the tiles")
    ap.add_argument("--separate-launches", action="store_true", help="the same as --mixed-arrangement separate")
    ap.add_argument("--append-sweep", action="store_true", help="also time cs_kv_append over growing token counts")
    ap.add_argument("--fit-latency-model", action="store_true",
                    help="also run the (P, C) timing grid and fit the paper's latency model to this path")
    ap.add_argument("--dump-latency-samples", default="", help="with --fit-latency-model: write the timed samples to this JSON file")
    ap.add_argument("--calibration-copy-gib", type=float, default=0.0,
                    help="also run the plain copy kernel on this many GiB three times (the known-size "
                         "reference that hardware byte counters are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build measures ONE GPU (the kernels of one GPU's share of the path); "
            "--gpus %d is not supported, run with --gpus 1." % args.gpus)
        sys.exit(2)

    import torch
    from paper_2410_01228_amd import binding as cs
    cs.lib()                                   # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    cs.cs_set_decode_split_tokens(args.split_tokens)
    if args.separate_launches:
        args.mixed_arrangement = "separate"
    cs.cs_set_mixed_fusion({"auto": 1, "separate": 0, "behind": 2, "beside": 3}[args.mixed_arrangement])
    if args.calibration_copy_gib > 0:
        n = int(args.calibration_copy_gib * (1 << 30)) // 16 * 16
        src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            cs.cs_debug_copy(dst, src)
        torch.cuda.synchronize()
        log("calibration: plain_copy_kernel moved %d bytes (read) + %d bytes (written) per launch" % (n, n))
        del src, dst
    if args.page_size != 16 and args.workload not in ("llama8b_decode", "qwen7b_mixed", "llama70b_long"):
        sys.exit("bench.py: --page-size 8 is for the workloads llama8b_decode, qwen7b_mixed and llama70b_long")

    fused = args.mixed_arrangement != "separate"
    b, info, legs, detail, sec_per_step = measure(args.workload, args.steps, args.warmup, args)
    by_name = {l.name: l for l in legs}
    att_us = by_name["kv_append"].us + by_name["paged_attention_mixed"].us
    dom = dominant_leg(args.workload, legs, detail)
    dom_rec = leg_record(dom, args.workload, args.dtype, args.page_size, fused)
    roofline = dict(dom.roofline(dom_rec.get("traffic")), kernel=dom_rec.get("kernel", dom.name),
                    us=dom_rec["us"], call=dom.name)
    if "traffic_source" in dom_rec:
        roofline["traffic_source"] = dom_rec["traffic_source"]
    if "also" in dom_rec:
        roofline["also"] = dom_rec["also"]
    result = {
        "metric": "mixed-batch paged-attn tokens/s per layer",
        "value": round(info["T"] / (att_us * 1e-6), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": info["name"], "num_seqs": info["S"], "num_tokens": info["T"],
                   "page_size": args.page_size, "layers_per_step": 1, "attention_launch": info["arrangement"],
                   "step": "+".join(l.name for l in legs)},
        "roofline": roofline,
        "legs": {l.name: leg_record(l, args.workload, args.dtype, args.page_size, fused) for l in legs + detail},
    }
    if args.detail and args.workload == "qwen14b_ckpt":
        result["ckpt_pipeline"] = checkpoint_pipeline(info)
    cpu_b = b
    del info["keep"][:]
    del legs, detail, dom, by_name
    import gc
    gc.collect()
    torch.cuda.empty_cache()

    if not args.only:
        # the other workloads, from the same run: every call of their step and, for the mixed ones,
        # the two attention paths on their own sub-batches
        result["workloads"] = {}
        o_steps, o_warm = min(args.steps, 20), min(args.warmup, 5)
        for name in WORKLOADS:
            if name == args.workload or (args.page_size != 16 and name in ("tiny", "qwen14b_ckpt")):
                continue
            ob, oinfo, olegs, odetail, osec = measure(name, o_steps, o_warm, args)
            on = {l.name: l for l in olegs}
            result["workloads"][oinfo["name"]] = {
                "num_seqs": oinfo["S"], "num_tokens": oinfo["T"], "steps": o_steps, "warmup": o_warm,
                "attention_launch": oinfo["arrangement"],
                "tokens_per_s": round(oinfo["T"] / ((on["kv_append"].us + on["paged_attention_mixed"].us) * 1e-6), 1),
                "ms_per_step": round(osec * 1e3, 4),
                "legs": {l.name: leg_record(l, name, args.dtype, args.page_size, fused) for l in olegs + odetail}}
            del oinfo["keep"][:]
            del olegs, odetail, on, ob, oinfo
            gc.collect()
            torch.cuda.empty_cache()
    if args.append_sweep:
        result["append_sweep"] = append_sweep()
    if args.fit_latency_model:
        result["latency_model"] = fit_latency_model(dump=args.dump_latency_samples)
    if args.detail and args.workload == "qwen7b_mixed":
        result["preemption_loop"] = preemption_loop(cpu_b)
    if args.detail and args.workload == "tiny":
        result["graph_replay"] = graph_replay(cpu_b)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cpu_b)
        if args.workload == "qwen14b_ckpt":
            result["cpu_baseline_copies"] = cpu_copy_baseline(cpu_b)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
