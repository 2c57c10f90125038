#!/usr/bin/env python3
"""Benchmark of the AdapShot KV-reuse hot path on one MI355X.

A step is one pass of the whole path over one query of the Llama-3-8B-shaped single-layer
workload (256 of 2000 cached shots, ~26k context tokens, 128 query tokens, 128 x 128256 logits):
    adapshot_assemble  ->  adapshot_query_attn  ->  adapshot_probe_entropy
with every input already resident in HBM.  Selections, caches and logits rotate over several
distinct buffers so that a step does not find its inputs in the 256 MB Infinity Cache.

Prints ONE JSON line: whole-path throughput (`value`, context tokens re-encoded and attended per
second), per-kernel durations from HIP events attached to the dispatches on the launch stream, the roofline of the dominant
kernel, and the CPU oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2605_03644_amd import workloads as wl  # noqa: E402

HBM_PEAK_GBPS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
# HBM bytes per launch (read + written) from two rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE),
# each scaled by what the same counter reads for a plain 256 MiB device copy; the summary with the commands and
# the raw counter values is profiles/bench_llama8b_1layer_hbm_traffic.txt.  Counters cannot be read from inside
# this process, so the figures are carried here and hold for the default workload only.
MEASURED_TRAFFIC_BYTES = {
    "llama8b_1layer": {"assemble_reencode": 223.5e6, "query_attn": 130.6e6, "entropy_chunk": 65.8e6},
}
SETTLE_STEPS = 100                        # untimed steps before the timed region, --warmup included
PROFILE_WARMUP, PROFILE_STEPS = 50, 200   # the per-kernel pass: untimed steps, then steps with timed dispatches
METRIC = "re-encoded KV tokens/s (HBM GB/s) + query-over-cache attn TFLOP/s at 26k ctx"


def attn_flops(w, t_ctx: int, t_q: int) -> float:
    """q.k^T and p.v over the context (all rows) plus the causal part over the query's own tokens."""
    return 4.0 * w.n_q_heads * w.head_dim * (t_q * t_ctx + t_q * (t_q + 1) / 2.0)


def cpu_baseline(w, k_pool, v_pool, off, ids, order, q, ks, vs, logits):
    """The oracle, as it stands, on one full step of the same workload."""
    import oracle
    oracle.build(force=False)
    kp, vp = wl.as_numpy_storage(k_pool), wl.as_numpy_storage(v_pool)
    qn, ksn, vsn = wl.as_numpy_storage(q), wl.as_numpy_storage(ks), wl.as_numpy_storage(vs)
    zn = logits.cpu().numpy()
    t0 = time.perf_counter()
    pl = oracle.plan(off, ids, order)
    ko, vo, _ = oracle.assemble(kp, vp, w.dtype, w.rope_theta, oracle.KEYS_UNROTATED, pl, 0, pl["n"])
    t1 = time.perf_counter()
    o = oracle.query_attn(ko[0], vo[0], w.dtype, pl["n"], qn, ksn, vsn, w.rope_theta, pl["n"])
    t2 = time.perf_counter()
    h = oracle.entropy(zn)
    t3 = time.perf_counter()
    return dict(value=pl["n"] / (t3 - t0), unit="tokens/s", cores=oracle.threads(), kind="oracle",
                sample=f"one full step of the same workload ({pl['n']} context tokens, {w.t_q} query tokens, "
                       f"{zn.shape[0]} logit rows), timed once",
                seconds=dict(assemble=t1 - t0, query_attn=t2 - t1, probe_entropy=t3 - t2)), o, h


def measured_ceilings(dev) -> dict:
    """What library routines reach on this very GPU, measured now: a device-to-device copy and a reduction
    over 512 MB (HBM), and a square bf16 GEMM (matrix cores).  Context for the fractions of the published peaks."""
    def per_call(f, n):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n

    src = torch.empty(256 << 20, dtype=torch.bfloat16, device=dev).normal_()
    dst = torch.empty_like(src)
    nbytes = src.numel() * 2
    t_copy = per_call(lambda: dst.copy_(src), 20)
    f32 = src.view(torch.float32)
    t_read = per_call(lambda: torch.sum(f32), 20)
    del dst
    gemm = {}
    for m, n, k in ((8192, 8192, 8192), (16384, 8192, 8192), (16384, 16384, 4096), (4096, 4096, 32768)):
        a = torch.randn(m, k, device=dev, dtype=torch.bfloat16)
        b = torch.randn(k, n, device=dev, dtype=torch.bfloat16)
        c = torch.empty(m, n, device=dev, dtype=torch.bfloat16)
        t = per_call(lambda: torch.matmul(a, b, out=c), 10)
        gemm[f"{m}x{n}x{k}"] = 2.0 * m * n * k / t * 1e-12
        del a, b, c
    return {"copy_gbps": 2.0 * nbytes / t_copy * 1e-9, "torch_sum_gbps": nbytes / t_read * 1e-9,
            "gemm_bf16_tflops": max(gemm.values()), "gemm_bf16_tflops_by_shape": gemm,
            "how": "torch copy_ and sum over 512 MB, torch.matmul in bf16 (best of the shapes listed), timed now on this GPU"}


def extras(ad, dev) -> dict:
    """Secondary measurements at the other workloads' shapes (one layer each, synthetic, wall-clock over
    back-to-back calls): relevance ranking over the whole pool, the probe sweep over nested prefixes and one
    decode step, all through the batched entry points, and the 70B-shaped workload at its full 80-layer size
    (wall clock of one assemble call, host planning included).  Reported beside the headline, not part of it."""
    out = {}

    def wall(f, n):
        for _ in range(10):  # more than the library's ring of pinned table buffers, which are allocated on first use
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    # ranking: config 2's pool and query
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, dev)
    ctx = ad.Context.for_workload(w)
    ctx.pool_register(k_pool, v_pool, off)
    q, _, _ = wl.make_query(w, dev)
    sc = torch.empty(w.n_shots, dtype=torch.float32, device=dev)
    dt = wall(lambda: ctx.rank_shots(0, q, out=sc), 10)
    n_tok = int(off[-1])
    out["rank_shots"] = {"workload": f"{w.n_shots} shots, {n_tok} pool tokens, {w.t_q} query tokens",
                         "us_per_query": dt * 1e6, "pool_tokens_per_s": n_tok / dt,
                         "mfma_tflops_both_products": 4.0 * w.n_q_heads * w.head_dim * w.t_q * n_tok / dt * 1e-12}
    ctx.close()
    del k_pool, v_pool

    # zero-copy form against assemble + attention, config 2's query (one layer, contexts rotating as in the headline)
    w = wl.WORKLOADS["llama8b_1layer"]
    k_pool, v_pool, off = wl.make_pool(w, dev)
    ctx = ad.Context.for_workload(w)
    ctx.pool_register(k_pool, v_pool, off)
    sels = [wl.selection(w, variant=v) for v in range(8)]
    lens = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    zc_caches = [ad.Cache(ctx, max(lens), with_index=False) for _ in range(4)]
    q, ks, vs = wl.make_query(w, dev)
    zo = torch.empty_like(q)
    it = iter(range(10 ** 9))

    def two_pass():
        i = next(it)
        c = zc_caches[i % 4]
        c.reset()
        ctx.assemble(c, *sels[i % 8])
        ctx.query_attn(c, 0, c.len, q, ks, vs, c.len, out=zo)

    def zero_copy():
        i = next(it)
        ctx.query_attn_pool(0, sels[i % 8][0], sels[i % 8][1], q, ks, vs, lens[i % 8], out=zo)

    t2, tz = wall(two_pass, 100), wall(zero_copy, 100)
    out["zero_copy_attention"] = {"workload": f"{w.m_select} shots ~{int(np.mean(lens))} tokens, {w.t_q} query tokens, 1 layer",
                                  "assemble_then_attend_us": t2 * 1e6, "zero_copy_us": tz * 1e6, "zero_copy_over_two_pass": tz / t2}
    ctx.close()
    del k_pool, v_pool, zc_caches

    # probe sweep: 8 queries x prefixes {16..512} of their own 512-shot ordering, 64 probe tokens each
    w = wl.WORKLOADS["llama8b_sweep"]
    k_pool, v_pool, off = wl.make_pool(w, dev, n_layers=1)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    sels = [wl.selection(w, query=qi) for qi in range(8)]
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    caches = [ad.Cache(ctx, t, with_index=False) for t in totals]
    ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
    items, flops = [], 0.0
    for qi in range(8):
        ids, order = sels[qi]
        seq = [int(ids[o]) for o in order]
        qq, ks, vs = wl.make_query(w, dev, query=qi, layer=0)
        for k in (16, 32, 64, 128, 256, 512):
            n_ctx = int(sum(off[s + 1] - off[s] for s in seq[:k]))
            items.append((qi, n_ctx, qq, ks, vs, n_ctx, torch.empty_like(qq)))
            flops += attn_flops(w, n_ctx, w.t_q)
    packed = ctx.pack_attn_items(items)
    dt = wall(lambda: ctx.query_attn_batched(caches, 0, packed), 20)
    out["probe_sweep_attention"] = {"workload": "48 probes (8 queries x 6 nested prefixes up to 512 shots), 64 tokens each, 1 layer",
                                    "us_per_call": dt * 1e6, "tflops": flops / dt * 1e-12}
    ctx.close()
    del k_pool, v_pool, caches, items

    # decode step: 32 queries x ~16k context, one new token each
    w = wl.WORKLOADS["qwen7b_decode"]
    k_pool, v_pool, off = wl.make_pool(w, dev, n_layers=1)
    ctx = ad.Context.for_workload(w, n_layers=1)
    ctx.pool_register(k_pool, v_pool, off)
    nq = w.n_queries
    sels = [wl.selection(w, query=qi) for qi in range(nq)]
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    caches = [ad.Cache(ctx, t + 8, with_index=False) for t in totals]
    ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
    g = torch.Generator(device=dev)
    g.manual_seed(wl.SEED_BASE + 5)
    qd = torch.randn(nq, 1, w.n_q_heads, w.head_dim, device=dev, generator=g).bfloat16()
    kd = torch.randn(nq, 1, w.n_kv_heads, w.head_dim, device=dev, generator=g).bfloat16()
    vd = torch.randn(nq, 1, w.n_kv_heads, w.head_dim, device=dev, generator=g).bfloat16()
    od = [torch.empty_like(qd[i]) for i in range(nq)]
    items = [(i, caches[i].len, qd[i], kd[i], vd[i], caches[i].len, od[i]) for i in range(nq)]
    packed = ctx.pack_attn_items(items)
    dt = wall(lambda: ctx.query_attn_batched(caches, 0, packed), 30)
    kv_bytes = sum(totals) * w.n_kv_heads * w.head_dim * 2 * 2
    out["decode_step_attention"] = {"workload": f"{nq} queries, ~{int(np.mean(totals))} context tokens each, 1 layer",
                                    "us_per_step": dt * 1e6, "kv_gbps": kv_bytes / dt * 1e-9,
                                    "frac_of_hbm_peak": kv_bytes / dt * 1e-9 / HBM_PEAK_GBPS}
    ctx.close()
    del k_pool, v_pool, caches, items, packed
    torch.cuda.empty_cache()

    def fits(name, need):
        free, _ = torch.cuda.mem_get_info()
        if free < need + (8 << 30):
            out[name] = {"skipped": f"needs {(need + (8 << 30)) / 2**30:.0f} GiB of device memory, {free / 2**30:.0f} GiB free"}
            return False
        return True

    # probe entropy at other batch sizes: one row is latency-bound, thousands of rows stream
    w = wl.WORKLOADS["llama8b_1layer"]
    ctx = ad.Context.for_workload(w)
    big = wl.make_logits(w, dev, n_rows=4096)
    ent = {}
    for rows in (1, 48, 128, 4096):
        views = [big[(i * rows) % (4096 - rows + 1):][:rows] for i in range(8)]  # different rows of the 2.1 GB buffer each call
        ho = torch.empty(rows, dtype=torch.float32, device=dev)
        it = iter(range(10 ** 9))
        dt = wall(lambda: ctx.probe_entropy(views[next(it) % 8], out=ho), 20)
        ent[str(rows)] = {"us": dt * 1e6, "gbps": rows * w.vocab * 4 / dt * 1e-9}
    out["probe_entropy_by_rows"] = {"workload": f"{w.vocab}-way fp32 logits, wall clock per call (chunks + merge; one launch from 256 rows on)", **ent}
    ctx.close()
    del big, views
    torch.cuda.empty_cache()

    # the probe sweep at its full size: 32 layers, 8 queries, one assembly of each query's 512-shot ordering
    # serves its six nested prefixes; then 48 probes attend, layer by layer, in one batched call per layer
    w = wl.WORKLOADS["llama8b_sweep"]
    off = wl.shot_offsets(w)
    row = w.n_kv_heads * w.head_dim * 2
    sels = [wl.selection(w, query=qi) for qi in range(w.n_queries)]
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    if fits("llama8b_sweep_full_size", 2 * w.n_layers * row * (int(off[-1]) + sum(totals))):
        k_pool, v_pool, off = wl.make_pool(w, dev)
        ctx = ad.Context.for_workload(w)
        ctx.pool_register(k_pool, v_pool, off)
        caches = [ad.Cache(ctx, t, with_index=False) for t in totals]
        best = None
        for _ in range(2):
            for c in caches:
                c.reset()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        moved = 4.0 * w.n_layers * row * sum(totals)
        items, flops = [], 0.0
        for qi in range(w.n_queries):
            ids, order = sels[qi]
            seq = [int(ids[o]) for o in order]
            qq, ks, vs = wl.make_query(w, dev, query=qi, layer=0)
            for k in w.prefixes:
                n_ctx = int(sum(off[s + 1] - off[s] for s in seq[:k]))
                items.append((qi, n_ctx, qq, ks, vs, n_ctx, torch.empty_like(qq)))
                flops += attn_flops(w, n_ctx, w.t_q)
        packed = ctx.pack_attn_items(items)
        for layer in (0, 1):
            ctx.query_attn_batched(caches, layer, packed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for layer in range(w.n_layers):
            ctx.query_attn_batched(caches, layer, packed)
        torch.cuda.synchronize()
        dta = time.perf_counter() - t0
        out["llama8b_sweep_full_size"] = {
            "workload": f"{w.n_layers} layers, {w.n_queries} queries x {len(w.prefixes)} nested prefixes up to 512 shots "
                        f"(~{int(np.mean(totals))} tokens), {w.t_q} probe tokens",
            "assemble_ms": best * 1e3, "assemble_gbps": moved / best * 1e-9,
            "assemble_frac_of_hbm_peak": moved / best * 1e-9 / HBM_PEAK_GBPS,
            "sweep_attention_all_layers_ms": dta * 1e3, "attention_tflops": flops * w.n_layers / dta * 1e-12}
        # the same 48 probes with no assembled caches at all: one zero-copy batched call per layer over the 8 ranked
        # lists where they lie in the pool (the items are the same, their cache index read as a list index)
        lists = ctx.pack_shot_lists([s[0] for s in sels], [s[1] for s in sels])
        for layer in (0, 1):
            ctx.query_attn_pool_batched(layer, lists, packed)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for layer in range(w.n_layers):
            ctx.query_attn_pool_batched(layer, lists, packed)
        torch.cuda.synchronize()
        dtz = time.perf_counter() - t0
        out["llama8b_sweep_full_size"].update({
            "zero_copy_sweep_all_layers_ms": dtz * 1e3, "zero_copy_tflops": flops * w.n_layers / dtz * 1e-12,
            "assemble_plus_attention_ms": (best + dta) * 1e3, "zero_copy_over_two_pass": dtz / (best + dta)})
        # the same sweep with every (query, prefix) assembled from scratch into a cache of its own, as the
        # workload is worded: 1008 shots per query instead of 512
        del caches, items, packed
        torch.cuda.empty_cache()
        pre = [(qi, k) for qi in range(w.n_queries) for k in w.prefixes]
        ptot = []
        for qi, k in pre:
            ids, order = sels[qi]
            ptot.append(int(sum(off[ids[o] + 1] - off[ids[o]] for o in order[:k])))
        if fits("llama8b_sweep_full_size_from_scratch", 2 * w.n_layers * row * sum(ptot)):
            pc = [ad.Cache(ctx, t, with_index=False) for t in ptot]
            pid, pord = [], []
            for qi, k in pre:
                ids, order = sels[qi]
                pid.append(np.asarray([ids[o] for o in order[:k]], dtype=np.int32))
                pord.append(None)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ctx.assemble_batched(pc, pid, pord)
            torch.cuda.synchronize()
            dts = time.perf_counter() - t0
            moved_s = 4.0 * w.n_layers * row * sum(ptot)
            out["llama8b_sweep_full_size"]["from_scratch_assemble_ms"] = dts * 1e3
            out["llama8b_sweep_full_size"]["from_scratch_assemble_gbps"] = moved_s / dts * 1e-9
            out["llama8b_sweep_full_size"]["from_scratch_gb_moved"] = moved_s * 1e-9
            del pc
        ctx.close()
        del k_pool, v_pool
        torch.cuda.empty_cache()

    # the decode workload at its full size: 28 layers, 32 queries with their own 200-shot contexts, 64 steps;
    # every step appends one token per query to every layer and attends with it, layer by layer
    w = wl.WORKLOADS["qwen7b_decode"]
    off = wl.shot_offsets(w)
    row = w.n_kv_heads * w.head_dim * 2
    nq, steps = w.n_queries, w.decode_steps
    sels = [wl.selection(w, query=qi) for qi in range(nq)]
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    if fits("qwen7b_decode_full_size", 2 * w.n_layers * row * (int(off[-1]) + sum(totals) + nq * steps)):
        k_pool, v_pool, off = wl.make_pool(w, dev)
        ctx = ad.Context.for_workload(w)
        ctx.pool_register(k_pool, v_pool, off)
        caches = [ad.Cache(ctx, t + steps, with_index=False) for t in totals]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.assemble_batched(caches, [s[0] for s in sels], [s[1] for s in sels])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        moved = 4.0 * w.n_layers * row * sum(totals)
        g = torch.Generator(device=dev)
        g.manual_seed(wl.SEED_BASE + 6)
        kn = torch.randn(w.n_layers, nq, w.n_kv_heads, w.head_dim, device=dev, generator=g).bfloat16()
        vn = torch.randn(w.n_layers, nq, w.n_kv_heads, w.head_dim, device=dev, generator=g).bfloat16()
        qd = torch.randn(nq, 1, w.n_q_heads, w.head_dim, device=dev, generator=g).bfloat16()
        kd = torch.randn(nq, 1, w.n_kv_heads, w.head_dim, device=dev, generator=g).bfloat16()
        vd = torch.randn(nq, 1, w.n_kv_heads, w.head_dim, device=dev, generator=g).bfloat16()
        od = [torch.empty_like(qd[i]) for i in range(nq)]
        kv_bytes = 0.0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            ctx.decode_append(caches, kn, vn)
            packed = ctx.pack_attn_items([(i, caches[i].len, qd[i], kd[i], vd[i], caches[i].len, od[i]) for i in range(nq)])
            for layer in range(w.n_layers):
                ctx.query_attn_batched(caches, layer, packed)
            kv_bytes += 2.0 * w.n_layers * row * sum(c.len for c in caches)
        torch.cuda.synchronize()
        dtd = time.perf_counter() - t0
        out["qwen7b_decode_full_size"] = {
            "workload": f"{w.n_layers} layers, {nq} queries x ~{int(np.mean(totals))} context tokens, {steps} decode steps "
                        "(append + attention in every layer)",
            "assemble_ms": dt * 1e3, "assemble_gbps": moved / dt * 1e-9,
            "decode_ms_per_step": dtd / steps * 1e3, "decode_tokens_per_s": nq * steps / dtd,
            "kv_gbps": kv_bytes / dtd * 1e-9, "frac_of_hbm_peak": kv_bytes / dtd * 1e-9 / HBM_PEAK_GBPS}
        ctx.close()
        del k_pool, v_pool, caches, packed
        torch.cuda.empty_cache()

    # the 70B-shaped workload at its full size: all 80 layers of the 4000-shot pool resident (~167 GB),
    # 1000 shots (~127k tokens, ~42 GB) assembled in one call, then the query attending layer by layer
    w = wl.WORKLOADS["llama70b_128k"]
    off = wl.shot_offsets(w)
    ids, order = wl.selection(w)
    total = int(sum(off[i + 1] - off[i] for i in ids))
    row = w.n_kv_heads * w.head_dim * 2
    if not fits("llama70b_128k_full_size", 2 * w.n_layers * row * (int(off[-1]) + total)):
        return out
    k_pool, v_pool, off = wl.make_pool(w, dev)
    ctx = ad.Context.for_workload(w)
    ctx.pool_register(k_pool, v_pool, off)
    cache = ad.Cache(ctx, total, with_index=False)
    best = None
    for _ in range(3):
        cache.reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.assemble(cache, ids, order)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    moved = 4.0 * w.n_layers * total * row  # K and V, read and written
    q, ks, vs = wl.make_query(w, dev)
    o = torch.empty_like(q)
    for layer in (0, 1):
        ctx.query_attn(cache, layer, total, q, ks, vs, total, out=o)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for layer in range(w.n_layers):
        ctx.query_attn(cache, layer, total, q, ks, vs, total, out=o)
    torch.cuda.synchronize()
    dta = time.perf_counter() - t0
    # consistency at full size: the last layer (byte offsets far beyond 2^32) against a one-layer context over
    # the same slice of the pool, whose path the parity tests check against the oracle
    last = w.n_layers - 1
    ctx.query_attn(cache, last, total, q, ks, vs, total, out=o)
    ctx1 = ad.Context.for_workload(w, n_layers=1)
    ctx1.pool_register(k_pool[last:last + 1], v_pool[last:last + 1], off)
    c1 = ad.Cache(ctx1, total, with_index=False)
    ctx1.assemble(c1, ids, order)
    o1 = ctx1.query_attn(c1, 0, total, q, ks, vs, total)
    torch.cuda.synchronize()
    same = bool(torch.equal(c1.k[0], cache.k[last]) and torch.equal(c1.v[0], cache.v[last]) and torch.equal(o1, o))
    ctx1.close()
    del c1
    out["llama70b_128k_full_size"] = {
        "last_layer_equals_one_layer_path": same,
        "workload": f"{w.n_layers} layers, pool {2 * w.n_layers * row * int(off[-1]) / 1e9:.0f} GB resident, "
                    f"{len(ids)} shots = {total} tokens assembled per call, {w.t_q} query tokens",
        "assemble_ms": best * 1e3, "assemble_gbps": moved / best * 1e-9,
        "assemble_frac_of_hbm_peak": moved / best * 1e-9 / HBM_PEAK_GBPS,
        "token_layers_per_s": total * w.n_layers / best,
        "attention_all_layers_ms": dta * 1e3,
        "attention_tflops": attn_flops(w, total, w.t_q) * w.n_layers / dta * 1e-12}
    ctx.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-extras", action="store_true", help="skip the secondary measurements (ranking, sweep, decode)")
    ap.add_argument("--workload", default="llama8b_1layer")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy 4 times (reference kernel of known traffic for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1

    from paper_2605_03644_amd import binding as ad
    ad.load_library()
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    w = wl.WORKLOADS[args.workload]
    assert w.n_layers == 1 and w.n_queries == 1, "bench times the single-query, single-layer configuration"

    n_var, n_buf = 8, 4
    k_pool, v_pool, off = wl.make_pool(w, dev)
    ctx = ad.Context.for_workload(w)
    ctx.pool_register(k_pool, v_pool, off)
    sels = [wl.selection(w, variant=v) for v in range(n_var)]
    totals = [int(sum(off[i + 1] - off[i] for i in ids)) for ids, _ in sels]
    cap = max(totals)
    caches = [ad.Cache(ctx, cap, with_index=False) for _ in range(n_buf)]
    q, ks, vs = wl.make_query(w, dev)
    outs = [torch.empty_like(q) for _ in range(n_buf)]
    logits = [wl.make_logits(w, dev, variant=b) for b in range(n_buf)]
    ents = [torch.empty(w.entropy_rows, dtype=torch.float32, device=dev) for _ in range(n_buf)]

    def step(i: int) -> int:
        v, b = i % n_var, i % n_buf
        cache = caches[b]
        cache.reset()
        ids, order = sels[v]
        ctx.assemble(cache, ids, order)
        n = cache.len
        ctx.query_attn(cache, 0, n, q, ks, vs, n, out=outs[b])
        ctx.probe_entropy(logits[b], out=ents[b])
        return n

    # Set-up, before the W warm-up steps and outside every timed figure: enough untimed steps for the library's
    # grow-only workspaces and its ring of pinned table buffers to exist and for the clocks to leave their idle state,
    # so that a run with a handful of --warmup steps times the same steady state as a long one.
    settle = max(0, SETTLE_STEPS - args.warmup)
    for i in range(settle):
        step(i)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tokens = 0
    for i in range(args.steps):
        tokens += step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # Per-kernel durations: the same steps again, every kernel's dispatch carrying a pair of HIP events on the
    # launch stream.  This pass has a length of its own, whatever --steps says, so that a short run reports the
    # same figures as a long one: PROFILE_WARMUP further untimed steps, then PROFILE_STEPS recorded ones.
    for i in range(PROFILE_WARMUP):
        step(i)
    ctx.profile_enable(True)
    for i in range(PROFILE_STEPS):
        step(i)
    torch.cuda.synchronize()
    prof = ctx.profile_read_each()
    ctx.profile_enable(False)
    kern = {k: dict(avg_us=float(ms.mean()) * 1e3, median_us=float(np.median(ms)) * 1e3, min_us=float(ms.min()) * 1e3,
                    launches=int(ms.size)) for k, ms in prof.items() if ms.size}

    t_ctx = tokens / args.steps
    row_bytes = w.kv_bytes_per_token_layer          # K row + V row
    asm_bytes = 2.0 * row_bytes * t_ctx * w.n_layers  # read + write
    ent_bytes = 4.0 * w.vocab * w.entropy_rows
    flops = attn_flops(w, t_ctx, w.t_q)
    asm_us, attn_us, ent_us = (kern[k]["avg_us"] for k in ("assemble_reencode", "query_attn", "entropy_chunk"))
    rl = {
        "assemble_reencode": dict(bound="hbm", achieved=asm_bytes / asm_us * 1e-3, peak=HBM_PEAK_GBPS, unit="GB/s",
                                  traffic=None, avg_us=asm_us, median_us=kern['assemble_reencode']['median_us'], min_us=kern['assemble_reencode']['min_us'], algorithmic_bytes=asm_bytes),
        "query_attn": dict(bound="mfma", achieved=flops / attn_us * 1e-6, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                           traffic=None, avg_us=attn_us, median_us=kern['query_attn']['median_us'],
                           min_us=kern['query_attn']['min_us'], algorithmic_flops=flops),
        "entropy_chunk": dict(bound="hbm", achieved=ent_bytes / ent_us * 1e-3, peak=HBM_PEAK_GBPS, unit="GB/s",
                              traffic=None, avg_us=ent_us, median_us=kern['entropy_chunk']['median_us'],
                              min_us=kern['entropy_chunk']['min_us'], algorithmic_bytes=ent_bytes),
    }
    for name, r in rl.items():
        r["frac"] = r["achieved"] / r["peak"]
        r["traffic"] = MEASURED_TRAFFIC_BYTES.get(w.name, {}).get(name)
        r["traffic_source"] = "profiles/bench_llama8b_1layer_hbm_traffic.txt (rocprofv3 --pmc of this script), not read in this run"
    dominant = max(rl, key=lambda k: rl[k]["avg_us"])
    roofline = dict(kernel=dominant, **{k: rl[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic",
                                                                       "traffic_source", "avg_us", "median_us", "min_us")},
                    launches_timed=PROFILE_STEPS, untimed_steps_before=settle + args.warmup + args.steps + PROFILE_WARMUP)

    result = {
        "metric": METRIC, "value": tokens / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic", "untimed_steps_before_timed_region": settle + args.warmup,
        "config": {"workload": f"{w.name}: {w.n_q_heads}q/{w.n_kv_heads}kv heads, d={w.head_dim}, theta={w.rope_theta:g}, "
                               f"pool {w.n_shots} shots [{w.len_lo},{w.len_hi}], {w.m_select} shots ~{t_ctx:.0f} tokens "
                               f"assembled per step, {w.t_q} query tokens, entropy over {w.entropy_rows}x{w.vocab} fp32 logits",
                   "layers": w.n_layers, "selections_cycled": n_var, "buffers_cycled": n_buf},
        "roofline": roofline,
        "roofline_all": rl,
        "kernels_us": {k: round(v["avg_us"], 3) for k, v in kern.items()},
        "kernels_median_us": {k: round(v["median_us"], 3) for k, v in kern.items()},
        "assemble_gbps": rl["assemble_reencode"]["achieved"],
        "attn_tflops": rl["query_attn"]["achieved"],
        "entropy_gbps": rl["entropy_chunk"]["achieved"],
        "paper_context": "paper reports 4.64x end-to-end speedup over DBSA on 8x Ascend 910B2 (not comparable)",
    }

    if not args.no_cpu_baseline:
        ids, order = sels[0]
        base, o_ref, h_ref = cpu_baseline(w, k_pool, v_pool, off, ids, order, q, ks, vs, logits[0])
        result["cpu_baseline"] = base
        result["gpu_over_cpu"] = result["value"] / base["value"]
        # the step the oracle just computed, once more on the GPU, as a sanity check of the timed path
        caches[0].reset()
        ctx.assemble(caches[0], ids, order)
        o = ctx.query_attn(caches[0], 0, caches[0].len, q, ks, vs, caches[0].len).float().cpu().numpy()
        h = ctx.probe_entropy(logits[0]).cpu().numpy()
        result["check"] = dict(attn_max_abs=float(np.abs(o - o_ref).max()), entropy_max_abs=float(np.abs(h - h_ref).max()))
    else:
        result["cpu_baseline"] = None
    if not args.no_extras and not args.copy_calibration:
        ctx.close()
        del k_pool, v_pool, caches, logits
        torch.cuda.empty_cache()
        try:
            ceil = measured_ceilings(dev)
            result["measured_ceilings"] = ceil
            rl["assemble_reencode"]["frac_of_measured_copy"] = rl["assemble_reencode"]["achieved"] / ceil["copy_gbps"]
            rl["entropy_chunk"]["frac_of_torch_sum"] = rl["entropy_chunk"]["achieved"] / ceil["torch_sum_gbps"]
            rl["query_attn"]["frac_of_measured_gemm"] = rl["query_attn"]["achieved"] / ceil["gemm_bf16_tflops"]
        except Exception as e:
            result["measured_ceilings"] = {"error": f"{type(e).__name__}: {e}"}
        try:
            result["extras"] = extras(ad, dev)
        except Exception as e:  # the headline above stands on its own; say what happened to the rest
            result["extras"] = {"error": f"{type(e).__name__}: {e}"}
        print(json.dumps(result))
        return 0
    if args.copy_calibration:
        src = torch.empty(128 << 20, dtype=torch.bfloat16, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["copy_calibration"] = {"bytes_read": src.numel() * 2, "bytes_written": src.numel() * 2, "launches": 4}
    print(json.dumps(result))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
