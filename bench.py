#!/usr/bin/env python3
"""Benchmark of the TableCache hot path on one MI355X.

A step is one pass of the whole path over one batch: tc_stitch_kv (gather of the selected
tables' KV into sequence blocks, all layers) followed by tc_prefill_attn for every layer
(suffix K/V append, GQA prefill attention, split-KV merge), then the host-side release of
the sequence blocks.  Inputs (table KV in the device table cache, per-layer q/k/v) are
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|c1|c2|c3|c4|c5|c5db] [--no-cpu-baseline]

The default (`all`) times the long-schema workload c4 - the largest single-GPU configuration,
26 TFLOP of counted attention work and 25.8 GB of gather per step - as the headline with exactly
K steps, and then the batch-1 case c2, the 32-query batch c3 and the cold-cache loading pipeline
c5 as labelled sub-records of the same line, each with its own kernel times and roofline fractions.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0          # MI355X dense bf16 matrix peak
PEAK_FP32_TFLOPS = 157.3           # MI355X fp32 vector peak
PEAK_HBM_GBPS = 8000.0
METRIC = "suffix prefill attn TFLOP/s + KV-stitch GB/s; per-query prefill ms (1 GPU)"
LLC_BYTES = 256 << 20               # last-level cache: destinations of small gathers are rotated past it


def attn_flops_per_layer(cfg, P, S):
    """4*Hq*D per unmasked (row, key) pair: QK^T and PV, 2 flops per multiply-add."""
    return sum(4 * cfg.n_q_heads * cfg.head_dim * (int(s) * int(p) + int(s) * (int(s) + 1) // 2)
               for p, s in zip(P, S))


def read_traffic(workload):
    """HBM bytes per attention launch (FETCH_SIZE + WRITE_SIZE counter runs of this same command,
    scaled by a copy kernel of known size) from the committed counter summary of the workload."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "prefill_attn_*_%s_pmc.txt" % workload))):
        try:
            for line in open(path):
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split()[1])
        except OSError:
            pass
    return None


def bench_pipeline(args):
    """Cold-cache loading pipeline (Sec. 4.2.2): the ordered requests are computed b_c at a time on
    the compute stream while the tables of the next b_m requests are copied from pinned host memory
    on a side stream, following the schedule of tc_plan_pipeline.  Three timings from the same warm
    start (tables 0..C-1 resident): the pipeline; the loads alone; the compute alone (same batches,
    every copy finished before the clock starts).  With --ablation the same measurement is repeated
    over the replacement rules of App. A, with and without the reranking of Sec. 4.2.1, with and
    without overlap (b_m = 0), which gives the shape of the paper's ablation tables on a synthetic
    trace: misses, pipeline time, and the load time the computation could not hide."""
    import torch
    from paper_2601_08743_amd import binding as B
    from paper_2601_08743_amd import pipeline as PL
    from paper_2601_08743_amd import workloads as W
    wl = W.get(args.workload)
    c = wl.cfg
    b_c = args.micro_batch
    b_m = b_c if args.prefetch < 0 else args.prefetch
    t_setup = time.time()
    P_all = np.array([int(wl.table_len[q].sum()) for q in wl.queries])
    S_all = wl.suffix_len.astype(int)
    need = [-(-(int(p) + int(s)) // 16) for p, s in zip(P_all, S_all)]
    max_tok = int(wl.table_len.max())
    n_blocks = c.capacity * (-(-max_tok // 16)) + 2 * b_c * max(need) + 16
    max_blocks = max(need) + 1
    pool, host_kv = None, []
    for t in range(c.n_tables):
        k, v = wl.table_kv(t)
        host_kv.append((torch.from_numpy(k).pin_memory(), torch.from_numpy(v).pin_memory()))
    s_main, s_load = torch.cuda.Stream(), torch.cuda.Stream()
    load_streams = [s_load] + [torch.cuda.Stream() for _ in range(max(args.load_streams, 1) - 1)]
    # suffix activations: two layers' worth of random q/k/v, reused cyclically by the layers
    # (their values do not change what is timed)
    qkv = []
    for l in range(2):
        q, k, v = wl.suffix_qkv(l)
        qkv.append(tuple(torch.from_numpy(x).view(torch.bfloat16).cuda() for x in (q, k, v)))
    out = torch.empty_like(qkv[0][0])
    L = c.n_layers
    setup_s = time.time() - t_setup

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    def case(policy, rerank, bc, bm, reps, warmup, serial=False):
        nonlocal pool
        cfg = B.make_config(c.n_layers, c.n_q_heads, c.n_kv_heads, c.head_dim, B.TC_BF16, n_blocks,
                            c.capacity, max_tok, policy)
        if pool is None:
            pool = torch.empty(B.tc_pool_bytes(cfg), dtype=torch.uint8, device="cuda")
        ctx = None

        def fresh():
            """A new context over the same pool, tables 0..C-1 resident (table 0 most recent): every
            phase of every repetition starts from the same cache and the same rule state."""
            nonlocal ctx
            if ctx is not None:
                torch.cuda.synchronize()
                ctx.tc_destroy()
            ctx = B.Context(cfg, pool)
            if args.attn_kernel:
                ctx.tc_set_attn_kernel(args.attn_kernel)
            for t in range(c.n_tables):
                ctx.tc_register_table_kv(t, int(wl.table_len[t]), host_kv[t][0], host_kv[t][1])
            ctx.tc_load_async(list(range(c.capacity - 1, -1, -1)), 0, L, s_load)
            torch.cuda.synchronize()
            ctx.tc_load_trace()

        order = list(range(c.batch))
        if rerank:
            order = B.tc_rerank(wl.table_ids, wl.cu_tables, c.n_tables, 0).tolist()
        queries = [wl.queries[i] for i in order]
        sl_all = wl.suffix_len[order].astype(np.int32)
        cu_r = np.concatenate([[0], np.cumsum(sl_all)]).astype(np.int64)     # rows of the reordered batch
        steps = PL.plan(queries, c.capacity, bc, bm, taper=not args.no_taper and bm > 0)
        steps_serial = PL.plan(queries, c.capacity, bc, 0)

        def stitch(c0, c1):
            ids = PL.flat_tables(queries, c0, c1)
            cu_t = np.concatenate([[0], np.cumsum([len(q) for q in queries[c0:c1]])]).astype(np.int32)
            sl = sl_all[c0:c1]
            bt, pl = ctx.tc_stitch_kv(ids, cu_t, sl, max_blocks, s_main)
            return bt, pl, sl

        def layers(c0, c1, h):
            bt, pl, sl = h
            cs = np.concatenate([[0], np.cumsum(sl)]).astype(np.int32)
            r0, r1 = int(cu_r[c0]), int(cu_r[c1])
            for l in range(L):
                q, kk, v = qkv[l & 1]
                ctx.tc_prefill_attn(l, q[r0:r1], kk[r0:r1], v[r0:r1], out[r0:r1], cs, bt, pl, sl,
                                    wl.sm_scale, s_main)
            ctx.tc_release_seqs(bt)

        t_compute = [0.0]

        def stitch_clocked(c0, c1):          # serial schedule: every copy is done before the clock starts
            torch.cuda.synchronize()
            t_compute.append(time.perf_counter())
            return stitch(c0, c1)

        def layers_clocked(c0, c1, h):
            layers(c0, c1, h)
            torch.cuda.synchronize()
            t_compute[0] += (time.perf_counter() - t_compute.pop()) * 1e3

        res_p, res_l, res_c, misses, nbytes = [], [], [], 0, 0
        for rep in range(reps + warmup):
            fresh()
            tp = timed(lambda: PL.run(ctx, queries, steps, 0, L, load_streams, stitch, layers,
                                      torch.cuda.synchronize if serial else None))
            tr = ctx.tc_load_trace()
            fresh()
            tl = timed(lambda: PL.run(ctx, queries, steps, 0, L, load_streams, lambda a, b: None, lambda a, b, h: None))
            fresh()
            t_compute[0] = 0.0
            PL.run(ctx, queries, steps_serial, 0, L, s_load, stitch_clocked, layers_clocked)
            if rep >= warmup:
                res_p.append(tp); res_l.append(tl); res_c.append(t_compute[0])
                miss_ids = tr[tr[:, 1] == 0][:, 0]
                misses = int(miss_ids.size)
                nbytes = int(sum(int(wl.table_len[t]) for t in miss_ids)) * 2 * c.kv_row_bytes * L
        torch.cuda.synchronize()
        ctx.tc_destroy()
        T_p, T_l, T_c = float(np.median(res_p)), float(np.median(res_l)), float(np.median(res_c))
        return {"policy": ["lru", "fifo", "lfu"][policy], "rerank": bool(rerank), "b_c": bc, "b_m": bm,
                "overlap": not serial,
                "misses": misses, "h2d_bytes": nbytes, "t_pipeline_ms": round(T_p, 3), "t_loads_ms": round(T_l, 3),
                "t_compute_ms": round(T_c, 3), "exposed_load_ms": round(T_p - T_c, 3)}

    link_peak = link_peak_gbps()
    policy = {"lru": 0, "fifo": 1, "lfu": 2}[args.policy]
    r = case(policy, args.rerank, b_c, b_m, args.steps, args.warmup)
    T_p, T_l, T_c, nbytes = r["t_pipeline_ms"], r["t_loads_ms"], r["t_compute_ms"], r["h2d_bytes"]
    ablation = None
    if args.ablation:
        # without overlap: b_m = 0 and the device idle before each micro-batch's loads are issued
        ablation = [case(pol, rr, b_c, 0 if serial else b_m, 1, 1, serial)
                    for pol in (0, 1, 2) for rr in (False, True) for serial in (True, False)]
    flops = attn_flops_per_layer(c, P_all, S_all) * L
    res = {
        "metric": METRIC, "what": "cold-cache pipeline: loads + stitch + per-layer attention",
        "value": round(flops / (T_p * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(T_p, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: L=%d Hq=%d Hkv=%d D=128, %d tables in pinned host memory, device cache C=%d (%s, "
                               "warm 0..%d), B=%d, b_c=%d%s, b_m=%d, reranking %s, sum P=%d, S=%d" % (
                                   c.name, L, c.n_q_heads, c.n_kv_heads, c.n_tables, c.capacity, args.policy.upper(),
                                   c.capacity - 1, c.batch, b_c, "" if args.no_taper else " (tapering tail)", b_m,
                                   "on" if args.rerank else "off",
                                   int(P_all.sum()), int(S_all[0]))},
        "prefill_ms_per_query": round(T_p / c.batch, 4),
        "t_compute_ms": round(T_c, 3), "t_loads_ms": round(T_l, 3), "t_pipeline_ms": round(T_p, 3),
        "pipeline_over_max": round(T_p / max(T_c, T_l), 4), "exposed_load_ms": r["exposed_load_ms"],
        "misses": r["misses"], "h2d_bytes": nbytes,
        "h2d_gbps_loads_only": round(nbytes / (T_l * 1e-3) / 1e9, 2),
        "h2d_gbps_in_pipeline": round(nbytes / (T_p * 1e-3) / 1e9, 2),
        "compute_tflops_no_loads": round(flops / (T_c * 1e-3) / 1e12, 2),
        "roofline": {"bound": "host-link", "achieved": round(nbytes / (T_p * 1e-3) / 1e9, 2),
                     "peak": round(link_peak, 2), "unit": "GB/s", "frac": round(nbytes / (T_p * 1e-3) / 1e9 / link_peak, 4),
                     "traffic": None,
                     "note": "link-bound: the copies of a batch take longer than its compute; peak = this box's own "
                             "pinned 1 GiB host-to-device copy, measured in this run"},
        "h2d_frac_of_link_loads_only": round(nbytes / (T_l * 1e-3) / 1e9 / link_peak, 4),
        "cpu_baseline": None, "setup_s": round(setup_s, 1),
    }
    if ablation is not None:
        res["ablation"] = ablation
    del pool
    torch.cuda.empty_cache()
    return res


def frontend_extras(wl):
    """Host front end (Table Trie matching of Alg. 1, reranking of Eq. 1-2): rates on this workload's
    prompts and on a batch of 1024 zipf-drawn table sets; results checked (ids recovered, order valid)."""
    from paper_2601_08743_amd import binding as B
    from paper_2601_08743_amd import workloads as W
    c = wl.cfg
    trie = B.Trie()
    for t in range(c.n_tables):
        trie.tc_trie_insert(t, wl.table_tokens(t))
    prompts = [wl.prompt_tokens(i) for i in range(c.batch)]
    reps = max(1, 200 // c.batch)
    t0 = time.perf_counter()
    for _ in range(reps):
        got = [trie.tc_trie_match(p)[0] for p in prompts]
    dt = (time.perf_counter() - t0) / reps
    for i, m in enumerate(got):
        assert [tid for tid, _ in m][:len(wl.queries[i])] == wl.queries[i].tolist(), "front end: tables not recovered"
    n_tok = sum(p.size for p in prompts)
    big = W.make_workload(W.scaled(c, batch=1024, choice="zipf", tables_per_query=(4, 12), seed=c.seed + 77))
    t0 = time.perf_counter()
    order = B.tc_rerank(big.table_ids, big.cu_tables, c.n_tables, 0)
    dt_r = time.perf_counter() - t0
    assert sorted(order.tolist()) == list(range(1024))
    return {"frontend_match_mtok_s": round(n_tok / dt / 1e6, 2), "frontend_rerank_1024q_ms": round(dt_r * 1e3, 3)}


def zero_copy_extras(args, wl, qkv, outs_copy, flops_step, stream):
    """The same step with the stitch that copies nothing (a second context whose table slots are
    kept in block format; tc_stitch_alias builds the sequences by pointing at them): an extra
    measurement beside the headline step, which keeps the gather it is named for.  The last
    layer's output is compared with the copying path's (same inputs; the padded key tiles change
    rounding only)."""
    import torch
    from paper_2601_08743_amd import binding as B
    c = wl.cfg
    max_tok = int(wl.table_len.max())
    need = [sum(-(-int(wl.table_len[t]) // 16) for t in q) + -(-int(s) // 16) for q, s in zip(wl.queries, wl.suffix_len)]
    n_blocks = c.capacity * (-(-max_tok // 16)) + sum(-(-int(s) // 16) for s in wl.suffix_len) + 8
    cfg = B.make_config(c.n_layers, c.n_q_heads, c.n_kv_heads, c.head_dim, B.TC_BF16, n_blocks, c.capacity, max_tok,
                        slot_layout=B.TC_SLOTS_BLOCKS)
    pool = torch.empty(B.tc_pool_bytes(cfg), dtype=torch.uint8, device="cuda")
    ctx = B.Context(cfg, pool)
    keep = []
    for t in range(c.n_tables):
        k, v = wl.table_kv(t)
        hk, hv = torch.from_numpy(k).pin_memory(), torch.from_numpy(v).pin_memory()
        keep.append((hk, hv))
        ctx.tc_register_table_kv(t, int(wl.table_len[t]), hk, hv)
    ctx.tc_load_async(list(range(c.n_tables))[:c.capacity], 0, c.n_layers, stream)
    torch.cuda.synchronize()
    ids, cu_t, cu_s, sl = wl.table_ids, wl.cu_tables, wl.cu_seqlens, wl.suffix_len
    max_blocks = max(need) + 1
    outs = [torch.empty_like(o) for o in outs_copy]

    def run(n):
        for _ in range(n):
            bt, pl = ctx.tc_stitch_alias(ids, cu_t, sl, max_blocks, stream)
            for l in range(c.n_layers):
                q, k, v = qkv[l]
                ctx.tc_prefill_attn(l, q, k, v, outs[l], cu_s, bt, pl, sl, wl.sm_scale, stream)
            ctx.tc_release_seqs(bt)

    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    t0 = time.perf_counter()
    for _ in range(20):
        bt, pl = ctx.tc_stitch_alias(ids, cu_t, sl, max_blocks, stream)
        ctx.tc_release_seqs(bt)
    host_us = (time.perf_counter() - t0) * 1e6 / 20
    torch.cuda.synchronize()
    ctx.tc_profile_enable(True)
    run(max(3, args.steps // 5))
    torch.cuda.synchronize()
    prof = ctx.tc_profile_read()
    ctx.tc_profile_enable(False)
    diff = float((outs[-1].float() - outs_copy[-1].float()).abs().max())
    res = {"zero_copy_ms_per_step": round(ms, 4), "zero_copy_tflops": round(flops_step / (ms * 1e-3) / 1e12, 3),
           "zero_copy_stitch_host_us": round(host_us, 1),
           "zero_copy_attn_kernel_us": round(prof["attn"][0] * 1e3 / max(prof["attn"][1], 1), 2),
           "zero_copy_max_abs_vs_copy": diff}
    torch.cuda.synchronize()
    ctx.tc_destroy()
    return res


def decode_extras(args, ctx, wl, prefill_layers, P, S, max_blocks, stream):
    """One generated token per query after the prefill (Sec. 2.2's decoding stage over the stitched
    cache): every layer appends the token's K/V and attends over the whole sequence.  The work is
    reading the sequences' K/V once per layer, so the figure is bytes per second of the decode
    attention kernel: kappa * sum(P + S) per launch."""
    import torch
    c = wl.cfg
    bt, pl = ctx.tc_stitch_kv(wl.table_ids, wl.cu_tables, wl.suffix_len, max_blocks, stream)
    prefill_layers(bt, pl)
    cur = (P + S).astype(np.int32)
    bt = ctx.tc_grow_seqs(bt, cur + 1)
    g = torch.Generator(device="cpu").manual_seed(7)
    q = torch.randn(c.batch, c.n_q_heads, c.head_dim, generator=g).bfloat16().cuda()
    k = torch.randn(c.batch, c.n_kv_heads, c.head_dim, generator=g).bfloat16().cuda()
    v = torch.randn(c.batch, c.n_kv_heads, c.head_dim, generator=g).bfloat16().cuda()
    out = torch.empty_like(q)
    one, cu1 = np.ones(c.batch, dtype=np.int32), np.arange(c.batch + 1, dtype=np.int32)

    def step():
        for l in range(c.n_layers):
            ctx.tc_prefill_attn(l, q, k, v, out, cu1, bt, cur, one, wl.sm_scale, stream)

    n = max(5, args.steps // 2)
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / n
    kernel, n_splits = ctx.tc_attn_kernel(), ctx.tc_kv_splits()
    ctx.tc_profile_enable(True)
    ctx.tc_profile_read()
    for _ in range(n):
        step()
    torch.cuda.synchronize()
    pr = ctx.tc_profile_read()
    ctx.tc_profile_enable(False)
    ctx.tc_release_seqs(bt)
    a_us = pr["attn"][0] * 1e3 / max(pr["attn"][1], 1)
    f_us = pr["merge"][0] * 1e3 / max(pr["merge"][1], 1)
    kv_bytes = 2 * c.n_kv_heads * c.head_dim * c.elem_bytes * int((P + S).sum())
    return {"decode_ms_per_token_step": round(ms, 4), "decode_attn_kernel_us": round(a_us, 2),
            "decode_finish_kernel_us": round(f_us, 2), "decode_kv_splits": n_splits,
            "decode_kernel": {3: "decode_attn_bf16_kernel"}.get(kernel, "prefill kernel %d" % kernel),
            "decode_kv_gbps": round(kv_bytes / (a_us * 1e-6) / 1e9, 1),
            "decode_frac_hbm": round(kv_bytes / (a_us * 1e-6) / 1e9 / PEAK_HBM_GBPS, 4)}


def link_peak_gbps():
    """The box's own large-transfer rate, pinned host memory to the device: the denominator for the loads."""
    import torch
    n = 1 << 30
    h = torch.empty(n, dtype=torch.uint8).pin_memory()
    d = torch.empty(n, dtype=torch.uint8, device="cuda")
    best = 0.0
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        d.copy_(h, non_blocking=True)
        torch.cuda.synchronize()
        best = max(best, n / (time.perf_counter() - t0) / 1e9)
    del h, d
    return best


def bench_resident(args, name, steps, warmup, extras=True, cpu_baseline=True):
    """One configuration whose tables all fit the device cache (c1-c4): returns its record."""
    import torch
    from paper_2601_08743_amd import binding as B
    from paper_2601_08743_amd import workloads as W

    wl = W.get(name)
    c = wl.cfg
    t_setup = time.time()
    P = np.array([int(wl.table_len[q].sum()) for q in wl.queries])
    S = wl.suffix_len.astype(int)
    need = [-(-(int(p) + int(s)) // 16) for p, s in zip(P, S)]
    max_blocks = max(need) + 1
    max_tok = int(wl.table_len.max())
    cap = c.capacity
    kappa = 2 * c.n_kv_heads * c.head_dim * c.elem_bytes
    # A gather whose destination fits the last-level cache would be timed against the cache, not HBM:
    # the blocks of a step are given back only `rotate` steps later, so the lowest-free allocator
    # hands every step fresh blocks and a destination is not written again before more than the
    # cache's size has gone by.  (The source tables are the same every step: on c1 and c2 they stay
    # cache-resident, which is why the HBM claim is made on c3 and c4.)
    dest_bytes = kappa * c.n_layers * sum(need) * 16
    rotate = int(min(8, max(1, -(-2 * LLC_BYTES // max(dest_bytes, 1)))))
    n_blocks = cap * (-(-max_tok // 16)) + (rotate + 1) * sum(need) + c.batch + 8   # + one more block per query for the decode extra
    cfg = B.make_config(c.n_layers, c.n_q_heads, c.n_kv_heads, c.head_dim,
                        B.TC_F32 if c.dtype == "f32" else B.TC_BF16, n_blocks, cap, max_tok)
    pool = torch.empty(B.tc_pool_bytes(cfg), dtype=torch.uint8, device="cuda")
    ctx = B.Context(cfg, pool)
    stream = torch.cuda.Stream()

    # offline part: register every table of the database, make the cache warm
    resident = list(range(c.n_tables))[:cap]
    tables_np, keep_host = {}, []
    used = set(wl.table_ids.tolist())
    for t in range(c.n_tables):
        k, v = wl.table_kv(t)
        hk, hv = torch.from_numpy(k).pin_memory(), torch.from_numpy(v).pin_memory()
        keep_host.append((hk, hv))
        ctx.tc_register_table_kv(t, int(wl.table_len[t]), hk, hv)
        if t in used:
            tables_np[t] = (k, v)
    ctx.tc_load_async(resident, 0, c.n_layers, stream)
    missing = [int(t) for t in wl.table_ids if t not in set(resident)]
    if missing:
        raise SystemExit("workload %s needs the loading pipeline (tables %s not resident)" % (c.name, missing[:5]))

    def dev(a):
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t if c.dtype == "f32" else t.view(torch.bfloat16)).cuda()

    qkv_np = [wl.suffix_qkv(l) for l in range(c.n_layers)]
    qkv = [tuple(dev(x) for x in qkv_np[l]) for l in range(c.n_layers)]
    outs = [torch.empty_like(qkv[l][0]) for l in range(c.n_layers)]
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup
    if args.splits:
        ctx.tc_set_kv_splits(args.splits)
    if args.row_blocks:
        ctx.tc_set_row_blocks(args.row_blocks)
    if args.attn_kernel:
        ctx.tc_set_attn_kernel(args.attn_kernel)

    ids, cu_t, cu_s, sl = wl.table_ids, wl.cu_tables, wl.cu_seqlens, wl.suffix_len
    scale = wl.sm_scale

    def layers(bt, pl):
        for l in range(c.n_layers):
            q, k, v = qkv[l]
            ctx.tc_prefill_attn(l, q, k, v, outs[l], cu_s, bt, pl, sl, scale, stream)

    def step():
        bt, pl = ctx.tc_stitch_kv(ids, cu_t, sl, max_blocks, stream)
        layers(bt, pl)
        return bt

    held = []

    def run(n):
        """n steps; the blocks of a step are released `rotate` steps later, once those steps have been
        enqueued on the same stream (stream order makes that safe for the earlier step's kernels)."""
        for _ in range(n):
            held.append(step())
            if len(held) > rotate - 1:
                ctx.tc_release_seqs(held.pop(0))

    def drain():
        while held:
            ctx.tc_release_seqs(held.pop(0))

    for _ in range(warmup):
        run(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # per-kernel durations: every launch carries two HIP events that receive its own begin and end
    # timestamps on the stream it is launched on (a second pass of the same steps)
    ctx.tc_profile_enable(True)
    run(steps)
    torch.cuda.synchronize()
    prof = ctx.tc_profile_read()
    ctx.tc_profile_enable(False)
    drain()
    bt, pl = ctx.tc_stitch_kv(ids, cu_t, sl, max_blocks, stream)
    n_splits = ctx.tc_kv_splits()
    kernel_name = {0: "attn_%s_kernel" % c.dtype, 1: "attn_bf16_kernel<1>", 2: "attn_bf16_pipe_kernel",
                   4: "attn_bf16_pp_kernel"}[ctx.tc_attn_kernel()]

    flops_layer = attn_flops_per_layer(c, P, S)
    flops_step = flops_layer * c.n_layers
    stitch_bytes = 2 * kappa * c.n_layers * int(P.sum())
    attn_us = prof["attn"][0] * 1e3 / max(prof["attn"][1], 1)
    merge_us = prof["merge"][0] * 1e3 / max(prof["merge"][1], 1)
    append_us = prof["append"][0] * 1e3 / max(prof["append"][1], 1)
    stitch_us = prof["stitch"][0] * 1e3 / max(prof["stitch"][1], 1)
    attn_tflops_kernel = flops_layer / (attn_us * 1e-6) / 1e12
    peak = PEAK_BF16_TFLOPS if c.dtype == "bf16" else PEAK_FP32_TFLOPS
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    extra = {}
    no_graph = args.no_graph or not extras
    # the re-encoding stitch (keys rotary-encoded by position while they are copied): same bytes, an
    # extra measurement beside the step; the step itself uses the plain stitch
    ctx.tc_release_seqs(bt)
    ctx.tc_profile_enable(extras)
    ctx.tc_profile_read()
    if extras:
        for _ in range(max(3, steps // 5)):
            bt_r, _ = ctx.tc_stitch_kv_rope(ids, cu_t, sl, None, 1.0e6, max_blocks, stream)
            ctx.tc_release_seqs(bt_r)
        torch.cuda.synchronize()
        prof_r = ctx.tc_profile_read()
        ctx.tc_profile_enable(False)
        rope_us = prof_r["stitch"][0] * 1e3 / max(prof_r["stitch"][1], 1)
        extra["stitch_rope_kernel_us"] = round(rope_us, 2)
        extra["stitch_rope_gbps"] = round(stitch_bytes / (rope_us * 1e-6) / 1e9, 1)
        extra["stitch_rope_frac_hbm"] = round(stitch_bytes / (rope_us * 1e-6) / 1e9 / PEAK_HBM_GBPS, 4)
        extra.update(frontend_extras(wl))
        if c.dtype == "bf16":
            sub = argparse.Namespace(**vars(args))
            sub.steps, sub.warmup = steps, warmup
            extra.update(zero_copy_extras(sub, wl, qkv, outs, flops_step, stream))
            extra.update(decode_extras(sub, ctx, wl, layers, P, S, max_blocks + 1, stream))
    bt, pl = ctx.tc_stitch_kv(ids, cu_t, sl, max_blocks, stream)
    if not no_graph:
        g = torch.cuda.CUDAGraph()
        layers(bt, pl)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=stream):
            layers(bt, pl)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / steps
        extra["graph_layers_ms"] = round(g_ms, 4)
        extra["graph_layers_tflops"] = round(flops_step / (g_ms * 1e-3) / 1e12, 2)
        del g

    # CPU baseline: the checker as it stands on the same workload - every row and head of a stated
    # sample of (layer, query) pairs, which is also a full-size parity check of those outputs; the
    # gather checker (a byte loop) is timed on the same pairs
    cpu = None
    parity = None
    if cpu_baseline:
        import oracle
        layers(bt, pl)
        torch.cuda.synchronize()
        fl_q = [4 * c.n_q_heads * c.head_dim * (int(s) * int(p) + int(s) * (int(s) + 1) // 2) for p, s in zip(P, S)]
        rate = 15e9                                               # the checker's usual rate on the box's 16 threads
        est_all = flops_step / rate
        if est_all <= 30:
            layer_set, q_set = list(range(c.n_layers)), list(range(c.batch))
        else:
            layer_set = [0, c.n_layers - 1]
            q_set = sorted({int(P.argmax()), int(P.argmin())} | set(np.linspace(0, c.batch - 1, 4).astype(int).tolist()))[:4]
            while len(q_set) > 1 and 2 * sum(fl_q[i] for i in q_set) / rate > 32:
                q_set.pop(len(q_set) // 2)
        t_cpu, t_gather, gather_bytes, worst, fl_done = 0.0, 0.0, 0, 0.0, 0
        for l in layer_set:
            q_np, k_np, v_np = qkv_np[l]
            got = outs[l].float().cpu().numpy().astype(np.float64)
            for i in q_set:
                tk = {int(t): tables_np[int(t)][0][l:l + 1] for t in wl.queries[i]}
                tv = {int(t): tables_np[int(t)][1][l:l + 1] for t in wl.queries[i]}
                t1 = time.perf_counter()
                ks, vs = oracle.stitch(tk, wl.queries[i])[0], oracle.stitch(tv, wl.queries[i])[0]
                t_gather += time.perf_counter() - t1
                gather_bytes += 2 * (ks.nbytes + vs.nbytes)
                s_ = slice(int(cu_s[i]), int(cu_s[i + 1]))
                a = [W.storage_to_f64(x, c.dtype) for x in (q_np[s_], ks, vs, k_np[s_], v_np[s_])]
                t1 = time.perf_counter()
                ref = oracle.prefill_attn(*a, scale)
                t_cpu += time.perf_counter() - t1
                fl_done += fl_q[i]
                worst = max(worst, float(np.abs(got[s_] - ref).max()))
        frac_done = fl_done / flops_step
        cpu = {"value": round(fl_done / t_cpu / 1e12, 6), "unit": "TFLOP/s",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "%s: every row and head of layers %s x queries %s = %.2f %% of the step's counted flops "
                         "(%.1f s of fp64 naive attention; the whole step extrapolates linearly to %.0f s)" % (
                             c.name, layer_set if len(layer_set) <= 4 else "0..%d" % (c.n_layers - 1),
                             q_set if len(q_set) <= 8 else "0..%d" % (c.batch - 1), 100 * frac_done, t_cpu,
                             t_cpu / frac_done),
               "gather": {"value": round(gather_bytes / max(t_gather, 1e-9) / 1e9, 3), "unit": "GB/s",
                          "sample": "the gather checker (byte loop, one thread) on the same (layer, query) pairs: "
                                    "%.1f MB read + written in %.3f s" % (gather_bytes / 1e6, t_gather)}}
        parity = worst
    ctx.tc_release_seqs(bt)

    stitch_gbps = stitch_bytes / (stitch_us * 1e-6) / 1e9
    res = {
        "metric": METRIC,
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": c.dtype, "data": "synthetic",
        "config": {"workload": "%s: L=%d Hq=%d Hkv=%d D=%d, %d tables U[%d,%d] tok, B=%d, P=%s, S=%s, block 16" % (
            c.name, c.n_layers, c.n_q_heads, c.n_kv_heads, c.head_dim, c.n_tables, c.table_len[0],
            c.table_len[1], c.batch, P.tolist() if c.batch <= 4 else "sum %d" % P.sum(),
            S.tolist() if c.batch <= 4 else "sum %d" % S.sum()), "kv_splits": n_splits,
            "stitch_destinations_rotated_over_steps": rotate},
        "what": "value = counted attention flops of a step / whole-step wall time (KV stitch + per-layer append, "
                "attention, split-KV merge)",
        "prefill_ms_per_query": round(ms_per_step / c.batch, 4),
        "attn_kernel_us": round(attn_us, 2), "merge_kernel_us": round(merge_us, 2),
        "append_kernel_us": round(append_us, 2), "stitch_kernel_us": round(stitch_us, 2),
        "attn_tflops_kernel_time": round(attn_tflops_kernel, 2),
        "stitch_gbps": round(stitch_gbps, 1),
        "stitch_frac_hbm": round(stitch_gbps / PEAK_HBM_GBPS, 4),
        "roofline": {"bound": "mfma" if c.dtype == "bf16" else "alu", "achieved": round(attn_tflops_kernel, 2),
                     "peak": peak, "unit": "TFLOP/s", "frac": round(attn_tflops_kernel / peak, 4),
                     "traffic": read_traffic(c.name), "kernel": kernel_name},
        "roofline_stitch": {"bound": "hbm", "achieved": round(stitch_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": round(stitch_gbps / PEAK_HBM_GBPS, 4), "kernel": "stitch_kernel",
                            "bytes_per_launch": stitch_bytes},
        "cpu_baseline": cpu, "parity_max_abs_vs_oracle": parity, "setup_s": round(setup_s, 1),
    }
    res.update(extra)
    torch.cuda.synchronize()
    ctx.tc_destroy()
    del pool, qkv, outs, keep_host
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    help="all (default: c4 as the headline, c2 / c3 / c5 as sub-records) or one of c1 c2 c3 c4 c5 c5db")
    ap.add_argument("--splits", type=int, default=0, help="force split-KV partitions (0 = automatic)")
    ap.add_argument("--row-blocks", type=int, default=0, help="force 128 (1) or 256 (2) rows per work-group")
    ap.add_argument("--attn-kernel", type=int, default=0,
                    help="force a bf16 attention kernel: 1 general, 2 pipelined, 4 alternating wave groups (0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline step: skip the extra measurements (re-encoding stitch, front end, "
                         "stitch without copying, decode steps, graph replay) and the sub-records; used for profiler runs")
    ap.add_argument("--no-graph", action="store_true", help="skip the extra timing of the layer loop replayed as a HIP graph")
    ap.add_argument("--micro-batch", type=int, default=8, help="b_c: requests computed per micro-batch (c5 pipeline)")
    ap.add_argument("--prefetch", type=int, default=-1, help="b_m: requests loaded ahead (c5 pipeline; default b_c, 0 = no overlap)")
    ap.add_argument("--load-streams", type=int, default=2,
                    help="c5 pipeline: side streams the load calls take in turn (2: one copy's start-up gap is covered by the other queue)")
    ap.add_argument("--policy", default="lru", choices=["lru", "fifo", "lfu"], help="replacement rule (c5 pipeline)")
    ap.add_argument("--rerank", action="store_true", help="visit the batch in reranked order (c5 pipeline)")
    ap.add_argument("--no-taper", action="store_true", help="c5 pipeline: micro-batches of b_c to the end (no shrinking tail)")
    ap.add_argument("--ablation", action="store_true", help="c5 pipeline: also run rules x reranking x overlap")
    ap.add_argument("--calibrate", action="store_true",
                    help="run one plain elementwise kernel of known size (reads 1 GiB, writes 1 GiB) before the "
                         "timed region, as the reference for scaling HBM counters of a --pmc run")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_08743_amd import binding as B          # noqa: F401  raises if the HIP library is not built

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate:
        x = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
        y = torch.empty_like(x)
        torch.add(x, 1, out=y)
        torch.cuda.synchronize()
        del x, y
    extras, cpu = not args.no_extras, not args.no_cpu_baseline
    if args.workload in ("c5", "c5db"):
        if args.steps == 20:
            args.steps, args.warmup = 3, 1
        res = bench_pipeline(args)
    elif args.workload != "all":
        res = bench_resident(args, args.workload, args.steps, args.warmup, extras, cpu)
    else:
        res = bench_resident(args, "c4", args.steps, args.warmup, extras, cpu)
        if extras:
            t0 = time.time()
            sub = {}
            sub["c2"] = bench_resident(args, "c2", 50, 5, True, cpu)
            sub["c3"] = bench_resident(args, "c3", 10, 3, True, cpu)
            pa = argparse.Namespace(**vars(args))
            pa.workload, pa.steps, pa.warmup = "c5", 2, 1
            sub["c5"] = bench_pipeline(pa)
            res["sub_records"] = sub
            res["sub_records_s"] = round(time.time() - t0, 1)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
