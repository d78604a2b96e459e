#!/usr/bin/env python3
"""Benchmark of the CHESS decode hot path on one MI355X.

A step is one pass of the whole path over one batch: tail-page summary refresh, cascade selection,
block-sparse decode attention and the split merge, with K/V, summaries and queries already resident
in HBM.  The timed step is the single-launch entry point (chess_decode_step with refresh_tail: tail
refresh, selection, attention and merge in one kernel); the same step through the three separate calls
(chess_summarize_tail, chess_select, chess_sparse_decode) is timed beside it.  Consecutive steps rotate over independent KV pools ("layers") and query sets so that the
bytes a step touches were not touched by the steps just before it (the set cycled through is larger
than the last-level cache); the K timed steps are captured once as a HIP graph and replayed.

Prints ONE JSON line: the step time in microseconds (the metric), the dominant kernel's HBM roofline
from HIP-event timing of that kernel alone, the dense full-KV kernel of this library on the same inputs,
and the CPU oracle timed on the host cores for the same step.  Further objects on the same line, each timed the
same way: `us_per_step_spread` (p10 / median / p90 over separately timed replays), `summarize_full_pass`,
`shared_scope` (the paper's model-wide selection over --shared-layers layers), `steady_state` (reuse and reselect
steps of the paper's operating point), `trigger` (the Sec. 3.3 monitor), `bf16_summaries` (the same step with the
summary vectors stored as bf16: half the bytes the selection reads).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E datasheet bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="cfg4a", choices=["cfg1", "cfg2", "cfg3", "cfg4a", "cfg4b", "cfg5"])
    ap.add_argument("--pools", type=int, default=0, help="independent KV pools rotated through (0 = auto)")
    ap.add_argument("--queries", type=int, default=0, help="query sets per pool (0 = auto)")
    ap.add_argument("--eager", action="store_true", help="launch step by step instead of replaying a HIP graph")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense full-KV comparison")
    ap.add_argument("--shared-layers", type=int, default=32,
                    help="layers of the model-wide selection timed beside the step (0 = skip)")
    ap.add_argument("--batch", type=int, default=0, help="sequences per step instead of the workload's own batch")
    ap.add_argument("--fanout", default="", help="NcxNg: pages per chunk x chunks per grid instead of the workload's 8x8")
    ap.add_argument("--cluster", type=int, default=0,
                    help="tuning aid: force the workgroups per (sequence, KV head) of select / decode_step (0 = automatic)")
    ap.add_argument("--summary-dtype", default="fp32", choices=["fp32", "bf16"],
                    help="storage type of the summary vectors for the headline step (the other one is timed beside it)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def algorithmic_bytes(sp, seq_lens, nsel, counts, elem=4):
    """Bytes the method must move per step (one pool): select = vectors of the units it scores (lazily: all grids,
    the chunks of kept grids, the pages of kept chunks), attention = K and V of the listed pages, summarize = the tail
    page + the child vectors re-read.  elem = bytes per summary element (4: fp32, 2: bf16)."""
    d, B, Nc, Ng = sp.head_dim, sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    sel = 0
    for b, L in enumerate(seq_lens):
        P = -(-L // B)
        ng = -(-(-(-P // Nc)) // Ng)
        for h in range(sp.n_kv_heads):
            kg, kc, _ = counts[b][h]
            sel += (ng + kg * Ng + kc * Nc) * d * elem
    attn = int(nsel.sum()) * B * d * 2 * 2
    summ = len(seq_lens) * sp.n_kv_heads * (B * d * 2 + (Nc + Ng + 3) * d * elem)
    return {"select": sel, "attention": attn, "summarize": summ, "step": sel + attn + summ}


def shared_scope(lib, sp, seq_lens, lens, plan, n_layers, timed):
    """The paper's own scope (Sec. 3.1 Eq. 1, Sec. 3.2 Eq. 3): anchors of n_layers layers + one selection per sequence
    for the whole model, on this workload's lengths.  The summary buffers hold seeded normal vectors (the
    selection reads nothing else; n_layers KV pools of this size would not add information)."""
    import torch
    gen = torch.Generator(device="cuda").manual_seed(20732)
    summs, probes = [], []
    for _ in range(n_layers):
        s = lib.new_summaries()
        for t in lib.summary_views(s):
            t.normal_(generator=gen)
        summs.append(s)
        probes.append(torch.empty((sp.batch, sp.n_kv_heads, sp.head_dim), device="cuda"))
    ws = lib.new_workspace()
    ids = torch.empty((sp.batch, sp.n_kv_heads, sp.max_selected), dtype=torch.int32, device="cuda")
    nsel = torch.empty((sp.batch, sp.n_kv_heads), dtype=torch.int32, device="cuda")

    torch.cuda.synchronize()        # the fills ran on another stream; a cluster needs the device to itself

    def both(i):
        lib.anchor(summs, seq_lens, plan.window_pages, probes)
        lib.select_shared(probes, summs, seq_lens, plan, ids, nsel, ws)

    def anchors(i):
        lib.anchor(summs, seq_lens, plan.window_pages, probes)

    ms, _ = timed(both, 8, 2, True)
    ms_a, _ = timed(anchors, 8, 2, True)
    if lib.workspace_error(ws) != 0:
        raise RuntimeError("the model-wide selection gave up a bounded wait")
    d, B, Nc, Ng = sp.head_dim, sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    units = 0
    for L in lens:
        P = -(-L // B); nc = -(-P // Nc); ng = -(-nc // Ng)
        k = sp.budget_for(P)
        kct = -(-plan.over_chunk * k // Nc)
        kg = min(ng, -(-plan.over_grid * kct // Ng))
        kc = min(kct, kg * Ng, nc)
        units += (ng if kg < ng else 0) + (kg * Ng if kc < min(kg * Ng, nc) else 0) + kc * Nc + plan.window_pages
    byts = units * n_layers * sp.n_kv_heads * d * (2 if lib.cfg.summary_dtype == 1 else 4)
    sel_ms = ms - ms_a
    return {"layers": n_layers, "us_per_selection": round(ms * 1e3, 1), "anchors_us": round(ms_a * 1e3, 1),
            "us_per_layer": round(ms * 1e3 / n_layers, 2), "algorithmic_bytes": byts,
            "gbs": round(byts / (ms * 1e-3) / 1e9, 1), "frac_of_hbm_peak": round(byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "data": "seeded normal summary vectors", "selection_alone_us": round(sel_ms * 1e3, 1)}


def steady_state(lib, sp, plan, pools, summs, n_pools, n_q, out, ws, timed, steps, pages_between=10):
    """The paper's operating point (Sec. 3.3, App. on reconstruction: a reselection about every 10 generated pages).
    Two step types, each timed cache-cold over the same rotation as the main step:
    reuse step = chess_reuse_step: append one token, extend the list's window and attend over the kept list, one launch
    (chess_append_kv + chess_sparse_decode timed beside it);
    reselect step = summaries of the pages generated since the last selection + the fused step.
    `us_per_step_at_interval` combines them for a reselection every pages_between * page_size steps."""
    import torch
    H, d = sp.n_kv_heads, sp.head_dim
    lists = {}
    for pi in range(n_pools):
        wl, qs = pools[pi]
        for qi in range(n_q):
            ids = torch.empty((sp.batch, H, sp.max_selected), dtype=torch.int32, device="cuda")
            nsel = torch.empty((sp.batch, H), dtype=torch.int32, device="cuda")
            lib.decode_step(qs[qi], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summs[pi], plan, ids, nsel, out, ws)
            lists[(pi, qi)] = (ids, nsel)
    rows_k = torch.randn((sp.batch, H, d), device="cuda").to(torch.bfloat16)
    rows_v = torch.randn((sp.batch, H, d), device="cuda").to(torch.bfloat16)
    before = [(pools[pi][0].seq_lens - 1).clamp_(min=0) for pi in range(n_pools)]        # the append rewrites the last token
    torch.cuda.synchronize()

    def reuse(i):
        pi, qi = i % n_pools, (i // n_pools) % n_q
        wl, qs = pools[pi]
        ids, nsel = lists[(pi, qi)]
        lib.reuse_step(qs[qi], rows_k, rows_v, wl.k_pool, wl.v_pool, wl.block_table, before[pi], ids, nsel, out, ws)

    def reuse_two_calls(i):
        pi, qi = i % n_pools, (i // n_pools) % n_q
        wl, qs = pools[pi]
        ids, nsel = lists[(pi, qi)]
        lib.append_kv(rows_k, rows_v, wl.k_pool, wl.v_pool, wl.block_table, before[pi], ids, nsel)
        lib.sparse_decode(qs[qi], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, ids, nsel, out, ws)

    def reselect(i):
        pi, qi = i % n_pools, (i // n_pools) % n_q
        wl, qs = pools[pi]
        ids, nsel = lists[(pi, qi)]
        lib.summarize_recent(wl.k_pool, wl.block_table, wl.seq_lens, pages_between, summs[pi])
        lib.decode_step(qs[qi], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summs[pi], plan, ids, nsel, out, ws,
                        refresh_tail=True)

    ms_reuse, _ = timed(reuse, steps, 8, True)
    ms_reuse2, _ = timed(reuse_two_calls, steps, 8, True)
    ms_resel, _ = timed(reselect, min(steps, 64), 4, True)
    interval = pages_between * sp.page_size
    avg = ((interval - 1) * ms_reuse + ms_resel) / interval
    return {"reuse_step_us": round(ms_reuse * 1e3, 2), "reselect_step_us": round(ms_resel * 1e3, 2),
            "reselect_every_steps": interval, "us_per_step_at_interval": round(avg * 1e3, 2),
            "reuse_step_as_two_calls_us": round(ms_reuse2 * 1e3, 2),
            "kernel_launches": {"reuse_step": 1, "reselect_step": 2}}


def trigger_monitor(lib, sp, timed, vocab=151936):
    """Sec. 3.3 monitor per decode step: entropy of the batch's logits rows (bf16, a 152K vocabulary) + page statistics."""
    import torch
    logits = [torch.randn((sp.batch, vocab), device="cuda").mul_(3).to(torch.bfloat16) for _ in range(4)]
    H = torch.empty((sp.batch,), device="cuda")
    ws = lib.new_workspace()
    hist = torch.zeros((sp.batch, sp.page_size), device="cuda")
    count = torch.zeros((sp.batch,), dtype=torch.int32, device="cuda")
    fire = torch.zeros((sp.batch,), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def monitor(i):
        lib.monitor_step(logits[i % 4], sp.page_size, 1e9, 1e9, H, hist, count, fire, ws)

    ms, _ = timed(monitor, 64, 4, True)
    byts = sp.batch * vocab * 2
    return {"us_per_step": round(ms * 1e3, 2), "logit_bytes": byts, "gbs": round(byts / (ms * 1e-3) / 1e9, 1),
            "vocab": vocab, "kernel_launches_per_step": 1}


TRAFFIC_FILE = os.path.join("profiles", "step_kernel_hbm_traffic.txt")


def measured_traffic(workload_name, summary_dtype):
    """HBM bytes per launch of the step kernel from the committed rocprofv3 counter summary (a separate run of this
    script under rocprofv3 --pmc, see the file's header: not measured in this run), or None."""
    key = workload_name + ("_bf16" if summary_dtype == "bf16" else "")
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_FILE)):
            f = line.split()
            if len(f) >= 5 and f[0] == key:
                return int((float(f[1]) * float(f[3]) + float(f[2]) * float(f[4])) * 1024)
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2602_20732_amd as pk
    import workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    sp = workload.spec(args.workload)
    if args.batch > 0:
        import dataclasses
        sp = dataclasses.replace(sp, batch=args.batch)
    if args.fanout:
        import dataclasses
        nc_, ng_ = (int(x) for x in args.fanout.lower().split("x"))
        sp = dataclasses.replace(sp, pages_per_chunk=nc_, chunks_per_grid=ng_)
    seed = workload.default_seed(args.workload)
    pool_bytes = sp.batch * sp.ctx[1] * sp.n_kv_heads * sp.head_dim * 2 * 2
    # ~2 GB of KV, at least 2 pools; cfg3 is defined as a stack of 32 layers with their own KV (about 100 GB)
    n_pools = args.pools or (32 if args.workload == "cfg3" else max(2, min(16, int(2.2e9 // pool_bytes))))
    n_q = args.queries or max(1, 16 // n_pools)

    t0 = time.time()
    lens = workload.seq_lengths(sp, seed)
    pools = []
    for l in range(n_pools):
        wl = workload.generate(sp, seed, layer=l, device="cuda", seq_lens=lens)
        qs = [wl.q] + [workload.extra_queries(wl, v) for v in range(1, n_q)]
        pools.append((wl, qs))
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    dt_code = {"fp32": pk.SUMMARY_F32, "bf16": pk.SUMMARY_BF16}
    other_dtype = "bf16" if args.summary_dtype == "fp32" else "fp32"
    cfg = pk.Config(sp.n_q_heads, sp.n_kv_heads, sp.page_size, sp.batch, sp.max_pages, sp.max_selected,
                    sp.pages_per_chunk, sp.chunks_per_grid, summary_dtype=dt_code[args.summary_dtype])
    lib = pk.Chess(cfg)
    lib.debug_force_cluster(args.cluster)
    plan = pk.SelectPlan(sink_pages=sp.sink_pages, window_pages=sp.window_pages, budget_pages=sp.budget_pages,
                         budget_bp=sp.budget_bp)
    summs = []
    for wl, _ in pools:                                   # prefill-time full pass, outside the timed region
        s = lib.new_summaries()
        lib.summarize(wl.k_pool, wl.block_table, wl.seq_lens, s)
        summs.append(s)
    ws = lib.new_workspace()
    ids = torch.empty((sp.batch, sp.n_kv_heads, sp.max_selected), dtype=torch.int32, device="cuda")
    nsel = torch.empty((sp.batch, sp.n_kv_heads), dtype=torch.int32, device="cuda")
    out = torch.empty((sp.batch, sp.n_q_heads, sp.head_dim), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    def step(i):
        wl, qs = pools[i % n_pools]
        q = qs[(i // n_pools) % n_q]
        s = summs[i % n_pools]
        lib.decode_step(q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, s, plan, ids, nsel, out, ws,
                        refresh_tail=True)

    def step_three_calls(i):
        wl, qs = pools[i % n_pools]
        q = qs[(i // n_pools) % n_q]
        s = summs[i % n_pools]
        lib.summarize_tail(wl.k_pool, wl.block_table, wl.seq_lens, s)
        lib.select(q, s, wl.seq_lens, plan, ids, nsel, ws)
        lib.sparse_decode(q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, ids, nsel, out, ws)

    def dense_step(i):
        wl, qs = pools[i % n_pools]
        lib.dense_decode(qs[(i // n_pools) % n_q], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, out, ws)

    def timed(fn, steps, warmup, graph):
        """Time exactly `steps` calls of fn after `warmup` untimed ones; returns ms per step."""
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            for i in range(warmup):
                fn(i)
            stream.synchronize()
            g = None
            if graph:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for i in range(steps):
                        fn(warmup + i)
                g.replay()                                 # untimed: first replay pays graph upload
                stream.synchronize()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t_wall = time.perf_counter()
            e0.record(stream)
            if g is not None:
                g.replay()
            else:
                for i in range(steps):
                    fn(warmup + i)
            e1.record(stream)
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t_wall) * 1e3
        return max(e0.elapsed_time(e1), 0.0) / steps, wall_ms / steps

    def spread(fn, block=16, replays=32):
        """p10 / median / p90 of the time per step over `replays` separately timed replays of a `block`-step graph."""
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            for i in range(block):
                fn(i)
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for i in range(block):
                    fn(i)
            g.replay()
            stream.synchronize()
            ts = []
            for _ in range(replays):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                g.replay()
                e1.record(stream)
                stream.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3 / block)
        ts.sort()
        pick = lambda f: round(ts[min(len(ts) - 1, int(f * len(ts)))], 3)
        return {"p10": pick(0.1), "median": pick(0.5), "p90": pick(0.9), "steps_per_sample": block, "samples": replays}

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_step, wall_ms_step = timed(step, args.steps, args.warmup, not args.eager)
    ms_three, _ = timed(step_three_calls, args.steps, min(args.warmup, 8), not args.eager)
    step_spread = None if args.eager else spread(step)

    # the full summarize pass (prefill time, not part of the step): a pure stream of the K pool
    def full_summarize(i):
        wl, _ = pools[i % n_pools]
        lib.summarize(wl.k_pool, wl.block_table, wl.seq_lens, summs[i % n_pools])

    ms_full, _ = timed(full_summarize, max(2, min(8, n_pools * 2)), 1, False)

    # per-phase durations: each phase alone, same rotation, replayed as its own HIP graph and timed with
    # HIP events on the launch stream (inside a graph the gaps between kernels are negligible, so the
    # time per launch is the kernel duration a kernel trace shows)
    n_slots = n_pools * n_q
    slot_ids = [torch.empty_like(ids) for _ in range(n_slots)]
    slot_nsel = [torch.empty_like(nsel) for _ in range(n_slots)]
    for j in range(n_slots):
        wl, qs = pools[j % n_pools]
        lib.select(qs[(j // n_pools) % n_q], summs[j % n_pools], wl.seq_lens, plan, slot_ids[j], slot_nsel[j], ws)
    torch.cuda.synchronize()

    def only_tail(i):
        wl, _ = pools[i % n_pools]
        lib.summarize_tail(wl.k_pool, wl.block_table, wl.seq_lens, summs[i % n_pools])

    def only_select(i):
        wl, qs = pools[i % n_pools]
        lib.select(qs[(i // n_pools) % n_q], summs[i % n_pools], wl.seq_lens, plan, ids, nsel, ws)

    def only_decode(i):
        wl, qs = pools[i % n_pools]
        j = i % n_slots
        lib.sparse_decode(qs[(i // n_pools) % n_q], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, slot_ids[j],
                          slot_nsel[j], out, ws)

    def only_fused(i):
        wl, qs = pools[i % n_pools]
        lib.decode_step(qs[(i // n_pools) % n_q], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summs[i % n_pools],
                        plan, ids, nsel, out, ws, refresh_tail=True)

    kern, kern3 = {}, {}
    for dst, name, fn in ((kern, "decode_step", only_fused), (kern3, "summarize_tail", only_tail),
                          (kern3, "select", only_select), (kern3, "sparse_decode", only_decode)):
        ms, _ = timed(fn, args.steps, min(args.warmup, 8), not args.eager)
        dst[name] = {"us_per_step": round(ms * 1e3, 3), "kernel_launches_per_step": 1}
    step(0)
    torch.cuda.synchronize()

    # bytes: keep-counts and list lengths of the last profiled step, from the device results
    nsel_h = nsel.cpu().numpy()
    B, Nc, Ng = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    counts = []
    for b, L in enumerate(lens):
        P = -(-L // B)
        k = sp.budget_for(P)
        kct = -(-plan.over_chunk * k // Nc)
        nc = -(-P // Nc)
        kg = min(-(-nc // Ng), -(-plan.over_grid * kct // Ng))
        counts.append([(kg, min(kct, kg * Ng, nc), k)] * sp.n_kv_heads)
    elem = {"fp32": 4, "bf16": 2}
    ab = algorithmic_bytes(sp, lens, nsel_h, counts, elem[args.summary_dtype])
    fused_us = kern["decode_step"]["us_per_step"]

    # the same step with the summaries stored the other way (its own context and summary buffers, same inputs)
    import dataclasses
    lib2 = pk.Chess(dataclasses.replace(cfg, summary_dtype=dt_code[other_dtype]))
    lib2.debug_force_cluster(args.cluster)
    summs2 = []
    for wl, _ in pools:
        s2 = lib2.new_summaries()
        lib2.summarize(wl.k_pool, wl.block_table, wl.seq_lens, s2)
        summs2.append(s2)
    ws2 = lib2.new_workspace()
    torch.cuda.synchronize()

    def only_fused_other(i):
        wl, qs = pools[i % n_pools]
        lib2.decode_step(qs[(i // n_pools) % n_q], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summs2[i % n_pools],
                         plan, ids, nsel, out, ws2, refresh_tail=True)

    ms_other, _ = timed(only_fused_other, args.steps, min(args.warmup, 8), not args.eager)
    if lib2.workspace_error(ws2) != 0:
        raise RuntimeError("a kernel gave up a bounded wait during the timed steps (was the device shared?)")
    ab_other = algorithmic_bytes(sp, lens, nsel.cpu().numpy(), counts, elem[other_dtype])
    del summs2, ws2
    lib2.close()
    achieved = ab["step"] / (fused_us * 1e-6) / 1e9
    dec_us = kern3["sparse_decode"]["us_per_step"]
    result = {
        "metric": "sparse decode attn us/step (tail summarize + select + sparse attention + merge), 1% KV budget",
        "value": round(ms_step * 1e3, 3), "unit": "us/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 K/V/q, fp32 accumulate, fp64 scores, %s summaries" % args.summary_dtype, "data": "synthetic",
        "config": {"workload": args.workload, "batch": sp.batch, "context": list(sp.ctx), "n_q_heads": sp.n_q_heads,
                   "n_kv_heads": sp.n_kv_heads, "page_size": sp.page_size, "budget_bp": sp.budget_bp,
                   "budget_pages": sp.budget_pages, "sink_pages": sp.sink_pages, "window_pages": sp.window_pages,
                   "pages_per_chunk": Nc, "chunks_per_grid": Ng, "summary_dtype": args.summary_dtype,
                   "kv_pools_rotated": n_pools,
                   "query_sets_per_pool": n_q, "launch": "eager" if args.eager else "hip_graph"},
        "step_gbs": round(ab["step"] / (ms_step * 1e-3) / 1e9, 1),
        "step_frac_of_hbm_peak": round(ab["step"] / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "wall_us_per_step": round(wall_ms_step * 1e3, 3),
        "us_per_step_spread": step_spread,
        "algorithmic_bytes": ab,
        "kernels": kern,
        "three_calls": {"us_per_step": round(ms_three * 1e3, 3), "kernels": kern3,
                        "sparse_decode_gbs": round(ab["attention"] / (dec_us * 1e-6) / 1e9, 1)},
        "roofline": {"bound": "hbm", "kernel": "step_kernel (tail refresh + selection levels + sparse attention over the list + split merge)",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(args.workload, args.summary_dtype),
                     "traffic_source": "committed counter summary " + TRAFFIC_FILE + " (rocprofv3 --pmc runs of this script, "
                                       "not this run; the runs behind it rotate over fewer KV pools, see the file's header)"},
        other_dtype + "_summaries": {"us_per_step": round(ms_other * 1e3, 3), "algorithmic_bytes": ab_other,
                                     "gbs": round(ab_other["step"] / (ms_other * 1e-3) / 1e9, 1),
                                     "frac_of_hbm_peak": round(ab_other["step"] / (ms_other * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                     "timed_as": "the fused step alone in its own HIP graph, like roofline.achieved"},
        "setup_seconds": round(gen_s, 1),
    }

    B_, d_ = sp.page_size, sp.head_dim
    e_ = elem[args.summary_dtype]
    full_bytes = sum(-(-L // B_) for L in lens) * sp.n_kv_heads * (B_ * d_ * 2 + d_ * e_) \
        + sum(-(-(-(-L // B_)) // sp.pages_per_chunk) for L in lens) * sp.n_kv_heads * d_ * e_
    result["summarize_full_pass"] = {"us": round(ms_full * 1e3, 1), "bytes": full_bytes,
                                     "gbs": round(full_bytes / (ms_full * 1e-3) / 1e9, 1),
                                     "frac_of_hbm_peak": round(full_bytes / (ms_full * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    if args.shared_layers > 0:
        result["shared_scope"] = shared_scope(lib, sp, pools[0][0].seq_lens, lens, plan, args.shared_layers, timed)
    result["trigger"] = trigger_monitor(lib, sp, timed)
    result["steady_state"] = steady_state(lib, sp, plan, pools, summs, n_pools, n_q, out, ws, timed, args.steps)
    if args.workload == "cfg3":
        result["stack_of_32_layers_us"] = round(ms_step * 1e3 * 32, 1)

    if not args.no_dense:
        d_steps = max(8, min(args.steps, 32))
        d_ms, _ = timed(dense_step, d_steps, 2, not args.eager)
        dense_bytes = sum(-(-L // B) for L in lens) * sp.n_kv_heads * B * sp.head_dim * 4
        result["dense"] = {"us_per_step": round(d_ms * 1e3, 2), "gbs": round(dense_bytes / (d_ms * 1e-3) / 1e9, 1),
                           "frac_of_hbm_peak": round(dense_bytes / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                           "bytes": dense_bytes, "sparse_speedup": round(d_ms / ms_step, 2)}

    # a cluster that gave up a bounded wait would have produced undefined results: no number is printed then
    if lib.workspace_error(ws) != 0:
        raise RuntimeError("a kernel gave up a bounded wait during the timed steps (was the device shared?)")

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(sp, pools[0][0], plan, dt_code[args.summary_dtype])

    print(json.dumps(result))


def cpu_baseline(sp, wl, plan, summary_dtype=0):
    """The oracle as it stands, on the host cores: full summarize + select + sparse attention for a bounded sample
    of the batch (whole sequences), scaled to the batch.  `value` is one thread; `all_cores` runs the same sample
    with one thread per sequence (the oracle is a plain C library called through ctypes, which releases the
    interpreter lock, so the threads run in parallel)."""
    import numpy as np

    import oracle
    import workload

    n_seq = max(1, min(sp.batch, int(2 ** 21 // max(1, sp.ctx[1]))))      # ~2M tokens of summarize at most
    geom = oracle.Geometry(sp.n_q_heads, sp.n_kv_heads, sp.head_dim, sp.page_size, sp.pages_per_chunk,
                           sp.chunks_per_grid, sp.max_pages, summary_dtype)
    oplan = oracle.Plan(sink_pages=plan.sink_pages, window_pages=plan.window_pages, budget_pages=plan.budget_pages,
                        budget_bp=plan.budget_bp)
    bt = wl.block_table[:n_seq].cpu()
    sl = wl.seq_lens[:n_seq].cpu().numpy()
    # gather the sample's pages into a compact host pool (identity block table)
    P = [-(-int(n) // sp.page_size) for n in sl]
    phys = np.concatenate([bt[b, :P[b]].numpy() for b in range(n_seq)])
    import torch
    idx = torch.as_tensor(phys, dtype=torch.long, device=wl.k_pool.device)
    K = workload.bf16_bits(wl.k_pool[idx])
    V = workload.bf16_bits(wl.v_pool[idx])
    Q = workload.bf16_bits(wl.q[:n_seq])
    bt2 = np.full((n_seq, sp.max_pages), -1, np.int32)
    off = 0
    for b in range(n_seq):
        bt2[b, :P[b]] = np.arange(off, off + P[b])
        off += P[b]
    oracle.build()

    def one_pass():
        t0 = time.perf_counter()
        pv, cv, gv = oracle.summarize(K, bt2, sl, geom)
        t1 = time.perf_counter()
        ids, nsel = oracle.select(Q, pv, cv, gv, sl, geom, oplan, sp.max_selected)
        t2 = time.perf_counter()
        oracle.attend(Q, K, V, bt2, sl, geom, ids, nsel)
        t3 = time.perf_counter()
        return t1 - t0, t2 - t1, t3 - t2

    # repeat the sample's step until about 10 s of CPU work have been timed; report the mean pass
    first = one_pass()
    reps = max(1, min(64, int(10.0 / max(sum(first), 1e-3))))
    passes = [first] + [one_pass() for _ in range(reps - 1)]
    t_sum, t_sel, t_att = (sum(p[i] for p in passes) / len(passes) for i in range(3))
    t0, t1, t2, t3 = 0.0, t_sum, t_sum + t_sel, t_sum + t_sel + t_att
    scale = sp.batch / n_seq

    # the same sample on all cores: one thread per sequence
    from concurrent.futures import ThreadPoolExecutor
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    n_thr = max(1, min(n_seq, avail))

    def one_seq(b):
        sl1, bt1 = sl[b:b + 1], bt2[b:b + 1]
        pv, cv, gv = oracle.summarize(K, bt1, sl1, geom)
        ids, nsel = oracle.select(Q[b:b + 1], pv, cv, gv, sl1, geom, oplan, sp.max_selected)
        oracle.attend(Q[b:b + 1], K, V, bt1, sl1, geom, ids, nsel)

    tp0 = time.perf_counter()
    with ThreadPoolExecutor(n_thr) as ex:
        list(ex.map(one_seq, range(n_seq)))
    t_par = time.perf_counter() - tp0
    all_cores = {"value": round(t_par * scale * 1e6, 1), "unit": "us/step", "cores": n_thr,
                 "sample": f"the same {n_seq} sequences, one thread each, one pass"}
    return {"value": round((t3 - t0) * scale * 1e6, 1), "unit": "us/step", "cores": 1, "kind": "oracle", "all_cores": all_cores,
            "sample": f"{n_seq} of {sp.batch} sequences, mean of {len(passes)} passes, whole step (full-pass summarize {t1 - t0:.2f}s, select "
                      f"{t2 - t1:.3f}s, sparse attention {t3 - t2:.3f}s), scaled x{scale:g} to the batch; the oracle "
                      "has no incremental summarize, so its step re-summarizes the whole context",
            "select_plus_attention_us": round((t3 - t1) * scale * 1e6, 1)}


if __name__ == "__main__":
    main()
