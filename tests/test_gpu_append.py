"""The decode loop's append: chess_append_kv writes one token per sequence into the paged pools; after every step
the pools must hold exactly the logical rows (checked through the test-side unpacking, which knows the two
layouts independently), and the summaries refreshed from them must equal a full pass over the grown sequence."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2602_20732_amd as pk
import workload
from gpu_common import host_views, config_of, gpu_plan, to_device
from helpers import bf16_to_f64, geom_of, logical_kv, plan_of

pytestmark = pytest.mark.gpu


def test_append_grows_the_cache_and_the_step_follows_it():
    sp = workload.WorkloadSpec("grow", 3, (0, 1200), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_pages=5,
                               pages_per_chunk=4, chunks_per_grid=4)
    start, steps = [1000, 527, 0], 40                        # crosses page, chunk and grid boundaries; one starts empty
    full = workload.generate(sp, 11, seq_lens=[n + steps for n in start])     # the grown sequences, as a reference
    d = to_device(full)
    K, V = workload.bf16_bits(full.k_pool), workload.bf16_bits(full.v_pool)
    bt = full.block_table.numpy()
    g = geom_of(sp)
    lib = pk.Chess(config_of(sp, max_selected=sp.max_pages))
    # the caches start as the first `start` tokens: everything behind them is poisoned
    k_pool, v_pool = d.k_pool.clone(), d.v_pool.clone()
    B = sp.page_size
    for b, n in enumerate(start):
        for j in range(n // B, -(-(n + steps) // B)):
            phys = int(bt[b, j])
            t0 = max(n - j * B, 0)
            k_pool[phys, :, t0:, :] = float("nan")
            v_pool[phys, :, :, t0:] = float("nan")
    lens = torch.tensor(start, dtype=torch.int32, device="cuda")
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(k_pool, d.block_table, lens, summ)
    plan = plan_of(sp)
    ids = torch.empty((3, sp.n_kv_heads, sp.max_pages), dtype=torch.int32, device="cuda")
    nsel = torch.empty((3, sp.n_kv_heads), dtype=torch.int32, device="cuda")
    out = torch.empty((3, sp.n_q_heads, 128), device="cuda")
    for step in range(steps):
        rows_k = torch.empty((3, sp.n_kv_heads, 128), dtype=torch.bfloat16, device="cuda")
        rows_v = torch.empty_like(rows_k)
        for b, n in enumerate(start):                         # the next token's rows, taken from the reference pools
            pos = n + step
            phys = int(bt[b, pos // B])
            rows_k[b] = d.k_pool[phys, :, pos % B, :]
            rows_v[b] = d.v_pool[phys, :, :, pos % B]
        lib.append_kv(rows_k, rows_v, k_pool, v_pool, d.block_table, lens)
        lens += 1
        lib.decode_step(d.q, k_pool, v_pool, d.block_table, lens, summ, gpu_plan(plan), ids, nsel, out, ws, refresh_tail=True)
        if step in (0, 11, 23, steps - 1):
            torch.cuda.synchronize()
            assert lib.workspace_error(ws) == 0
            Kh, Vh = workload.bf16_bits(k_pool.cpu()), workload.bf16_bits(v_pool.cpu())
            sl = lens.cpu().numpy()
            for b in range(3):
                for h in range(sp.n_kv_heads):
                    got_k, got_v = logical_kv(Kh, Vh, bt, sl[b], b, h)
                    ref_k, ref_v = logical_kv(K, V, bt, sl[b], b, h)
                    assert np.array_equal(got_k, ref_k) and np.array_equal(got_v, ref_v), (step, b, h)
            # summaries kept current by the per-step refresh == the oracle's full pass over the grown prefix
            rp, rc, rg = oracle.summarize(K, bt, sl, g)
            pv, cv, gv = host_views(lib, summ, 3)
            for b in range(3):
                P = -(-int(sl[b]) // B); nc = -(-P // 4); ng = -(-nc // 4)
                assert np.array_equal(pv[b, :, :P], rp[b, :, :P]) and np.array_equal(cv[b, :, :nc], rc[b, :, :nc])
                assert np.array_equal(gv[b, :, :ng], rg[b, :, :ng]), (step, b)
            Q = workload.bf16_bits(full.q)
            rids, rn = oracle.select(Q, rp, rc, rg, sl, g, plan, sp.max_pages)
            rout = oracle.attend(Q, K, V, bt, sl, g, rids, rn)
            assert np.array_equal(ids.cpu().numpy(), rids) and np.array_equal(nsel.cpu().numpy(), rn), step
            assert np.abs(out.cpu().numpy() - rout).max() <= 2e-3
    # a full sequence is left alone
    lens_full = torch.tensor([sp.max_pages * B] * 3, dtype=torch.int32, device="cuda")
    before = k_pool.clone()
    lib.append_kv(rows_k, rows_v, k_pool, v_pool, d.block_table, lens_full)
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), k_pool.view(torch.int16))
    lib.close()


def test_list_reuse_between_reselections_follows_the_tail():
    """The paper's operating point (Sec. 3.3): select once, then decode for several pages with the same list while the
    cache grows.  chess_extend_window keeps the recent pages in the list; each step's attention equals the oracle's
    attention over (list at selection time) + (every page generated since)."""
    sp = workload.WorkloadSpec("reuse", 2, (0, 1400), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_pages=5,
                               pages_per_chunk=4, chunks_per_grid=4)
    start, steps = [1200, 700], 50
    full = workload.generate(sp, 21, seq_lens=[n + steps for n in start])
    d = to_device(full)
    K, V, Q = workload.bf16_bits(full.k_pool), workload.bf16_bits(full.v_pool), workload.bf16_bits(full.q)
    bt = full.block_table.numpy()
    g = geom_of(sp)
    B = sp.page_size
    room = 1 + 5 + 2 + -(-steps // B) + 1
    lib = pk.Chess(config_of(sp, max_selected=room))
    plan = plan_of(sp)
    lens = torch.tensor(start, dtype=torch.int32, device="cuda")
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(d.k_pool, d.block_table, lens, summ)
    ids = torch.empty((2, sp.n_kv_heads, room), dtype=torch.int32, device="cuda")
    nsel = torch.empty((2, sp.n_kv_heads), dtype=torch.int32, device="cuda")
    out = torch.empty((2, sp.n_q_heads, 128), device="cuda")
    lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, lens, summ, gpu_plan(plan), ids, nsel, out, ws)
    torch.cuda.synchronize()
    ids0, n0 = ids.cpu().numpy().copy(), nsel.cpu().numpy().copy()
    rp, rc, rg = oracle.summarize(K, bt, np.array(start, np.int32), g)
    rids, rn = oracle.select(Q, rp, rc, rg, np.array(start, np.int32), g, plan, room)
    assert np.array_equal(ids0, rids) and np.array_equal(n0, rn)
    for step in range(1, steps + 1):
        if step % 2:                                       # the two ways to extend a list: a call of its own ...
            lens += 1                                      # (the pools already hold the rows)
            lib.extend_window(lens, ids, nsel)
        else:                                              # ... or inside the append (which rewrites the row that is there)
            rows_k = torch.stack([d.k_pool[int(bt[b, int(lens[b]) // B]), :, int(lens[b]) % B, :] for b in range(2)])
            rows_v = torch.stack([d.v_pool[int(bt[b, int(lens[b]) // B]), :, :, int(lens[b]) % B] for b in range(2)])
            lib.append_kv(rows_k.contiguous(), rows_v.contiguous(), d.k_pool, d.v_pool, d.block_table, lens, ids, nsel)
            lens += 1
        lib.sparse_decode(d.q, d.k_pool, d.v_pool, d.block_table, lens, ids, nsel, out, ws)
        if step in (1, 15, 16, 17, 33, steps):
            sl = lens.cpu().numpy()
            want_ids = np.full_like(rids, -1)
            want_n = np.zeros_like(rn)
            for b in range(2):
                P = -(-int(sl[b]) // B)
                for h in range(sp.n_kv_heads):
                    row = rids[b, h, :rn[b, h]].tolist()
                    row += list(range(row[-1] + 1, P))
                    want_ids[b, h, :len(row)] = row
                    want_n[b, h] = len(row)
            got_ids, got_n = ids.cpu().numpy(), nsel.cpu().numpy()
            assert np.array_equal(got_n, want_n), step
            for b in range(2):
                for h in range(sp.n_kv_heads):
                    assert np.array_equal(got_ids[b, h, :got_n[b, h]], want_ids[b, h, :want_n[b, h]]), (step, b, h)
            ref = oracle.attend(Q, K, V, bt, sl, g, want_ids, want_n)
            assert np.abs(out.cpu().numpy() - ref).max() <= 2e-3, step
    # a row that is full stops growing and stays valid
    small = pk.Chess(config_of(sp, max_selected=9))
    ids9 = torch.as_tensor(np.ascontiguousarray(rids[:, :, :9])).cuda()
    n9 = torch.as_tensor(np.minimum(rn, 9)).cuda()
    small.extend_window(lens, ids9, n9)
    torch.cuda.synchronize()
    assert int(n9.max()) == 9 and int(ids9.max()) < -(-int(lens.max()) // B)
    small.close()
    lib.close()


def test_the_decode_loop_in_a_hip_graph_replays_like_eager():
    """One iteration of the loop around the step -- anchors + model-wide selection, then per step: append with list
    extension, sparse attention, entropy of a logits row, trigger update -- captured once and replayed with eager
    work and synchronisations between the replays; every replay must give what the same calls give eagerly."""
    sp = workload.WorkloadSpec("loop", 2, (0, 2100), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_pages=5,
                               pages_per_chunk=4, chunks_per_grid=4)
    start = [2000, 900]
    full = to_device(workload.generate(sp, 31, seq_lens=[n + 40 for n in start]))
    room = 1 + 5 + 2 + 4
    lib = pk.Chess(config_of(sp, max_selected=room))
    plan = gpu_plan(plan_of(sp))
    H = sp.n_kv_heads
    gen = torch.Generator(device="cuda").manual_seed(5)
    logits = (torch.randn((2, 4096), device="cuda", generator=gen) * 3).to(torch.bfloat16)
    rows_k = torch.randn((2, H, 128), device="cuda", generator=gen).to(torch.bfloat16)
    rows_v = torch.randn((2, H, 128), device="cuda", generator=gen).to(torch.bfloat16)

    def fresh_state():
        st = dict(k=full.k_pool.clone(), v=full.v_pool.clone(), lens=torch.tensor(start, dtype=torch.int32, device="cuda"),
                  summ=lib.new_summaries(), ws=lib.new_workspace(), anc=torch.empty((2, H, 128), device="cuda"),
                  ids=torch.full((2, H, room), -7, dtype=torch.int32, device="cuda"),
                  nsel=torch.full((2, H), -7, dtype=torch.int32, device="cuda"),
                  out=torch.full((2, sp.n_q_heads, 128), float("nan"), device="cuda"), ent=torch.zeros((2,), device="cuda"),
                  hist=torch.zeros((2, 2), device="cuda"), count=torch.zeros((2,), dtype=torch.int32, device="cuda"),
                  fire=torch.full((2,), -1, dtype=torch.int32, device="cuda"), stats=torch.zeros((2, 2), dtype=torch.float64, device="cuda"))
        lib.summarize(st["k"], full.block_table, st["lens"], st["summ"])
        return st

    def iteration(st):
        lib.anchor(st["summ"], st["lens"], 2, st["anc"])
        lib.select_shared([st["anc"]], [st["summ"]], st["lens"], plan, st["ids"], st["nsel"], st["ws"])
        lib.append_kv(rows_k, rows_v, st["k"], st["v"], full.block_table, st["lens"], st["ids"], st["nsel"])
        st["lens"].add_(1)
        lib.sparse_decode(full.q, st["k"], st["v"], full.block_table, st["lens"], st["ids"], st["nsel"], st["out"], st["ws"])
        lib.entropy(logits, st["ent"], st["ws"])
        lib.trigger_update(st["ent"], 2, 0.5, 1e9, st["hist"], st["count"], st["fire"], st["stats"])

    # eager: three iterations (the sequences grow by one token each), results after each
    e = fresh_state()
    want = []
    for _ in range(3):
        iteration(e)
        torch.cuda.synchronize()
        want.append({k: e[k].clone() for k in ("ids", "nsel", "out", "ent", "fire", "stats", "lens", "count")})
    assert lib.workspace_error(e["ws"]) == 0
    assert int(want[1]["fire"].sum()) == 2, "the trigger must fire when its page of two steps completes"

    g = fresh_state()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        warm = fresh_state()
        iteration(warm)                                    # every kernel has run once before the capture
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            iteration(g)
        for rep in range(3):
            graph.replay()
            stream.synchronize()
            for k, v in want[rep].items():
                assert torch.equal(g[k], v), (rep, k)
            scratch = torch.empty_like(g["out"])           # eager work between the replays
            lib.dense_decode(full.q, g["k"], g["v"], full.block_table, g["lens"], scratch, g["ws"])
            stream.synchronize()
    assert lib.workspace_error(g["ws"]) == 0
    lib.close()


@pytest.mark.parametrize("page,splits", [(16, 0), (16, 1), (16, 3), (32, 0), (32, 2)])
def test_reuse_step_equals_append_then_attention(page, splits):
    """chess_reuse_step against chess_append_kv (with the lists) + chess_sparse_decode on copies of the same state,
    step after step across page boundaries (one sequence starts empty, one is full): outputs, lists and pools must be
    identical bit for bit; and the first and last steps against the oracle."""
    sp = workload.WorkloadSpec("reuse1", 4, (0, 1408), 8, 2, page, ("fixed", 128), (2, 2), 1, 2, budget_pages=5,
                               pages_per_chunk=4, chunks_per_grid=4)
    start, steps = [1200, 700 - 700 % page, 0, 1408], 2 * page + 3
    lens_full = [min(n + steps, 1408) for n in start]
    full = to_device(workload.generate(sp, 41, seq_lens=lens_full))
    room = 1 + 5 + 2 + 4
    lib = pk.Chess(config_of(sp, max_selected=room))
    lib.debug_force_splits(splits, 4)
    plan = gpu_plan(plan_of(sp))
    lens = torch.tensor(start, dtype=torch.int32, device="cuda")
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(full.k_pool, full.block_table, lens, summ)
    ids = torch.full((4, sp.n_kv_heads, room), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((4, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    lib.select(full.q, summ, lens, plan, ids, nsel, ws)
    torch.cuda.synchronize()
    bt = full.block_table
    B = page
    # state A: two calls; state B: one launch
    A = dict(k=full.k_pool.clone(), v=full.v_pool.clone(), ids=ids.clone(), nsel=nsel.clone(), lens=lens.clone(),
             out=torch.full((4, sp.n_q_heads, 128), float("nan"), device="cuda"))
    Bs = dict(k=full.k_pool.clone(), v=full.v_pool.clone(), ids=ids.clone(), nsel=nsel.clone(), lens=lens.clone(),
              out=torch.full((4, sp.n_q_heads, 128), float("nan"), device="cuda"))
    for st in (A, Bs):                                     # nothing behind the current lengths is valid yet
        for b, n in enumerate(start):
            for j in range(n // B, -(-lens_full[b] // B)):
                phys = int(bt[b, j]); t0 = max(n - j * B, 0)
                st["k"][phys, :, t0:, :] = float("nan"); st["v"][phys, :, :, t0:] = float("nan")
    gen = torch.Generator(device="cuda").manual_seed(9)
    for step in range(steps):
        rk = torch.randn((4, sp.n_kv_heads, 128), device="cuda", generator=gen).to(torch.bfloat16)
        rv = torch.randn((4, sp.n_kv_heads, 128), device="cuda", generator=gen).to(torch.bfloat16)
        lib.append_kv(rk, rv, A["k"], A["v"], bt, A["lens"], A["ids"], A["nsel"])
        A["lens"] = torch.clamp(A["lens"] + 1, max=1408)
        lib.sparse_decode(full.q, A["k"], A["v"], bt, A["lens"], A["ids"], A["nsel"], A["out"], ws)
        lib.reuse_step(full.q, rk, rv, Bs["k"], Bs["v"], bt, Bs["lens"], Bs["ids"], Bs["nsel"], Bs["out"], ws)
        Bs["lens"] = torch.clamp(Bs["lens"] + 1, max=1408)
        torch.cuda.synchronize()
        assert torch.equal(A["nsel"], Bs["nsel"]), step
        live = torch.arange(room, device="cuda").view(1, 1, -1) < A["nsel"].unsqueeze(-1)
        assert torch.equal(torch.where(live, A["ids"], -1), torch.where(live, Bs["ids"], -1)), step
        assert torch.equal(A["out"], Bs["out"]), (step, (A["out"] - Bs["out"]).abs().max())
        if step in (0, steps - 1):
            for b in range(4):
                P = -(-int(A["lens"][b]) // B)
                for j in range(P):
                    phys = int(bt[b, j]); n = min(B, int(A["lens"][b]) - j * B)
                    assert torch.equal(A["k"][phys, :, :n].view(torch.int16), Bs["k"][phys, :, :n].view(torch.int16))
                    assert torch.equal(A["v"][phys, :, :, :n].view(torch.int16), Bs["v"][phys, :, :, :n].view(torch.int16))
            K, V, Q = workload.bf16_bits(Bs["k"].cpu()), workload.bf16_bits(Bs["v"].cpu()), workload.bf16_bits(full.q.cpu())
            sl = Bs["lens"].cpu().numpy()
            ref = oracle.attend(Q, K, V, bt.cpu().numpy(), sl, geom_of(sp), Bs["ids"].cpu().numpy(), Bs["nsel"].cpu().numpy())
            assert np.abs(Bs["out"].cpu().numpy() - ref).max() <= 2e-3, step
    assert int(Bs["nsel"][2, 0]) == -(-steps // B), "the sequence that started empty has all its pages in the list"
    lib.close()


@pytest.mark.parametrize("seed", range(12))
def test_reuse_step_random_shapes(seed):
    """Seeded draws of page size, heads, group, batch, lengths (incl. empty and nearly full sequences) and split count:
    several chess_reuse_step launches against the two calls, bit for bit."""
    rng = np.random.default_rng(4000 + seed)
    B, H, G = int(rng.choice([16, 32])), int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4, 7, 16]))
    batch, hi = int(rng.integers(1, 5)), int(rng.choice([256, 1024, 3072]))
    steps = int(rng.integers(2, 2 * B + 2))
    start = [int(rng.integers(0, hi - steps + 1)) for _ in range(batch)]
    start[0] = hi - int(rng.integers(0, steps))                 # runs out of room on the way
    s, w, k = int(rng.choice([0, 1, 2])), int(rng.choice([1, 2, 3])), int(rng.integers(1, 12))
    sp = workload.WorkloadSpec(f"rr{seed}", batch, (0, hi), H * G, H, B, ("fixed", 96), (1, 1), s, w, budget_pages=k,
                               pages_per_chunk=4, chunks_per_grid=4)
    lens_full = [min(n + steps, hi) for n in start]
    full = to_device(workload.generate(sp, 600 + seed, seq_lens=lens_full))
    room = min(sp.max_pages, s + w + k + (steps // B + 2 if seed % 3 else 0))    # every third case: rows fill up
    lib = pk.Chess(config_of(sp, max_selected=room))
    lib.debug_force_splits(int(rng.choice([0, 0, 1, 2, 5])), 4)
    print(f"[reuse rand {seed}] page {B} H {H} G {G} start {start} steps {steps} s {s} w {w} k {k} room {room}", flush=True)
    lens = torch.tensor(start, dtype=torch.int32, device="cuda")
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(full.k_pool, full.block_table, lens, summ)
    ids = torch.full((batch, H, room), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((batch, H), -7, dtype=torch.int32, device="cuda")
    lib.select(full.q, summ, lens, gpu_plan(plan_of(sp)), ids, nsel, ws)
    bt = full.block_table
    mk = lambda: dict(k=full.k_pool.clone(), v=full.v_pool.clone(), ids=ids.clone(), nsel=nsel.clone(), lens=lens.clone(),
                      out=torch.full((batch, sp.n_q_heads, 128), float("nan"), device="cuda"))
    A, Bs = mk(), mk()
    gen = torch.Generator(device="cuda").manual_seed(seed)
    cap = sp.max_pages * B
    for step in range(steps):
        rk = torch.randn((batch, H, 128), device="cuda", generator=gen).to(torch.bfloat16)
        rv = torch.randn((batch, H, 128), device="cuda", generator=gen).to(torch.bfloat16)
        lib.append_kv(rk, rv, A["k"], A["v"], bt, A["lens"], A["ids"], A["nsel"])
        A["lens"] = torch.clamp(A["lens"] + 1, max=cap)
        lib.sparse_decode(full.q, A["k"], A["v"], bt, A["lens"], A["ids"], A["nsel"], A["out"], ws)
        lib.reuse_step(full.q, rk, rv, Bs["k"], Bs["v"], bt, Bs["lens"], Bs["ids"], Bs["nsel"], Bs["out"], ws)
        Bs["lens"] = torch.clamp(Bs["lens"] + 1, max=cap)
        torch.cuda.synchronize()
        assert torch.equal(A["nsel"], Bs["nsel"]), step
        live = torch.arange(room, device="cuda").view(1, 1, -1) < A["nsel"].unsqueeze(-1)
        assert torch.equal(torch.where(live, A["ids"], -1), torch.where(live, Bs["ids"], -1)), step
        assert torch.equal(A["out"], Bs["out"]), (step, (A["out"] - Bs["out"]).abs().max())
    lib.close()
