"""GPU parity at the benchmark configurations' full sizes, in the launch shapes bench.py times (automatic cluster
and split choices).  The GPU runs the whole batch; the oracle checks whole sampled sequences (all of their
summaries, page lists and sparse outputs, and the dense output of one of them)."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2602_20732_amd as pk
import workload
from gpu_common import host_views, config_of, gpu_plan, host_subset, to_device
from helpers import geom_of, plan_of

pytestmark = pytest.mark.gpu
ATOL = 1e-2


def run_case(name, sample, dense_seq=0, seed=None, layer=0):
    sp = workload.spec(name)
    wl = workload.generate(sp, workload.default_seed(name) if seed is None else seed, layer=layer, device="cuda")
    lib = pk.Chess(config_of(sp))
    plan = plan_of(sp)
    summ, ws = lib.new_summaries(), lib.new_workspace()
    ids = torch.full((sp.batch, sp.n_kv_heads, sp.max_selected), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((sp.batch, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    out = torch.full((sp.batch, sp.n_q_heads, 128), float("nan"), device="cuda")
    dense = torch.full_like(out, float("nan"))
    lib.summarize(wl.k_pool, wl.block_table, wl.seq_lens, summ)
    lib.summarize_tail(wl.k_pool, wl.block_table, wl.seq_lens, summ)          # the per-step refresh, as in bench.py
    lib.select(wl.q, summ, wl.seq_lens, gpu_plan(plan), ids, nsel, ws)
    lib.sparse_decode(wl.q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, ids, nsel, out, ws)
    lib.dense_decode(wl.q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, dense, ws)
    # the same step through the single-launch entry point, as bench.py times it
    ids2, nsel2, out2 = torch.full_like(ids, -7), torch.full_like(nsel, -7), torch.full_like(out, float("nan"))
    lib.decode_step(wl.q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summ, gpu_plan(plan), ids2, nsel2, out2, ws)
    # ... and exactly the call bench.py times: the tail page / chunk / grid vectors are stale (junk here) and the
    # launch refreshes them itself (refresh_tail), automatic cluster, before it scores them
    summ3 = summ.clone()
    pv3, cv3, gv3 = lib.summary_views(summ3)
    for b in range(sp.batch):
        P = -(-int(wl.seq_lens[b]) // sp.page_size)
        if P > 0:
            tp = P - 1; tc = tp // sp.pages_per_chunk; tg = tc // sp.chunks_per_grid
            pv3[b, :, tp] = 12345.0; cv3[b, :, tc] = -777.0; gv3[b, :, tg] = 31.0
    ids3, nsel3, out3 = torch.full_like(ids, -7), torch.full_like(nsel, -7), torch.full_like(out, float("nan"))
    lib.decode_step(wl.q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summ3, gpu_plan(plan), ids3, nsel3, out3, ws,
                    refresh_tail=True)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    assert torch.equal(ids2, ids) and torch.equal(nsel2, nsel), (name, "fused step: page lists differ")
    assert torch.equal(summ3, summ), (name, "fused step with refresh_tail: the refreshed summaries differ bit-wise")
    assert torch.equal(ids3, ids) and torch.equal(nsel3, nsel), (name, "fused step with refresh_tail: page lists differ")
    out2_h = out2.cpu().numpy()
    out3_h = out3.cpu().numpy()
    pv, cv, gv = host_views(lib, summ)
    ids_h, nsel_h, out_h, dense_h = ids.cpu().numpy(), nsel.cpu().numpy(), out.cpu().numpy(), dense.cpu().numpy()
    assert np.isfinite(out_h).all() and np.isfinite(dense_h).all()

    K, V, Q, bt, sl = host_subset(wl, sample)
    g = geom_of(sp)
    rp, rc, rg = oracle.summarize(K, bt, sl, g)
    rids, rn = oracle.select(Q, rp, rc, rg, sl, g, plan, sp.max_selected)
    rout = oracle.attend(Q, K, V, bt, sl, g, rids, rn)
    B, Nc, Ng = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    for i, b in enumerate(sample):
        P = -(-int(sl[i]) // B); nc = -(-P // Nc); ng = -(-nc // Ng)
        assert np.array_equal(pv[b, :, :P].view(np.uint32), rp[i, :, :P].view(np.uint32)), (name, b, "page vectors")
        assert np.array_equal(cv[b, :, :nc].view(np.uint32), rc[i, :, :nc].view(np.uint32)), (name, b, "chunk vectors")
        assert np.array_equal(gv[b, :, :ng].view(np.uint32), rg[i, :, :ng].view(np.uint32)), (name, b, "grid vectors")
        assert np.array_equal(nsel_h[b], rn[i]) and np.array_equal(ids_h[b], rids[i]), (name, b, "page lists")
        err = np.abs(out_h[b] - rout[i]).max()
        err2 = np.abs(out2_h[b] - rout[i]).max()
        err3 = np.abs(out3_h[b] - rout[i]).max()
        print(f"[{name}] seq {b}: page lists exact, max|out - oracle| = {err:.2e} (two calls), {err2:.2e} (fused step), "
              f"{err3:.2e} (fused step refreshing the tail, as timed)")
        assert err <= ATOL and err2 <= ATOL and err3 <= ATOL
    # every sequence, not only the sampled ones: list shape invariants
    for b in range(sp.batch):
        P = -(-int(wl.seq_lens[b]) // B)
        for h in range(sp.n_kv_heads):
            row = ids_h[b, h, :nsel_h[b, h]]
            assert nsel_h[b, h] == min(P, sp.sink_pages + sp.window_pages + sp.budget_for(P))
            assert (np.diff(row) > 0).all() and row[0] == 0 and row[-1] == P - 1 and (ids_h[b, h, nsel_h[b, h]:] == -1).all()
    if dense_seq is not None:
        Kd, Vd, Qd, btd, sld = host_subset(wl, [dense_seq])
        rd = oracle.attend(Qd, Kd, Vd, btd, sld, g)
        derr = np.abs(dense_h[dense_seq] - rd[0]).max()
        print(f"[{name}] seq {dense_seq}: dense max|out - oracle| = {derr:.2e}")
        assert derr <= ATOL
    lib.close()


def test_cfg2_full():
    run_case("cfg2", [0])


def test_cfg3_one_layer_full_batch():
    run_case("cfg3", [0, 13, 31], dense_seq=13)


def test_cfg3_last_layer_of_the_stack():
    """cfg3 is a stack of 32 layers with fresh seeded KV each; the last one, as bench.py generates it."""
    run_case("cfg3", [7], dense_seq=None, layer=31)


def test_cfg4a_full():
    run_case("cfg4a", [0, 5], dense_seq=5)


def test_cfg4b_full():
    run_case("cfg4b", [3], dense_seq=None)


def test_cfg5_full_and_equal_norm_variant():
    run_case("cfg5", [0])
    run_case("cfg5adv", [0], dense_seq=None)


@pytest.mark.parametrize("name,sample", [("cfg4a", 5), ("cfg3", 13), ("cfg5", 0)])
def test_reuse_step_at_benchmark_shapes(name, sample):
    """The step between reselections as bench.py times it: the lists selected one token earlier, then
    chess_reuse_step with the last token's rows.  The pools must end up unchanged (the token's own rows are written
    back), the output must be bit-identical to chess_append_kv + chess_sparse_decode, and on a sampled sequence equal
    the oracle's attention over the list on the full length."""
    sp = workload.spec(name)
    wl = workload.generate(sp, workload.default_seed(name), device="cuda")
    lib = pk.Chess(config_of(sp))
    plan = plan_of(sp)
    B, H = sp.page_size, sp.n_kv_heads
    before = (wl.seq_lens - 1).clamp_(min=0)
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(wl.k_pool, wl.block_table, before, summ)
    ids = torch.full((sp.batch, H, sp.max_selected), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((sp.batch, H), -7, dtype=torch.int32, device="cuda")
    lib.select(wl.q, summ, before, gpu_plan(plan), ids, nsel, ws)
    # the last token's rows, taken out of the pools
    bt = wl.block_table
    pos = before.long()
    phys = bt[torch.arange(sp.batch, device="cuda"), pos // B].long()
    rk = torch.stack([wl.k_pool[phys[b], :, int(pos[b]) % B, :] for b in range(sp.batch)]).contiguous()
    rv = torch.stack([wl.v_pool[phys[b], :, :, int(pos[b]) % B] for b in range(sp.batch)]).contiguous()
    k2, v2 = wl.k_pool.clone(), wl.v_pool.clone()
    for b in range(sp.batch):                                   # the slot is junk until the call stores the token
        k2[phys[b], :, int(pos[b]) % B, :] = float("nan")
        v2[phys[b], :, :, int(pos[b]) % B] = float("nan")
    ids1, nsel1, ids2, nsel2 = ids.clone(), nsel.clone(), ids.clone(), nsel.clone()
    out1 = torch.full((sp.batch, sp.n_q_heads, 128), float("nan"), device="cuda")
    out2 = torch.full_like(out1, float("nan"))
    lib.reuse_step(wl.q, rk, rv, k2, v2, bt, before, ids1, nsel1, out1, ws)
    k3, v3 = k2.clone(), v2.clone()                              # (k2 has the token by now; junk it again for the two calls)
    for b in range(sp.batch):
        k3[phys[b], :, int(pos[b]) % B, :] = float("nan")
        v3[phys[b], :, :, int(pos[b]) % B] = float("nan")
    lib.append_kv(rk, rv, k3, v3, bt, before, ids2, nsel2)
    lib.sparse_decode(wl.q, k3, v3, bt, wl.seq_lens, ids2, nsel2, out2, ws)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    assert torch.equal(out1, out2) and torch.equal(nsel1, nsel2)
    assert torch.equal(k2.view(torch.int16), wl.k_pool.view(torch.int16)) and torch.equal(v2.view(torch.int16), wl.v_pool.view(torch.int16))
    K, V, Q, bts, sls = host_subset(wl, [sample])
    ref = oracle.attend(Q, K, V, bts, sls, geom_of(sp), ids1[sample:sample + 1].cpu().numpy(), nsel1[sample:sample + 1].cpu().numpy())
    err = np.abs(out1[sample].cpu().numpy() - ref[0]).max()
    print(f"[{name}] reuse step, seq {sample}: max|out - oracle| = {err:.2e}")
    assert err <= ATOL
    lib.close()


def test_cfg4a_threshold_rule_and_ragged_budgets():
    """The benchmark shape with the switches a serving engine would use: a page budget per sequence (device array, some
    entries falling back to the plan's 1 %) and the S >= tau cut rule; select, the fused step with its tail refresh, and
    the attention over the list, whole sampled sequences against the oracle in the same modes."""
    sp = workload.spec("cfg4a")
    wl = workload.generate(sp, workload.default_seed("cfg4a") + 7, device="cuda")
    per = (41, 0, 164, 82, 1, 120, 0, 60)
    plan = plan_of(sp, budget_per_seq=per, cut_rule=oracle.CUT_THRESHOLD)
    max_sel = sp.sink_pages + sp.window_pages + 164
    lib = pk.Chess(config_of(sp, max_selected=max_sel))
    summ, ws = lib.new_summaries(), lib.new_workspace()
    ids = torch.full((sp.batch, sp.n_kv_heads, max_sel), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((sp.batch, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    out = torch.full((sp.batch, sp.n_q_heads, 128), float("nan"), device="cuda")
    lib.summarize(wl.k_pool, wl.block_table, wl.seq_lens, summ)
    gp = gpu_plan(plan)
    lib.select(wl.q, summ, wl.seq_lens, gp, ids, nsel, ws)
    ids2, nsel2 = torch.full_like(ids, -7), torch.full_like(nsel, -7)
    lib.decode_step(wl.q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summ, gp, ids2, nsel2, out, ws, refresh_tail=True)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    assert torch.equal(ids, ids2) and torch.equal(nsel, nsel2)
    want = [sp.sink_pages + sp.window_pages + (k if k > 0 else sp.budget_for(sp.max_pages)) for k in per]
    assert nsel.cpu().numpy().tolist() == [[n] * sp.n_kv_heads for n in want]
    sample = [2, 4]
    K, V, Q, bt, sl = host_subset(wl, sample)
    g = geom_of(sp)
    rp, rc, rg = oracle.summarize(K, bt, sl, g)
    sub_plan = plan_of(sp, budget_per_seq=tuple(per[b] for b in sample), cut_rule=oracle.CUT_THRESHOLD)
    rids, rn = oracle.select(Q, rp, rc, rg, sl, g, sub_plan, max_sel)
    rout = oracle.attend(Q, K, V, bt, sl, g, rids, rn)
    for i, b in enumerate(sample):
        assert np.array_equal(ids[b].cpu().numpy(), rids[i]) and np.array_equal(nsel[b].cpu().numpy(), rn[i]), (b, "page lists")
        err = np.abs(out[b].cpu().numpy() - rout[i]).max()
        print(f"[cfg4a ragged budgets, threshold rule] seq {b}: k = {per[b]}, page lists exact, max|out - oracle| = {err:.2e}")
        assert err <= ATOL
    lib.close()
