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
from gpu_common import config_of, gpu_plan, host_subset, to_device
from helpers import geom_of, plan_of

pytestmark = pytest.mark.gpu
ATOL = 1e-2


def run_case(name, sample, dense_seq=0, seed=None):
    sp = workload.spec(name)
    wl = workload.generate(sp, workload.default_seed(name) if seed is None else seed, device="cuda")
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
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    assert torch.equal(ids2, ids) and torch.equal(nsel2, nsel), (name, "fused step: page lists differ")
    out2_h = out2.cpu().numpy()
    pv, cv, gv = (t.cpu().numpy() for t in lib.summary_views(summ))
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
        print(f"[{name}] seq {b}: page lists exact, max|out - oracle| = {err:.2e} (two calls), {err2:.2e} (fused step)")
        assert err <= ATOL and err2 <= ATOL
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


def test_cfg4a_full():
    run_case("cfg4a", [0, 5], dense_seq=5)


def test_cfg4b_full():
    run_case("cfg4b", [3], dense_seq=None)


def test_cfg5_full_and_equal_norm_variant():
    run_case("cfg5", [0])
    run_case("cfg5adv", [0], dense_seq=None)
