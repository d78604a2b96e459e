"""Seeded random shapes: geometry (page size, GQA group, hierarchy fan-outs), batch, ragged lengths, sink / window,
plan and its parameters, probe, cluster size, general cut, in-launch tail refresh, schedule of the levels, cut rule,
per-sequence budgets -- each drawn per case, the GPU
(three calls and the fused step) against the oracle with the bars of test_gpu_parity.  The draws are fixed by the
seed, so a failure names a reproducible case."""
from __future__ import annotations

import os

import numpy as np
import pytest
import torch

import oracle
import paper_2602_20732_amd as pk
import workload
from gpu_common import host_views, assert_summaries_equal, classify_selection, config_of, gpu_plan, run_oracle, to_device
from helpers import plan_of

pytestmark = pytest.mark.gpu
ATOL_TIGHT = 2e-3


def draw(seed):
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.choice([16, 32]))
    H = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4, 7, 8, 16]))
    nc = int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
    ng = int(rng.choice([1, 2, 3, 4, 8, 16]))
    batch = int(rng.integers(1, 5))
    hi = int(rng.choice([300, 1500, 4000, 9000]))
    lens = [int(rng.integers(0, hi + 1)) for _ in range(batch)]
    lens[0] = hi                                                  # one sequence at the configured maximum
    s, w = int(rng.choice([0, 1, 3])), int(rng.choice([0, 1, 2, 5]))
    kind = int(rng.choice([oracle.PLAN_BUDGET, oracle.PLAN_RATIO, oracle.PLAN_FLAT]))
    kw = dict(plan=kind, sink_pages=s, window_pages=w)
    if kind == oracle.PLAN_RATIO:
        kw.update(rho_g_bp=int(rng.integers(1, 10001)), rho_c_bp=int(rng.integers(1, 10001)), rho_p_bp=int(rng.integers(1, 10001)))
    elif rng.random() < 0.5:
        kw.update(budget_pages=int(rng.integers(1, 40)), over_chunk=int(rng.integers(1, 12)), over_grid=int(rng.integers(1, 8)))
    else:
        kw.update(budget_bp=int(rng.integers(1, 3000)), over_chunk=int(rng.integers(1, 12)), over_grid=int(rng.integers(1, 8)))
    anchor = w > 0 and rng.random() < 0.3
    if anchor:
        kw.update(probe=oracle.PROBE_ANCHOR)
    sp = workload.WorkloadSpec(f"rand{seed}", batch, (0, hi), H * G, H, B, ("fixed", 96), (2, 2), s, w,
                               pages_per_chunk=nc, chunks_per_grid=ng)
    cluster, general, refresh = int(rng.choice([0, 1, 2, 5])), bool(rng.random() < 0.25), bool(rng.random() < 0.5) and not anchor
    # (drawn after everything else, so that the earlier draws of a seed stay what they were)
    schedule = int(rng.choice([0, 1, 2]))
    if rng.random() < 0.3:
        kw.update(cut_rule=oracle.CUT_THRESHOLD)
    if kind != oracle.PLAN_RATIO and rng.random() < 0.3:
        kw.update(budget_per_seq=tuple(int(rng.choice([0, 1, 3, 17])) for _ in range(batch)))
    return sp, lens, kw, cluster, general, refresh, schedule


@pytest.mark.parametrize("seed", range(int(os.environ.get("CHESS_RANDOM_SEEDS", "96"))))
def test_random_shape(seed):
    sp, lens, kw, cluster, general, refresh, schedule = draw(seed)
    print(f"[rand {seed}] page {sp.page_size} H {sp.n_kv_heads} G {sp.group} fan {sp.pages_per_chunk}x{sp.chunks_per_grid} "
          f"lens {lens} plan {kw} cluster {cluster} general {general} refresh {refresh} schedule {schedule}", flush=True)
    wl = workload.generate(sp, 500 + seed, seq_lens=lens)
    plan = plan_of(sp, **kw)
    max_sel = sp.max_pages
    lib = pk.Chess(config_of(sp, max_selected=max_sel))
    ref = run_oracle(wl, plan, max_sel, dense=False)
    d = to_device(wl)
    batch = len(lens)
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
    lib.debug_force_cluster(cluster)
    lib.debug_force_general_cut(general)
    lib.debug_force_schedule(schedule)
    ids = torch.full((batch, sp.n_kv_heads, max_sel), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((batch, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    out = torch.full((batch, sp.n_q_heads, 128), float("nan"), device="cuda")
    lib.select(d.q, summ, d.seq_lens, gpu_plan(plan), ids, nsel, ws)
    lib.sparse_decode(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, ids, nsel, out, ws)
    ids2, nsel2, out2 = torch.full_like(ids, -7), torch.full_like(nsel, -7), torch.full_like(out, float("nan"))
    if refresh:                                                   # stale tail vectors: the step has to recompute them
        pv, cv, gv = lib.summary_views(summ)
        for b, L in enumerate(lens):
            if L > 0:
                P = -(-L // sp.page_size); c = (P - 1) // sp.pages_per_chunk; g = c // sp.chunks_per_grid
                pv[b, :, P - 1] = 7.0; cv[b, :, c] = -3.0; gv[b, :, g] = 11.0
    lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids2, nsel2, out2, ws,
                    refresh_tail=refresh)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0

    class Got:
        pages, chunks, grids = host_views(lib, summ, batch)
    assert_summaries_equal(Got, ref, sp, lens)
    for name, i, n, o in (("three calls", ids, nsel, out), ("fused step", ids2, nsel2, out2)):
        gi, gn, go = i.cpu().numpy(), n.cpu().numpy(), o.cpu().numpy()
        hard, near = classify_selection(gi, gn, ref, wl, plan)
        assert not hard and not near, (name, hard[:2], near[:2])
        assert np.array_equal(gn, ref.nsel), name
        err = np.abs(go - ref.out).max()
        assert np.isfinite(go).all() and err <= ATOL_TIGHT, (name, err)
    lib.close()
