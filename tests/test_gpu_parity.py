"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on the same
seeded inputs.  Bars: summaries and page lists bit-exact (near-ties under 1e-5 reported separately and not
expected, both sides score in fp64); attention outputs within 1e-2 max-abs (bf16 inputs, fp32 accumulate).
Small cases span several tiles and ragged tails; full-size cases run the benchmark's launch shapes."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2602_20732_amd as pk
import workload
from gpu_common import (assert_summaries_equal, classify_selection, config_of, gpu_plan, host_views, run_gpu, run_oracle,
                        to_device)
from helpers import geom_of, host_arrays, plan_of

pytestmark = pytest.mark.gpu

ATOL = 1e-2          # the stated bar for attention outputs
ATOL_TIGHT = 2e-3    # what the arithmetic should achieve (bf16 inputs exact, fp32 accumulate, P split in two bf16)


def check_all(sp, wl, plan, max_sel=None, dense=True, label=""):
    max_sel = sp.max_selected if max_sel is None else max_sel
    lib = pk.Chess(config_of(sp, max_selected=max_sel))
    gpu = run_gpu(lib, wl, plan, dense=dense)
    ref = run_oracle(wl, plan, max_sel, dense=dense)
    sl = ref.host[4]
    assert_summaries_equal(gpu, ref, sp, sl)
    hard, near = classify_selection(gpu.ids, gpu.nsel, ref, wl, plan)
    print(f"[{label}] selection rows: hard mismatches {len(hard)}, near-ties {len(near)}")
    assert not hard, hard[:3]
    assert not near, near[:3]
    assert np.array_equal(gpu.nsel, ref.nsel)
    err = np.abs(gpu.out - ref.out).max()
    print(f"[{label}] sparse max|out - oracle| = {err:.3e}")
    assert np.isfinite(gpu.out).all() and err <= ATOL and err <= ATOL_TIGHT
    # the single-launch step: the same list, attention over it against the oracle
    assert np.array_equal(gpu.step_ids, gpu.ids) and np.array_equal(gpu.step_nsel, gpu.nsel), "fused step: page lists differ"
    serr = np.abs(gpu.step_out - ref.out).max()
    print(f"[{label}] fused step max|out - oracle| = {serr:.3e}")
    assert np.isfinite(gpu.step_out).all() and serr <= ATOL and serr <= ATOL_TIGHT
    if dense:
        derr = np.abs(gpu.dense - ref.dense).max()
        print(f"[{label}] dense  max|out - oracle| = {derr:.3e}")
        assert np.isfinite(gpu.dense).all() and derr <= ATOL and derr <= ATOL_TIGHT
    lib.close()
    return gpu, ref


def test_cfg1_full_size():
    sp = workload.spec("cfg1")
    wl = workload.generate(sp, workload.default_seed("cfg1"))
    check_all(sp, wl, plan_of(sp), label="cfg1")


RAGGED = workload.WorkloadSpec("ragged", 5, (0, 3000), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_bp=300,
                               pages_per_chunk=4, chunks_per_grid=4)
RAGGED_LENS = [3000, 1237, 641, 16, 0]


@pytest.mark.parametrize("plan_kw", [
    dict(plan=oracle.PLAN_BUDGET),
    dict(plan=oracle.PLAN_BUDGET, budget_pages=9, over_chunk=2, over_grid=1),
    dict(plan=oracle.PLAN_RATIO, rho_g_bp=5000, rho_c_bp=2000, rho_p_bp=1000),
    dict(plan=oracle.PLAN_RATIO, rho_g_bp=8000, rho_c_bp=7000, rho_p_bp=7000),
    dict(plan=oracle.PLAN_RATIO, rho_g_bp=9000, rho_c_bp=9000, rho_p_bp=9000),
    dict(plan=oracle.PLAN_FLAT, budget_pages=16),
    dict(plan=oracle.PLAN_RATIO),                                  # ratios 1,1,1: Full-KV through the sparse path
    dict(plan=oracle.PLAN_BUDGET, probe=oracle.PROBE_ANCHOR),      # Eq. 3: units scored against the window's key anchor
    dict(plan=oracle.PLAN_RATIO, rho_g_bp=5000, rho_c_bp=2000, rho_p_bp=1000, probe=oracle.PROBE_ANCHOR, window_pages=3),
])
def test_ragged_batch_all_plans(plan_kw):
    """GQA 4, ragged lengths incl. a partial tail page, partial chunk / grid, a one-page and an empty sequence."""
    sp = RAGGED
    wl = workload.generate(sp, 77, seq_lens=RAGGED_LENS)
    check_all(sp, wl, plan_of(sp, **plan_kw), max_sel=sp.max_pages, label=f"ragged {plan_kw}")


@pytest.mark.parametrize("nc,ng", [(2, 2), (8, 8), (4, 16), (1, 1), (16, 16)])
def test_hierarchy_shapes(nc, ng):
    sp = workload.WorkloadSpec("hier", 2, (500, 5000), 8, 2, 16, ("fixed", 128), (3, 3), 1, 4, budget_bp=200,
                               pages_per_chunk=nc, chunks_per_grid=ng)
    wl = workload.generate(sp, 31 + nc, seq_lens=[5000, 2049])
    check_all(sp, wl, plan_of(sp), dense=False, label=f"hier {nc}x{ng}")


@pytest.mark.parametrize("cluster", [1, 2, 3, 8, 32])
def test_cluster_sizes_give_the_same_page_lists(cluster):
    """The number of workgroups cooperating on one (sequence, head) must not change anything; twice in a row
    on one workspace, alternating with the fused step, so the key words and counters are shown to be left
    clean by both kernels."""
    sp = workload.spec("cfg2", scale=1 / 2)
    wl = workload.generate(sp, workload.default_seed("cfg2"))
    plan = plan_of(sp)
    lib = pk.Chess(config_of(sp))
    ref = run_oracle(wl, plan, sp.max_selected, dense=False)
    d = to_device(wl)
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
    lib.debug_force_cluster(cluster)
    for _ in range(2):
        ids = torch.full((1, sp.n_kv_heads, sp.max_selected), -7, dtype=torch.int32, device="cuda")
        nsel = torch.full((1, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
        lib.select(d.q, summ, d.seq_lens, gpu_plan(plan), ids, nsel, ws)
        torch.cuda.synchronize()
        assert lib.workspace_error(ws) == 0
        assert np.array_equal(ids.cpu().numpy(), ref.ids) and np.array_equal(nsel.cpu().numpy(), ref.nsel)
        ids2, nsel2 = torch.full_like(ids, -7), torch.full_like(nsel, -7)
        out2 = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
        lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids2, nsel2, out2, ws)
        torch.cuda.synchronize()
        assert lib.workspace_error(ws) == 0
        assert np.array_equal(ids2.cpu().numpy(), ref.ids) and np.array_equal(nsel2.cpu().numpy(), ref.nsel)
        err = np.abs(out2.cpu().numpy() - ref.out).max()
        assert err <= ATOL_TIGHT, err


@pytest.mark.parametrize("cluster", [1, 3])
def test_fused_step_refreshes_the_tail_summaries(cluster):
    """chess_decode_step with refresh_tail: the vectors of the tail page, its chunk and its grid are stale
    (overwritten with junk here); the step must recompute them bit-exactly, score the fresh ones and leave them
    in the summaries buffer.  Ragged lengths incl. a tail page that starts a new chunk and a new grid; window 0
    in the second plan, so that the tail page itself competes."""
    sp = RAGGED
    lens = [3000, 1237, 641, 16 * 16 + 1, 16]        # 16*16+1: the tail page opens a chunk and a grid (N_c = N_g = 4)
    wl = workload.generate(sp, 78, seq_lens=lens)
    for plan in (plan_of(sp), plan_of(sp, window_pages=0, sink_pages=0)):
        lib = pk.Chess(config_of(sp, max_selected=sp.max_pages))
        ref = run_oracle(wl, plan, sp.max_pages, dense=False)
        d = to_device(wl)
        summ, ws = lib.new_summaries(), lib.new_workspace()
        lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
        pv, cv, gv = lib.summary_views(summ)
        B, Nc, Ng = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
        for b, L in enumerate(lens):
            tp = -(-L // B) - 1
            pv[b, :, tp] = 1e9; cv[b, :, tp // Nc] = -1e9; gv[b, :, tp // Nc // Ng] = float("nan")
        lib.debug_force_cluster(cluster)
        for _ in range(2):                               # the second call starts from refreshed summaries: same result
            ids = torch.full((len(lens), sp.n_kv_heads, sp.max_pages), -7, dtype=torch.int32, device="cuda")
            nsel = torch.full((len(lens), sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
            out = torch.full((len(lens), sp.n_q_heads, 128), float("nan"), device="cuda")
            lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids, nsel, out, ws,
                            refresh_tail=True)
            torch.cuda.synchronize()
            assert lib.workspace_error(ws) == 0
            got = GpuRunLike(*host_views(lib, summ, len(lens)))
            assert_summaries_equal(got, ref, sp, lens)
            assert np.array_equal(ids.cpu().numpy(), ref.ids) and np.array_equal(nsel.cpu().numpy(), ref.nsel)
            assert np.abs(out.cpu().numpy() - ref.out).max() <= ATOL_TIGHT
        lib.close()


class GpuRunLike:
    def __init__(self, pages, chunks, grids):
        self.pages, self.chunks, self.grids = pages, chunks, grids


def test_anchor_probe_at_cfg1_and_refusals():
    """Eq. 3 probe on the 4K configuration, several members per (sequence, head); it cannot be combined with the
    in-launch tail refresh, needs a window, and lets chess_select run without a query."""
    sp = workload.spec("cfg1")
    wl = workload.generate(sp, workload.default_seed("cfg1"))
    plan = plan_of(sp, probe=oracle.PROBE_ANCHOR)
    check_all(sp, wl, plan, dense=False, label="cfg1 anchor")
    lib = pk.Chess(config_of(sp))
    d = to_device(wl)
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
    ids = torch.zeros((1, sp.n_kv_heads, sp.max_selected), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((1, sp.n_kv_heads), dtype=torch.int32, device="cuda")
    out = torch.zeros((1, sp.n_q_heads, 128), device="cuda")
    lib.select(None, summ, d.seq_lens, gpu_plan(plan), ids, nsel, ws)             # no query needed
    torch.cuda.synchronize()
    ref = run_oracle(wl, plan, sp.max_selected, dense=False)
    assert np.array_equal(ids.cpu().numpy(), ref.ids)
    with pytest.raises(pk.ChessError):
        lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids, nsel, out, ws,
                        refresh_tail=True)
    with pytest.raises(pk.ChessError):
        lib.select(d.q, summ, d.seq_lens, gpu_plan(plan_of(sp, probe=oracle.PROBE_ANCHOR, window_pages=0)), ids, nsel, ws)
    lib.close()


def test_page32_gqa7_and_equal_norm_topics():
    """The stress shape scaled down (page 32, 28 / 4 heads), plus its equal-norm variant (near-tied scores)."""
    for name in ("cfg5", "cfg5adv"):
        sp = workload.spec(name, scale=1 / 16)
        wl = workload.generate(sp, workload.default_seed(name))
        check_all(sp, wl, plan_of(sp), label=name + "/16")


def test_exact_ties_go_to_lowest_index():
    """All key rows identical: every score ties at every level; uniform softmax -> mean of listed V rows."""
    sp = workload.WorkloadSpec("ties", 1, (2048, 2048), 4, 1, 16, ("fixed", 128), (1, 1), 1, 2, budget_pages=5,
                               pages_per_chunk=2, chunks_per_grid=2)
    wl = workload.generate(sp, 3)
    row = wl.k_pool[wl.block_table[0, 0].item(), 0, 0].clone()
    wl.k_pool[:] = row                                   # every token of every page gets the same key row
    plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=1, window_pages=2, rho_g_bp=5000, rho_c_bp=5000, rho_p_bp=5000)
    gpu, ref = check_all(sp, wl, plan, max_sel=sp.max_pages, dense=False, label="ties")
    # 128 pages -> 64 chunks -> 32 grids; keeps grids 0..15, chunks 0..15, candidate pages 1..31 -> 16 lowest
    assert gpu.ids[0, 0, :gpu.nsel[0, 0]].tolist() == list(range(0, 17)) + [126, 127]


def test_tie_groups_at_the_cut():
    """Three distinct key rows dealt by page number: every level has a few large groups of exactly tied scores,
    so a cut falls inside a group (lowest indices win), with fewer and with more tied keys than the
    in-register ranking of the select kernel holds."""
    sp = workload.WorkloadSpec("groups", 2, (8192, 8192), 4, 1, 16, ("fixed", 128), (1, 1), 1, 2, budget_pages=5,
                               pages_per_chunk=2, chunks_per_grid=2)
    wl = workload.generate(sp, 9, seq_lens=[8192, 5000])
    rows = [wl.k_pool[wl.block_table[0, j].item(), 0, 0].clone() for j in (0, 1, 2)]
    for b in range(2):
        for j in range(-(-int(wl.seq_lens[b]) // 16)):
            wl.k_pool[wl.block_table[b, j].item(), 0, :] = rows[j % 3]
    for bp in (5000, 3000, 9000):
        plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=1, window_pages=2, rho_g_bp=bp, rho_c_bp=5000, rho_p_bp=bp)
        check_all(sp, wl, plan, max_sel=sp.max_pages, dense=False, label=f"tie groups {bp}")


@pytest.mark.parametrize("cluster", [1, 4])
def test_general_cut_gives_the_same_page_lists(cluster):
    """The cut that tied or very large levels fall back to (radix select in LDS), forced on every level."""
    for sp, wl in ((workload.spec("cfg2", scale=1 / 2), None), (RAGGED, RAGGED_LENS)):
        wl = workload.generate(sp, 123, seq_lens=wl)
        plan = plan_of(sp)
        lib = pk.Chess(config_of(sp, max_selected=sp.max_pages))
        lib.debug_force_general_cut(True)
        gpu = run_gpu(lib, wl, plan, dense=False, cluster=cluster)
        ref = run_oracle(wl, plan, sp.max_pages, dense=False)
        assert np.array_equal(gpu.ids, ref.ids) and np.array_equal(gpu.nsel, ref.nsel)
        lib.close()


def test_short_and_boundary_lengths():
    sp = workload.WorkloadSpec("short", 8, (0, 161), 4, 2, 16, ("fixed", 32), (1, 1), 2, 3, budget_pages=2,
                               pages_per_chunk=2, chunks_per_grid=2)
    wl = workload.generate(sp, 5, seq_lens=[0, 1, 15, 16, 17, 80, 96, 161])
    check_all(sp, wl, plan_of(sp), label="short")


def test_nan_in_unused_slots_is_never_read():
    """The generator fills unused tail slots and spare pages with NaN; outputs must stay finite (checked in
    check_all) and must not depend on what the unused slots hold."""
    sp = workload.WorkloadSpec("nan", 2, (100, 1000), 8, 2, 32, ("fixed", 64), (2, 2), 1, 1, budget_bp=500,
                               pages_per_chunk=2, chunks_per_grid=4)
    wl = workload.generate(sp, 9, seq_lens=[1000 - 7, 333])
    gpu, _ = check_all(sp, wl, plan_of(sp), label="nan")
    wl.k_pool[wl.k_pool.isnan()] = 123.0
    wl.v_pool[wl.v_pool.isnan()] = -55.0
    lib = pk.Chess(config_of(sp))
    gpu2 = run_gpu(lib, wl, plan_of(sp))
    assert np.array_equal(gpu.out, gpu2.out) and np.array_equal(gpu.dense, gpu2.dense) and np.array_equal(gpu.ids, gpu2.ids)


def test_incremental_and_tail_summaries_match_full_pass():
    sp = RAGGED
    lens0 = [2990, 1237, 630, 16, 0]
    lens1 = [3000, 1239, 641, 17, 3]                      # grows within the page, across pages, from nothing
    wl = to_device(workload.generate(sp, 77, seq_lens=lens1))
    lib = pk.Chess(config_of(sp, max_selected=sp.max_pages))
    full = lib.new_summaries()
    lib.summarize(wl.k_pool, wl.block_table, wl.seq_lens, full)
    inc = lib.new_summaries()
    l0 = torch.tensor(lens0, dtype=torch.int32, device="cuda")
    lib.summarize(wl.k_pool, wl.block_table, l0, inc)                       # state before the new tokens
    from_page = torch.tensor([max(0, n - 1) // sp.page_size for n in lens0], dtype=torch.int32, device="cuda")
    lib.summarize(wl.k_pool, wl.block_table, wl.seq_lens, inc, from_page=from_page)
    torch.cuda.synchronize()
    B, Nc, Ng = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    for a, b, per in zip(lib.summary_views(full), lib.summary_views(inc), (1, Nc, Nc * Ng)):
        for i, L in enumerate(lens1):
            n = -(-(-(-L // B)) // per)
            assert torch.equal(a[i, :, :n], b[i, :, :n])
    # tail refresh: one more token in the tail page of every sequence
    tail = lib.new_summaries()
    lm = torch.tensor([max(n - 1, 0) for n in lens1], dtype=torch.int32, device="cuda")   # incl. 16 -> 17: a new page
    lib.summarize(wl.k_pool, wl.block_table, lm, tail)
    lib.summarize_tail(wl.k_pool, wl.block_table, wl.seq_lens, tail)
    torch.cuda.synchronize()
    for a, b, per in zip(lib.summary_views(full), lib.summary_views(tail), (1, Nc, Nc * Ng)):
        for i, L in enumerate(lens1):
            n = -(-(-(-L // B)) // per)
            assert torch.equal(a[i, :, :n], b[i, :, :n])


@pytest.mark.parametrize("recent", [1, 2, 5, 17, 40, 1000])
def test_recent_pages_catch_up_matches_full_pass(recent):
    """chess_summarize_recent on summaries that were current `gained` pages ago (the pages since hold junk, and so do
    their chunks and grids): the result equals a full pass.  recent may exceed what the sequence gained or has."""
    sp = RAGGED
    lens1 = [3000, 1239, 641, 17, 3]
    gained = [min(recent, -(-n // sp.page_size)) for n in lens1]
    lens0 = [max(0, (-(-n // sp.page_size) - g) * sp.page_size) for n, g in zip(lens1, gained)]   # whole pages earlier
    wl = to_device(workload.generate(sp, 77, seq_lens=lens1))
    lib = pk.Chess(config_of(sp, max_selected=sp.max_pages))
    full, inc = lib.new_summaries(), lib.new_summaries()
    lib.summarize(wl.k_pool, wl.block_table, wl.seq_lens, full)
    for t in lib.summary_views(inc):
        t.fill_(123.0)
    lib.summarize(wl.k_pool, wl.block_table, torch.tensor(lens0, dtype=torch.int32, device="cuda"), inc)
    lib.summarize_recent(wl.k_pool, wl.block_table, wl.seq_lens, recent, inc)
    torch.cuda.synchronize()
    B, Nc, Ng = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    for a, b, per in zip(lib.summary_views(full), lib.summary_views(inc), (1, Nc, Nc * Ng)):
        for i, L in enumerate(lens1):
            n = -(-(-(-L // B)) // per)
            assert torch.equal(a[i, :, :n], b[i, :, :n]), (recent, i, per)
    with pytest.raises(pk.ChessError):
        lib.summarize_recent(wl.k_pool, wl.block_table, wl.seq_lens, 0, inc)
    lib.close()


def test_split_count_invariance_and_determinism():
    sp = workload.spec("cfg2", scale=1 / 4)
    wl = to_device(workload.generate(sp, workload.default_seed("cfg2")))
    lib = pk.Chess(config_of(sp))
    ws = lib.new_workspace()
    outs = []
    for n_splits, waves in ((1, 1), (1, 4), (2, 4), (7, 1), (16, 4), (64, 1), (0, 4)):
        lib.debug_force_splits(n_splits, waves)
        out = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
        lib.dense_decode(wl.q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, out, ws)
        out2 = torch.full_like(out, float("nan"))
        lib.dense_decode(wl.q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, out2, ws)
        torch.cuda.synchronize()
        assert torch.equal(out, out2), "run-to-run bit identity at a fixed split shape"
        outs.append(out.cpu().numpy())
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() < 1e-5
    K, V, Q, bt, sl = host_arrays(wl)
    ref = oracle.attend(Q, K, V, bt, sl, geom_of(sp))
    assert np.abs(outs[0] - ref).max() <= ATOL_TIGHT


def test_step_in_a_hip_graph_replays_like_eager():
    """The whole step captured in a HIP graph (as bench.py runs it): every replay, with eager launches and
    synchronisations between the replays and a different query each time, gives the eager result bit for bit;
    page_ids / n_selected may be NULL."""
    sp = workload.spec("cfg2", scale=1 / 4)
    wl = to_device(workload.generate(sp, workload.default_seed("cfg2")))
    lib = pk.Chess(config_of(sp))
    plan = gpu_plan(plan_of(sp))
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(wl.k_pool, wl.block_table, wl.seq_lens, summ)
    qs = [wl.q] + [workload.extra_queries(wl, v) for v in range(1, 4)]
    eager = []
    for q in qs:
        out = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
        lib.decode_step(q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summ, plan, None, None, out, ws, refresh_tail=True)
        torch.cuda.synchronize()
        eager.append(out.clone())
    q_in = torch.empty_like(wl.q)
    out_g = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        q_in.copy_(qs[0])
        lib.decode_step(q_in, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summ, plan, None, None, out_g, ws, refresh_tail=True)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            lib.decode_step(q_in, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, summ, plan, None, None, out_g, ws,
                            refresh_tail=True)
        for rep in range(6):
            i = rep % len(qs)
            q_in.copy_(qs[i])
            out_g.fill_(float("nan"))
            graph.replay()
            stream.synchronize()
            assert torch.equal(out_g, eager[i]), f"replay {rep}"
            scratch = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")     # eager work between replays
            lib.dense_decode(qs[i], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, scratch, ws)
            stream.synchronize()
    assert lib.workspace_error(ws) == 0
    lib.close()


def test_a_wait_that_is_given_up_raises_the_error_flag_and_every_kernel_still_ends():
    """The members of a cluster wait for each other's keys with a bounded number of polls.  With the bound forced
    down to one poll the waits fail: the launches must still end by themselves, the workspace's error flag must be
    up, and after re-initialising the workspace (and restoring the bound) the results are right again."""
    sp = workload.spec("cfg2", scale=1 / 2)
    wl = workload.generate(sp, workload.default_seed("cfg2"))
    plan = plan_of(sp)
    lib = pk.Chess(config_of(sp))
    ref = run_oracle(wl, plan, sp.max_selected, dense=False)
    d = to_device(wl)
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
    ids = torch.full((1, sp.n_kv_heads, sp.max_selected), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((1, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    out = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
    lib.debug_force_cluster(4)
    lib.debug_set_poll_limit(-1)                          # every wait for other members' keys is given up at once
    lib.select(d.q, summ, d.seq_lens, gpu_plan(plan), ids, nsel, ws)
    lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids, nsel, out, ws)
    torch.cuda.synchronize()                              # returns: nobody is left waiting
    assert lib.workspace_error(ws) == 1
    lib.debug_set_poll_limit(0)
    ws = lib.new_workspace()
    lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids, nsel, out, ws)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    assert np.array_equal(ids.cpu().numpy(), ref.ids) and np.array_equal(nsel.cpu().numpy(), ref.nsel)
    assert np.abs(out.cpu().numpy() - ref.out).max() <= ATOL_TIGHT
    lib.close()


def test_zero_copy_pools_untouched_and_placement_invariance():
    sp = RAGGED
    wl = workload.generate(sp, 78, seq_lens=RAGGED_LENS)
    d = to_device(wl)
    k0, v0 = d.k_pool.clone(), d.v_pool.clone()
    lib = pk.Chess(config_of(sp))
    plan = plan_of(sp)
    a = run_gpu(lib, d, plan)
    assert torch.equal(d.k_pool.view(torch.int16), k0.view(torch.int16)) and torch.equal(d.v_pool.view(torch.int16), v0.view(torch.int16))
    perm = torch.randperm(d.k_pool.shape[0], generator=torch.Generator().manual_seed(1)).cuda()
    k2, v2 = torch.empty_like(d.k_pool), torch.empty_like(d.v_pool)
    k2[perm], v2[perm] = d.k_pool, d.v_pool
    bt2 = torch.where(d.block_table >= 0, perm[d.block_table.clamp(min=0).long()].int(), d.block_table)
    moved = workload.Workload(sp, 78, 0, k2, v2, bt2, d.seq_lens, d.q)
    b = run_gpu(lib, moved, plan)
    assert np.array_equal(a.ids, b.ids) and np.array_equal(a.nsel, b.nsel)
    assert np.array_equal(a.pages, b.pages) and np.abs(a.out - b.out).max() <= 1e-6


def test_error_codes():
    sp = RAGGED
    lib = pk.Chess(config_of(sp))
    d = to_device(workload.generate(sp, 77, seq_lens=RAGGED_LENS))
    summ, ws = lib.new_summaries(), lib.new_workspace()
    ids = torch.zeros((5, 2, sp.max_selected), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((5, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(pk.ChessError):       # budget + safety pages do not fit max_selected_pages
        lib.select(d.q, summ, d.seq_lens, pk.SelectPlan(budget_pages=sp.max_selected), ids, nsel, ws)
    with pytest.raises(pk.ChessError):       # unknown plan
        lib.select(d.q, summ, d.seq_lens, pk.SelectPlan(plan=9), ids, nsel, ws)
    with pytest.raises(pk.ChessError):       # batch beyond max_batch
        big = torch.zeros(6, dtype=torch.int32, device="cuda")
        lib.summarize(d.k_pool, d.block_table, big, summ)
    out = torch.zeros((5, sp.n_q_heads, 128), device="cuda")
    with pytest.raises(pk.ChessError):       # the fused step checks its plan the same way
        lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, pk.SelectPlan(budget_pages=sp.max_selected),
                        ids, nsel, out, ws)
    with pytest.raises(pk.ChessError):       # ... and refuses a missing buffer
        lib.decode_step(d.q, d.k_pool, None, d.block_table, d.seq_lens, summ, pk.SelectPlan(), ids, nsel, out, ws)
    with pytest.raises(pk.ChessError):
        pk.Chess(pk.Config(8, 3, 16, 1, 64, 8))          # 8 q heads over 3 kv heads
    with pytest.raises(pk.ChessError):
        pk.Chess(pk.Config(8, 2, 24, 1, 64, 8))          # page size


@pytest.mark.parametrize("plan_kw", [dict(plan=oracle.PLAN_BUDGET), dict(plan=oracle.PLAN_FLAT),
                                     dict(plan=oracle.PLAN_BUDGET, probe=oracle.PROBE_ANCHOR)])
def test_per_sequence_budgets(plan_kw):
    """budget_per_seq (device int32 [batch]): ragged budgets in one batch, an entry <= 0 falls back to the plan's
    own budget; select, the fused step and the model-wide scope against the oracle with the same budgets."""
    sp = RAGGED
    wl = workload.generate(sp, 79, seq_lens=RAGGED_LENS)
    per = (12, 0, 3, 5, 2)
    check_all(sp, wl, plan_of(sp, budget_per_seq=per, **plan_kw), max_sel=sp.max_pages, label=f"per-seq budgets {plan_kw}")
    # a budget above what a page_ids row can hold is clamped to the room the row has
    small = 1 + 2 + 6
    plan = plan_of(sp, budget_per_seq=(500, 0, 3, 5, 2), **plan_kw)
    lib = pk.Chess(config_of(sp, max_selected=small))
    gpu = run_gpu(lib, wl, plan, dense=False)
    ref = run_oracle(wl, plan_of(sp, budget_per_seq=(6, 0, 3, 5, 2), **plan_kw), small, dense=False)
    assert np.array_equal(gpu.ids, ref.ids) and np.array_equal(gpu.nsel, ref.nsel)
    assert np.array_equal(gpu.step_ids, ref.ids) and np.array_equal(gpu.step_nsel, ref.nsel)
    lib.close()


def test_shared_device_switch_never_waits():
    """chess_config.shared_device: every (sequence, KV head) is one workgroup's, so no launch waits for another
    workgroup.  With every wait set to fail at once (any wait would raise the error flag) select, the fused
    step with its tail refresh and the model-wide selection must still return the oracle's lists, flag clear."""
    sp = workload.spec("cfg2", scale=1 / 2)
    wl = workload.generate(sp, workload.default_seed("cfg2"))
    plan = plan_of(sp)
    ref = run_oracle(wl, plan, sp.max_selected, dense=False)
    d = to_device(wl)
    import dataclasses
    lib = pk.Chess(dataclasses.replace(config_of(sp), shared_device=True))
    lib.debug_set_poll_limit(-1)
    lib.debug_force_cluster(8)                                       # must not override the switch
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
    ids = torch.full((1, sp.n_kv_heads, sp.max_selected), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((1, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    out = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
    lib.select(d.q, summ, d.seq_lens, gpu_plan(plan), ids, nsel, ws)
    assert lib.workspace_error(ws) == 0
    assert np.array_equal(ids.cpu().numpy(), ref.ids) and np.array_equal(nsel.cpu().numpy(), ref.nsel)
    ids.fill_(-7); nsel.fill_(-7)
    lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids, nsel, out, ws,
                    refresh_tail=True)
    assert lib.workspace_error(ws) == 0
    assert np.array_equal(ids.cpu().numpy(), ref.ids) and np.array_equal(nsel.cpu().numpy(), ref.nsel)
    assert np.abs(out.cpu().numpy() - ref.out).max() <= ATOL_TIGHT
    anc = torch.empty((1, sp.n_kv_heads, 128), device="cuda")
    lib.anchor(summ, d.seq_lens, plan.window_pages, anc)
    lib.select_shared([anc], [summ], d.seq_lens, gpu_plan(plan), ids, nsel, ws)
    assert lib.workspace_error(ws) == 0
    oanc = oracle.anchor(ref.pages, ref.host[4], geom_of(sp), plan.window_pages)
    sids, sn = oracle.select_shared([oanc], [ref.pages], [ref.chunks], [ref.grids], ref.host[4], geom_of(sp), plan, sp.max_selected)
    assert all(np.array_equal(ids[:, h].cpu().numpy(), sids) for h in range(sp.n_kv_heads))
    lib.close()


@pytest.mark.parametrize("schedule,cluster", [(1, 1), (1, 3), (2, 1), (2, 3), (2, 8)])
def test_schedules_give_the_same_page_lists(schedule, cluster):
    """The two schedules of the levels -- lazy (three phases) and merged (all chunks scored with the grids) -- forced
    in turn: select, the fused step with its tail refresh (window 0 as well, so that the tail page competes), ragged
    lengths, a budget that keeps every grid (no grid cut) and ratios that prune hard."""
    sp = RAGGED
    lens = [3000, 1237, 641, 16 * 16 + 1, 16]
    wl = workload.generate(sp, 83, seq_lens=lens)
    d = to_device(wl)
    for plan in (plan_of(sp), plan_of(sp, window_pages=0, sink_pages=0), plan_of(sp, budget_pages=40),
                 plan_of(sp, plan=oracle.PLAN_RATIO, rho_g_bp=3000, rho_c_bp=3000, rho_p_bp=1000)):
        lib = pk.Chess(config_of(sp, max_selected=sp.max_pages))
        lib.debug_force_schedule(schedule)
        lib.debug_force_cluster(cluster)
        ref = run_oracle(wl, plan, sp.max_pages, dense=False)
        summ, ws = lib.new_summaries(), lib.new_workspace()
        lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
        for refresh in (False, True):
            ids = torch.full((len(lens), sp.n_kv_heads, sp.max_pages), -7, dtype=torch.int32, device="cuda")
            nsel = torch.full((len(lens), sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
            out = torch.full((len(lens), sp.n_q_heads, 128), float("nan"), device="cuda")
            if refresh:
                pv, cv, gv = lib.summary_views(summ)
                for b, L in enumerate(lens):
                    tp = -(-L // 16) - 1
                    pv[b, :, tp] = 5.0; cv[b, :, tp // 4] = -9.0; gv[b, :, tp // 16] = 3.0
                lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids, nsel, out, ws,
                                refresh_tail=True)
            else:
                lib.select(d.q, summ, d.seq_lens, gpu_plan(plan), ids, nsel, ws)
            torch.cuda.synchronize()
            assert lib.workspace_error(ws) == 0
            assert np.array_equal(ids.cpu().numpy(), ref.ids) and np.array_equal(nsel.cpu().numpy(), ref.nsel), (plan, refresh)
            if refresh:
                assert np.abs(out.cpu().numpy() - ref.out).max() <= ATOL_TIGHT
                assert_summaries_equal(GpuRunLike(*host_views(lib, summ, len(lens))), ref, sp, lens)
        lib.close()


@pytest.mark.parametrize("cluster,general", [(1, False), (3, False), (2, True)])
def test_threshold_rule_keeps_every_tie_at_the_cut(cluster, general):
    """CHESS_CUT_THRESHOLD (Alg. 1 stage 2 as printed, S >= tau): tied groups at every level's cut (three distinct key
    rows dealt by page number) are kept whole, through every cut path, against the oracle's threshold mode; on
    continuous scores the rule changes nothing; a list that outgrows its row raises the overflow bit of the
    workspace's error word."""
    sp = workload.WorkloadSpec("groups", 2, (8192, 8192), 4, 1, 16, ("fixed", 128), (1, 1), 1, 2, budget_pages=5,
                               pages_per_chunk=2, chunks_per_grid=2)
    wl = workload.generate(sp, 9, seq_lens=[8192, 5000])
    rows = [wl.k_pool[wl.block_table[0, j].item(), 0, 0].clone() for j in (0, 1, 2)]
    for b in range(2):
        for j in range(-(-int(wl.seq_lens[b]) // 16)):
            wl.k_pool[wl.block_table[b, j].item(), 0, :] = rows[j % 3]
    for bp in (5000, 3000):
        plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=1, window_pages=2, rho_g_bp=bp, rho_c_bp=5000, rho_p_bp=bp,
                           cut_rule=oracle.CUT_THRESHOLD)
        lib = pk.Chess(config_of(sp, max_selected=sp.max_pages))
        lib.debug_force_general_cut(general)
        gpu = run_gpu(lib, wl, plan, dense=False, cluster=cluster)
        ref = run_oracle(wl, plan, sp.max_pages, dense=False)
        assert np.array_equal(gpu.ids, ref.ids) and np.array_equal(gpu.nsel, ref.nsel)
        assert np.array_equal(gpu.step_ids, ref.ids) and np.array_equal(gpu.step_nsel, ref.nsel)
        count = run_oracle(wl, oracle.Plan(**{**plan.__dict__, "cut_rule": oracle.CUT_COUNT}), sp.max_pages, dense=False)
        assert (ref.nsel >= count.nsel).all() and (ref.nsel > count.nsel).any(), "the ties must add pages somewhere"
        lib.close()
    # continuous scores: nothing ties, both rules agree
    wl2 = workload.generate(RAGGED, 77, seq_lens=RAGGED_LENS)
    lib = pk.Chess(config_of(RAGGED, max_selected=RAGGED.max_pages))
    lib.debug_force_general_cut(general)
    a = run_gpu(lib, wl2, plan_of(RAGGED, cut_rule=oracle.CUT_THRESHOLD), dense=False, cluster=cluster)
    ref2 = run_oracle(wl2, plan_of(RAGGED), RAGGED.max_pages, dense=False)
    assert np.array_equal(a.ids, ref2.ids) and np.array_equal(a.nsel, ref2.nsel)
    lib.close()
    # all keys identical, a row too short for all the ties: the list is cut short and the overflow bit is raised
    sp3 = workload.WorkloadSpec("ties", 1, (2048, 2048), 4, 1, 16, ("fixed", 128), (1, 1), 1, 2, budget_pages=5,
                                pages_per_chunk=2, chunks_per_grid=2)
    wl3 = workload.generate(sp3, 3)
    wl3.k_pool[:] = wl3.k_pool[wl3.block_table[0, 0].item(), 0, 0].clone()
    d3 = to_device(wl3)
    lib = pk.Chess(config_of(sp3, max_selected=20))
    lib.debug_force_general_cut(general)
    lib.debug_force_cluster(cluster)
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(d3.k_pool, d3.block_table, d3.seq_lens, summ)
    ids = torch.full((1, 1, 20), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((1, 1), -7, dtype=torch.int32, device="cuda")
    lib.select(d3.q, summ, d3.seq_lens, gpu_plan(plan_of(sp3, cut_rule=oracle.CUT_THRESHOLD)), ids, nsel, ws)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) & 2, "every page ties: 125 candidates cannot fit 17 places"
    assert int(nsel[0, 0]) == 20 and ids[0, 0].tolist() == list(range(0, 18)) + [126, 127]
    lib.close()


@pytest.mark.parametrize("schedule,cluster", [(1, 0), (2, 0), (2, 5)])
def test_long_context_with_more_than_1024_chunks(schedule, cluster):
    """200K tokens in 16-token pages: 12500 pages, 1563 chunks, 196 grids.  Under the merged schedule the chunk cut
    runs over more than 1024 unit-ordered keys with the kept-grid mask (the many-keys-per-thread cut); the tail
    refresh rides along; ragged second sequence."""
    sp = workload.WorkloadSpec("long", 2, (1000, 200000), 8, 2, 16, ("geometric", 256), (1, 3), 1, 4, budget_bp=100)
    wl = workload.generate(sp, 91, seq_lens=[200000, 70001])
    plan = plan_of(sp)
    ref = run_oracle(wl, plan, sp.max_selected, dense=False)
    d = to_device(wl)
    lib = pk.Chess(config_of(sp))
    lib.debug_force_schedule(schedule)
    lib.debug_force_cluster(cluster)
    summ, ws = lib.new_summaries(), lib.new_workspace()
    lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
    pv, cv, gv = lib.summary_views(summ)
    for b, L in enumerate([200000, 70001]):
        tp = -(-L // 16) - 1
        pv[b, :, tp] = 3.0; cv[b, :, tp // 8] = -2.0; gv[b, :, tp // 64] = 9.0
    ids = torch.full((2, sp.n_kv_heads, sp.max_selected), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((2, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    out = torch.full((2, sp.n_q_heads, 128), float("nan"), device="cuda")
    lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids, nsel, out, ws, refresh_tail=True)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    assert np.array_equal(ids.cpu().numpy(), ref.ids) and np.array_equal(nsel.cpu().numpy(), ref.nsel)
    assert np.abs(out.cpu().numpy() - ref.out).max() <= ATOL_TIGHT
    ids2, nsel2 = torch.full_like(ids, -7), torch.full_like(nsel, -7)
    lib.select(d.q, summ, d.seq_lens, gpu_plan(plan), ids2, nsel2, ws)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    assert torch.equal(ids2, ids) and torch.equal(nsel2, nsel)
    lib.close()
