"""GPU parity of the model-wide scope (Sec. 3.1 Eq. 1 flattening over layers and heads, Sec. 3.2 Eq. 3 anchor):
chess_anchor and chess_select_shared through the C ABI against the oracle, bit-exact page lists; then the
per-layer sparse attention over the shared list within 1e-2."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2602_20732_amd as pk
import workload
from gpu_common import config_of, gpu_plan, to_device
from helpers import geom_of, host_arrays, plan_of

pytestmark = pytest.mark.gpu


def layers_of(sp, seeds, lens):
    return [workload.generate(sp, seed, seq_lens=lens) for seed in seeds]


def run_both(sp, wls, plan, cluster=0, window=None, max_sel=None):
    """(gpu ids, gpu n_selected, gpu anchors, oracle ids [b, max_sel], oracle n_selected [b], oracle anchors, lib, device layers, summaries)."""
    max_sel = sp.max_selected if max_sel is None else max_sel
    g = geom_of(sp)
    window = plan.window_pages if window is None else window
    lib = pk.Chess(config_of(sp, max_selected=max_sel))
    batch = wls[0].seq_lens.shape[0]
    ds = [to_device(w) for w in wls]
    summs, probes = [], []
    for d in ds:
        s = lib.new_summaries()
        lib.summarize(d.k_pool, d.block_table, d.seq_lens, s)
        summs.append(s)
        probes.append(torch.full((batch, sp.n_kv_heads, 128), float("nan"), device="cuda"))
    lib.anchor(summs, ds[0].seq_lens, window, probes)                  # all layers in one launch
    ws = lib.new_workspace()
    ids = torch.full((batch, sp.n_kv_heads, max_sel), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((batch, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    lib.debug_force_cluster(cluster)
    lib.select_shared(probes, summs, ds[0].seq_lens, gpu_plan(plan), ids, nsel, ws)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    # the oracle, from its own summaries
    host = [host_arrays(w) for w in wls]
    sl = host[0][4]
    osum = [oracle.summarize(K, bt, sl, g) for (K, V, Q, bt, _) in host]
    oanc = [oracle.anchor(x[0], sl, g, window) for x in osum]
    oids, onsel = oracle.select_shared(oanc, [x[0] for x in osum], [x[1] for x in osum], [x[2] for x in osum], sl, g,
                                       plan, max_sel)
    return (ids.cpu().numpy(), nsel.cpu().numpy(), [p.cpu().numpy() for p in probes], oids, onsel, oanc, lib, ds, summs,
            host)


def assert_lists_equal(ids, nsel, oids, onsel, H):
    for h in range(H):                                   # the sequence's list, once per KV head
        assert np.array_equal(ids[:, h], oids), f"page list of head {h}"
        assert np.array_equal(nsel[:, h], onsel)


SP = workload.WorkloadSpec("ragged", 5, (0, 3000), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_bp=300,
                           pages_per_chunk=4, chunks_per_grid=4)
LENS = [3000, 1237, 641, 16, 0]


@pytest.mark.parametrize("n_layers,cluster", [(1, 1), (3, 0), (3, 2), (5, 7)])
def test_shared_scope_on_a_ragged_batch(n_layers, cluster):
    wls = layers_of(SP, range(40, 40 + n_layers), LENS)
    for kw in (dict(), dict(plan=oracle.PLAN_RATIO, rho_g_bp=5000, rho_c_bp=5000, rho_p_bp=2500),
               dict(plan=oracle.PLAN_FLAT, budget_pages=11)):
        plan = plan_of(SP, **kw)
        ids, nsel, anc, oids, onsel, oanc, lib, ds, summs, host = run_both(SP, wls, plan, cluster, max_sel=SP.max_pages)
        for a, o in zip(anc, oanc):
            assert np.array_equal(a.view(np.uint32), o.view(np.uint32)), "anchor vectors"
        assert_lists_equal(ids, nsel, oids, onsel, SP.n_kv_heads)
        lib.close()


def test_shared_scope_at_cfg1_then_attention_per_layer():
    """Four layers of the 4K configuration (8 KV heads: 32 rows per unit), automatic cluster; every layer then
    attends over the shared list, against the oracle's attention over the oracle's list."""
    sp = workload.spec("cfg1")
    wls = layers_of(sp, [workload.default_seed("cfg1") + i for i in range(4)], None)
    plan = plan_of(sp)
    ids, nsel, anc, oids, onsel, oanc, lib, ds, summs, host = run_both(sp, wls, plan)
    assert_lists_equal(ids, nsel, oids, onsel, sp.n_kv_heads)
    g = geom_of(sp)
    ws = lib.new_workspace()
    ids_d, nsel_d = torch.as_tensor(ids).cuda(), torch.as_tensor(nsel).cuda()
    o_ids = np.repeat(oids[:, None, :], sp.n_kv_heads, axis=1)
    o_n = np.repeat(onsel[:, None], sp.n_kv_heads, axis=1)
    for d, (K, V, Q, bt, sl) in zip(ds, host):
        out = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
        lib.sparse_decode(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, ids_d, nsel_d, out, ws)
        ref = oracle.attend(Q, K, V, bt, sl, g, o_ids, o_n)
        err = np.abs(out.cpu().numpy() - ref).max()
        assert np.isfinite(err) and err <= 2e-3
    lib.close()


def test_shared_scope_with_identical_units_ties_to_the_lowest_pages():
    """Every key row the same in every layer: all scores of a level tie exactly, whichever group or member
    computed them, so the kept pages are the lowest candidates."""
    sp = workload.WorkloadSpec("ties", 1, (2048, 2048), 4, 2, 16, ("fixed", 128), (1, 1), 1, 2, budget_pages=6,
                               pages_per_chunk=4, chunks_per_grid=4)
    wls = layers_of(sp, [3, 4], None)
    row = torch.linspace(-1, 1, 128).to(torch.bfloat16)
    for w in wls:
        w.k_pool[:] = row
    plan = plan_of(sp)
    for cluster in (1, 5):
        ids, nsel, anc, oids, onsel, oanc, lib, ds, summs, host = run_both(sp, wls, plan, cluster)
        assert_lists_equal(ids, nsel, oids, onsel, sp.n_kv_heads)
        assert oids[0, :onsel[0]].tolist() == [0, 1, 2, 3, 4, 5, 6, 126, 127]
        lib.close()


def test_shared_scope_refusals():
    sp = workload.spec("cfg1")
    lib = pk.Chess(config_of(sp))
    wl = to_device(workload.generate(sp, 1))
    s, ws = lib.new_summaries(), lib.new_workspace()
    a = torch.zeros((1, sp.n_kv_heads, 128), device="cuda")
    ids = torch.zeros((1, sp.n_kv_heads, sp.max_selected), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((1, sp.n_kv_heads), dtype=torch.int32, device="cuda")
    with pytest.raises(pk.ChessError):
        lib.anchor(s, wl.seq_lens, 0, a)                                       # no window
    with pytest.raises(pk.ChessError):
        lib.select_shared([a] * 65, [s] * 65, wl.seq_lens, gpu_plan(plan_of(sp)), ids, nsel, ws)   # too many layers
    with pytest.raises(pk.ChessError):
        lib.select_shared([a[:, :, 1:]], [s], wl.seq_lens, gpu_plan(plan_of(sp)), ids, nsel, ws)   # misaligned probe
    lib.close()


@pytest.mark.parametrize("batch,lo,hi,n_layers,sample", [(32, 16384, 32768, 32, (0, 21)), (8, 131072, 131072, 8, (5,))])
def test_shared_scope_at_benchmark_shapes(batch, lo, hi, n_layers, sample):
    """The launch shapes of the benchmark (32 KV-head rows x layers per unit, automatic cluster) on summary buffers
    filled with seeded normal vectors (the selection reads nothing else); whole sampled sequences against the oracle."""
    sp = workload.WorkloadSpec("shape", batch, (lo, hi), 32, 8, 16, ("fixed", 128), (3, 3), 1, 4, budget_bp=100)
    g = geom_of(sp)
    plan = plan_of(sp)
    lib = pk.Chess(config_of(sp))
    gen = torch.Generator(device="cuda").manual_seed(1234)
    lens = torch.randint(lo, hi + 1, (batch,), generator=torch.Generator().manual_seed(7)).to(torch.int32)
    sl = lens.cuda()
    summs, probes = [], []
    for _ in range(n_layers):
        s = lib.new_summaries()
        for t in lib.summary_views(s):
            t.normal_(generator=gen)
        summs.append(s)
        probes.append(torch.empty((batch, sp.n_kv_heads, 128), device="cuda"))
    lib.anchor(summs, sl, plan.window_pages, probes)
    ws = lib.new_workspace()
    ids = torch.full((batch, sp.n_kv_heads, sp.max_selected), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((batch, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    lib.select_shared(probes, summs, sl, gpu_plan(plan), ids, nsel, ws)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0
    ids_h, nsel_h = ids.cpu().numpy(), nsel.cpu().numpy()
    assert (ids_h == ids_h[:, :1]).all() and (nsel_h == nsel_h[:, :1]).all()
    for b in sample:
        pv, cv, gv = [], [], []
        for s in summs:
            p, c, gr = lib.summary_views(s)
            pv.append(p[b:b + 1].float().cpu().numpy()); cv.append(c[b:b + 1].float().cpu().numpy()); gv.append(gr[b:b + 1].float().cpu().numpy())
        one = lens[b:b + 1].numpy()
        oanc = [oracle.anchor(p, one, g, plan.window_pages) for p in pv]
        for a, o in zip(probes, oanc):
            assert np.array_equal(a[b:b + 1].cpu().numpy().view(np.uint32), o.view(np.uint32))
        oids, on = oracle.select_shared(oanc, pv, cv, gv, one, g, plan, sp.max_selected)
        assert nsel_h[b, 0] == on[0] and np.array_equal(ids_h[b, 0], oids[0]), (b, "page list")
        print(f"[shared {batch}x{n_layers}] seq {b} ({int(lens[b])} tokens): page list exact, {on[0]} pages")
    lib.close()


@pytest.mark.parametrize("seed", range(16))
def test_shared_scope_random_shapes(seed):
    """Seeded draws of geometry, batch, lengths, layers, plan and cluster size."""
    rng = np.random.default_rng(7000 + seed)
    B, H = int(rng.choice([16, 32])), int(rng.choice([1, 2, 4, 8]))
    nc, ng = int(rng.choice([1, 2, 4, 5, 8])), int(rng.choice([1, 2, 3, 8]))
    batch, hi = int(rng.integers(1, 4)), int(rng.choice([400, 2000, 6000]))
    lens = [hi] + [int(rng.integers(0, hi + 1)) for _ in range(batch - 1)]
    s, w = int(rng.choice([0, 1, 2])), int(rng.choice([1, 2, 4]))
    kind = int(rng.choice([oracle.PLAN_BUDGET, oracle.PLAN_RATIO, oracle.PLAN_FLAT]))
    kw = dict(plan=kind, sink_pages=s, window_pages=w)
    if kind == oracle.PLAN_RATIO:
        kw.update(rho_g_bp=int(rng.integers(1, 10001)), rho_c_bp=int(rng.integers(1, 10001)), rho_p_bp=int(rng.integers(1, 10001)))
    else:
        kw.update(budget_pages=int(rng.integers(1, 30)), over_chunk=int(rng.integers(1, 12)), over_grid=int(rng.integers(1, 8)))
    n_layers, cluster = int(rng.integers(1, 7)), int(rng.choice([0, 1, 3, 9]))
    sp = workload.WorkloadSpec(f"srand{seed}", batch, (0, hi), H, H, B, ("fixed", 96), (1, 1), s, w,
                               pages_per_chunk=nc, chunks_per_grid=ng)
    print(f"[shared rand {seed}] page {B} H {H} fan {nc}x{ng} lens {lens} layers {n_layers} plan {kw} cluster {cluster}", flush=True)
    wls = layers_of(sp, range(900 + 10 * seed, 900 + 10 * seed + n_layers), lens)
    ids, nsel, anc, oids, onsel, oanc, lib, ds, summs, host = run_both(sp, wls, plan_of(sp, **kw), cluster, max_sel=sp.max_pages)
    for a, o in zip(anc, oanc):
        assert np.array_equal(a.view(np.uint32), o.view(np.uint32)), "anchor vectors"
    assert_lists_equal(ids, nsel, oids, onsel, sp.n_kv_heads)
    lib.close()
