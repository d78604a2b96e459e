"""Seeded random shapes for the oracle's own pins (CPU only): on every draw of geometry, lengths and plan the page
lists obey the structural invariants of Sec. 3.2 (safety pages, order, containment of kept pages in kept chunks in
kept grids, integer keep-counts), the flat plan equals a stable argsort of page scores rebuilt with numpy from the raw
keys, and a budget that covers every candidate makes the sparse attention equal the dense one."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
import workload
from helpers import bf16_to_f64, geom_of, host_arrays, logical_kv, plan_of


def draw(seed):
    rng = np.random.default_rng(9000 + seed)
    B, H, G = int(rng.choice([16, 32])), int(rng.choice([1, 2, 3])), int(rng.choice([1, 2, 4]))
    nc, ng = int(rng.choice([1, 2, 3, 4, 8])), int(rng.choice([1, 2, 4, 8]))
    batch, hi = int(rng.integers(1, 4)), int(rng.choice([200, 900, 2500]))
    lens = [hi] + [int(rng.integers(0, hi + 1)) for _ in range(batch - 1)]
    s, w = int(rng.choice([0, 1, 2])), int(rng.choice([0, 1, 3]))
    sp = workload.WorkloadSpec(f"orand{seed}", batch, (0, hi), H * G, H, B, ("fixed", 64), (2, 2), s, w,
                               pages_per_chunk=nc, chunks_per_grid=ng)
    return rng, sp, lens


@pytest.mark.parametrize("seed", range(20))
def test_random_shape_invariants_flat_plan_and_full_budget(seed):
    rng, sp, lens = draw(seed)
    wl = workload.generate(sp, 70 + seed, seq_lens=lens)
    K, V, Q, bt, sl = host_arrays(wl)
    g = geom_of(sp)
    B, Nc, Ng, s, w = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid, sp.sink_pages, sp.window_pages
    pv, cv, gv = oracle.summarize(K, bt, sl, g)

    # (1) structural invariants under a random ratio plan and a random budget plan
    for kw in (dict(plan=oracle.PLAN_RATIO, rho_g_bp=int(rng.integers(1, 10001)), rho_c_bp=int(rng.integers(1, 10001)),
                    rho_p_bp=int(rng.integers(1, 10001))),
               dict(plan=oracle.PLAN_BUDGET, budget_pages=int(rng.integers(1, 20)), over_chunk=int(rng.integers(1, 12)),
                    over_grid=int(rng.integers(1, 8)))):
        plan = plan_of(sp, **kw)
        ids, nsel, kg, kc, cnt = oracle.select(Q, pv, cv, gv, sl, g, plan, sp.max_pages, detail=True)
        for b, L in enumerate(lens):
            P = -(-L // B); nch = -(-P // Nc); ngr = -(-nch // Ng)
            for h in range(sp.n_kv_heads):
                row = ids[b, h, :nsel[b, h]].tolist()
                assert row == sorted(set(row)) and all(0 <= p < P for p in row) and (ids[b, h, nsel[b, h]:] == -1).all()
                if P <= s + w:
                    assert row == list(range(P))
                    continue
                assert set(range(s)) <= set(row) and set(range(P - w, P)) <= set(row)
                k_g, k_c, k_p = cnt[b, h]
                assert kg[b, h, :ngr].sum() == k_g and kc[b, h, :nch].sum() == k_c and nsel[b, h] == s + k_p + w
                assert not kg[b, h, ngr:].any() and not kc[b, h, nch:].any()
                for c in np.flatnonzero(kc[b, h]):
                    assert kg[b, h, c // Ng], "a kept chunk's grid is kept"
                for p in row:
                    if s <= p < P - w:
                        assert kc[b, h, p // Nc], "a kept page's chunk is kept"
                if kw["plan"] == oracle.PLAN_RATIO:
                    ceil_bp = lambda n, bp: (n * bp + 9999) // 10000
                    assert k_g == min(max(ceil_bp(ngr, plan.rho_g_bp), 1), ngr)
                    n_act = sum(min(Ng, nch - gi * Ng) for gi in np.flatnonzero(kg[b, h]))
                    assert k_c == min(max(ceil_bp(n_act, plan.rho_c_bp), 1), n_act)

    # (2) the flat plan is a stable argsort of page scores rebuilt from the raw keys
    k = int(rng.integers(1, 12))
    flat = plan_of(sp, plan=oracle.PLAN_FLAT, budget_pages=k)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, flat, sp.max_pages)
    for b, L in enumerate(lens):
        P = -(-L // B)
        if P <= s + w:
            continue
        for h in range(sp.n_kv_heads):
            probe = bf16_to_f64(Q[b, h * sp.group:(h + 1) * sp.group]).sum(0)
            Kl, _ = logical_kv(K, V, bt, L, b, h)
            score = np.array([(Kl[j * B:min(L, (j + 1) * B)] @ probe).mean() for j in range(P)])
            cand = np.arange(s, P - w)
            order = cand[np.argsort(-score[cand], kind="stable")]
            kk = min(k, len(cand))
            if kk < len(cand) and score[order[kk - 1]] - score[order[kk]] < 1e-6:
                continue                                     # a near-tie at the cut: fp64 summation order decides
            want = sorted(list(range(s)) + order[:kk].tolist() + list(range(P - w, P)))
            assert ids[b, h, :nsel[b, h]].tolist() == want, (b, h)

    # (3) a budget that covers every candidate: sparse == dense
    full = plan_of(sp, plan=oracle.PLAN_RATIO)                # ratios 1, 1, 1
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, full, sp.max_pages)
    sparse = oracle.attend(Q, K, V, bt, sl, g, ids, nsel)
    dense = oracle.attend(Q, K, V, bt, sl, g)
    assert np.array_equal(sparse, dense)
