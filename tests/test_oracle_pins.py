"""Pins for the CPU oracle: each test checks ``oracle/`` against something other than itself --
values the paper prints, closed forms, a textbook routine, brute force, or an invariant the method
states -- so that a dropped term, wrong sign / index or transposed operand in the oracle fails here.
CPU only."""
from __future__ import annotations

import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workload
from helpers import (bf16_to_f64, f32_to_bf16_bits, geom_of, host_arrays, listed_tokens, logical_kv, pack_pools,
                     plan_of, softmax_attention)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def cfg1():
    sp = workload.spec("cfg1")
    wl = workload.generate(sp, workload.default_seed("cfg1"))
    return sp, wl, host_arrays(wl)


@pytest.fixture(scope="module")
def ragged():
    """GQA 4, three sequences with a partial tail page, a partial last chunk and a partial last grid."""
    sp = workload.WorkloadSpec("ragged", 3, (64, 3000), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_bp=300,
                               pages_per_chunk=4, chunks_per_grid=4)
    wl = workload.generate(sp, 77, seq_lens=[3000, 1237, 641])
    return sp, wl, host_arrays(wl)


# ------------------------------------------------------------------ P1: Full-KV == textbook attention
def test_dense_equals_textbook_attention(ragged):
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    out = oracle.attend(Q, K, V, bt, sl, g)
    G = sp.group
    for b in range(sp.batch):
        for hq in range(sp.n_q_heads):
            Kl, Vl = logical_kv(K, V, bt, sl[b], b, hq // G)
            ref = softmax_attention(bf16_to_f64(Q[b, hq]), Kl, Vl, 1.0 / np.sqrt(sp.head_dim))
            np.testing.assert_allclose(out[b, hq], ref, rtol=0, atol=2e-7)


def test_budget_covering_all_pages_is_dense(ragged):
    """rho = 1 at every level is the paper's Full-KV (Sec. 5.1): same pages, hence the same numbers."""
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    for plan in (plan_of(sp, plan=oracle.PLAN_RATIO),                       # ratios default to 1,1,1
                 plan_of(sp, plan=oracle.PLAN_FLAT, budget_pages=sp.max_pages),
                 plan_of(sp, plan=oracle.PLAN_BUDGET, budget_pages=sp.max_pages)):
        ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, sp.max_pages)
        for b in range(sp.batch):
            P = -(-sl[b] // sp.page_size)
            assert (nsel[b] == P).all()
            assert (ids[b, :, :P] == np.arange(P)).all()
        sparse = oracle.attend(Q, K, V, bt, sl, g, ids, nsel)
        dense = oracle.attend(Q, K, V, bt, sl, g)
        assert np.array_equal(sparse, dense)


def test_sparse_attention_is_textbook_on_listed_tokens(ragged):
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp), sp.max_selected)
    out = oracle.attend(Q, K, V, bt, sl, g, ids, nsel)
    G = sp.group
    for b in range(sp.batch):
        for hq in (0, 3, 5):
            h = hq // G
            Kl, Vl = logical_kv(K, V, bt, sl[b], b, h)
            toks = listed_tokens(ids[b, h], nsel[b, h], sl[b], sp.page_size)
            ref = softmax_attention(bf16_to_f64(Q[b, hq]), Kl[toks], Vl[toks], 1.0 / np.sqrt(sp.head_dim))
            np.testing.assert_allclose(out[b, hq], ref, rtol=0, atol=2e-7)


# ------------------------------------------------------------------ P4: softmax rows and convexity
def test_softmax_rows_sum_to_one_and_output_is_convex(cfg1):
    sp, wl, (K, V, Q, bt, sl) = cfg1
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp), sp.max_selected)
    for hq in (0, 5):
        out, wts = oracle.attend(Q, K, V, bt, sl, g, ids, nsel, weights_head=hq)
        h = hq // sp.group
        toks = listed_tokens(ids[0, h], nsel[0, h], sl[0], sp.page_size)
        w = wts[:len(toks)]
        assert (w >= 0).all() and abs(w.sum() - 1.0) < 1e-12 and (wts[len(toks):] == 0).all()
        _, Vl = logical_kv(K, V, bt, sl[0], 0, h)
        assert (out[0, hq] <= Vl[toks].max(0) + 1e-6).all() and (out[0, hq] >= Vl[toks].min(0) - 1e-6).all()
        np.testing.assert_allclose(out[0, hq], w @ Vl[toks], atol=2e-7)


# ------------------------------------------------------------------ P3: Eq. 1, 2, 4 are linear
def test_scores_are_means_of_child_scores(cfg1):
    """On full units S(chunk) = mean S(page), S(grid) = mean S(chunk), S(page) = mean_t probe.K_t."""
    sp, wl, (K, V, Q, bt, sl) = cfg1
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    ps, cs, gs = oracle.scores(Q, pv, cv, gv, sl, g)
    Nc, Ng, B = sp.pages_per_chunk, sp.chunks_per_grid, sp.page_size
    for h in range(sp.n_kv_heads):
        probe = bf16_to_f64(Q[0, h * sp.group:(h + 1) * sp.group]).sum(0)
        Kl, _ = logical_kv(K, V, bt, sl[0], 0, h)
        tok_scores = Kl @ probe
        np.testing.assert_allclose(ps[0, h], tok_scores.reshape(-1, B).mean(1), rtol=1e-5, atol=1e-5)
        np.testing.assert_allclose(cs[0, h], ps[0, h].reshape(-1, Nc).mean(1), rtol=1e-5, atol=1e-5)
        np.testing.assert_allclose(gs[0, h], cs[0, h].reshape(-1, Ng).mean(1), rtol=1e-5, atol=1e-5)


def test_partial_units_average_over_existing_members(ragged):
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    B, Nc, Ng = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    for b in range(sp.batch):
        L = int(sl[b]); P = -(-L // B); nc = -(-P // Nc); ng = -(-nc // Ng)
        for h in range(sp.n_kv_heads):
            Kl, _ = logical_kv(K, V, bt, L, b, h)
            tail = Kl[(P - 1) * B:L].mean(0)
            np.testing.assert_allclose(pv[b, h, P - 1], tail, rtol=1e-6, atol=1e-7)
            np.testing.assert_allclose(cv[b, h, nc - 1], pv[b, h, (nc - 1) * Nc:P].astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)
            np.testing.assert_allclose(gv[b, h, ng - 1], cv[b, h, (ng - 1) * Ng:nc].astype(np.float64).mean(0), rtol=1e-6, atol=1e-7)
            assert not pv[b, h, P:].any() and not cv[b, h, nc:].any() and not gv[b, h, ng:].any()


# ------------------------------------------------------------------ bf16 storage of the summaries
def test_bf16_summaries_are_the_rounded_means(ragged):
    """The bf16 switch: a stored page vector is the fp32 mean rounded to nearest-even bf16 -- which is what torch's
    own conversion gives, from the fp32 mean and from the fp64 mean alike -- and a chunk / grid vector is the
    rounded mean of the STORED child vectors (not of the exact ones).  Everything built here with numpy + torch."""
    import torch
    sp, wl, (K, V, Q, bt, sl) = ragged
    g32, g16 = geom_of(sp), geom_of(sp, summary_dtype=oracle.SUMMARY_BF16)
    pv32, cv32, gv32 = oracle.summarize(K, bt, sl, g32)
    pv, cv, gv = oracle.summarize(K, bt, sl, g16)
    to_bf = lambda a: torch.as_tensor(np.ascontiguousarray(a)).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(pv, to_bf(pv32))
    B, Nc, Ng = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    differs = 0
    for b in range(sp.batch):
        L = int(sl[b]); P = -(-L // B); nc = -(-P // Nc); ng = -(-nc // Ng)
        for h in range(sp.n_kv_heads):
            Kl, _ = logical_kv(K, V, bt, L, b, h)
            means = np.stack([Kl[j * B:min((j + 1) * B, L)].mean(0) for j in range(P)])          # fp64, numpy's own summation
            assert np.abs(to_bf(means.astype(np.float64)) - pv[b, h, :P]).max() <= 2.0 ** -7 * np.abs(means).max()   # <= 1 bf16 ulp (summation order)
            cref = np.stack([pv[b, h, c * Nc:min(P, (c + 1) * Nc)].astype(np.float64).mean(0) for c in range(nc)])
            assert np.array_equal(cv[b, h, :nc], to_bf(cref.astype(np.float32)))
            gref = np.stack([cv[b, h, k * Ng:min(nc, (k + 1) * Ng)].astype(np.float64).mean(0) for k in range(ng)])
            assert np.array_equal(gv[b, h, :ng], to_bf(gref.astype(np.float32)))
            differs += int((cv[b, h, :nc] != to_bf(cv32[b, h, :nc])).sum())
            assert (pv[b, h, :P].view(np.uint32) & 0xffff == 0).all()
    assert differs > 0, "averaging stored children must differ somewhere from rounding the fp32 chunk means"
    # the scores and the selection read the stored values: flat plan == stable argsort of numpy's dots with them
    ps, _, _ = oracle.scores(Q, pv, cv, gv, sl, g16)
    k, s, w = 9, sp.sink_pages, sp.window_pages
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g16, plan_of(sp, plan=oracle.PLAN_FLAT, budget_pages=k), s + w + k)
    for b in range(sp.batch):
        P = -(-int(sl[b]) // B)
        for h in range(sp.n_kv_heads):
            probe = bf16_to_f64(Q[b, h * sp.group:(h + 1) * sp.group]).sum(0)
            sc = pv[b, h, :P].astype(np.float64) @ probe
            np.testing.assert_allclose(ps[b, h, :P], sc, rtol=1e-12, atol=1e-12)
            cand = np.arange(s, P - w)
            top = cand[np.argsort(-sc[cand], kind="stable")][:k]
            assert ids[b, h, :nsel[b, h]].tolist() == sorted(set(range(s)) | set(top.tolist()) | set(range(P - w, P)))


def test_bf16_summaries_keep_table1_budgets():
    """The keep-counts are integer arithmetic on the hierarchy's shape: the storage type of the vectors does not
    enter (Table 1's budgets are reproduced in both modes)."""
    P, Nc, Ng = 640, 8, 8
    rng = np.random.default_rng(4)
    Klog = rng.standard_normal((P, 1, 16)).astype(np.float32)
    K, V, bt = pack_pools(Klog, Klog, 1)
    Q = f32_to_bf16_bits(rng.standard_normal((1, 1, 16)).astype(np.float32))
    sl = np.array([P], np.int32)
    for line in open(os.path.join(GOLDEN, "table1_budgets.txt")):
        f = line.split("#")[0].split()
        if len(f) < 5:
            continue
        rho = [int(round(float(x) * 10000)) for x in f[1:4]]
        counts = []
        for dt in (oracle.SUMMARY_F32, oracle.SUMMARY_BF16):
            g = oracle.Geometry(1, 1, 16, 1, Nc, Ng, P, dt)
            pv, cv, gv = oracle.summarize(K, bt, sl, g)
            plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=0, window_pages=0, rho_g_bp=rho[0], rho_c_bp=rho[1], rho_p_bp=rho[2])
            _, nsel, _, _, cnt = oracle.select(Q, pv, cv, gv, sl, g, plan, P, detail=True)
            counts.append((int(nsel[0, 0]), cnt[0, 0].tolist()))
        assert counts[0] == counts[1]
        assert abs(100.0 * counts[1][0] / P - float(f[4])) <= 1.0       # the printed budget, to the percent


# ------------------------------------------------------------------ P2: flat plan == brute-force top-k
@pytest.mark.parametrize("which", ["cfg1", "ragged"])
def test_flat_plan_is_bruteforce_topk(which, cfg1, ragged):
    """Page scores rebuilt from raw token dots of the group-summed query (not from the oracle's summaries),
    stable argsort, first k -- on a G=1 and a G=4 (ragged, partial tail page) workload."""
    sp, wl, (K, V, Q, bt, sl) = cfg1 if which == "cfg1" else ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    k, s, w, B = 16, sp.sink_pages, sp.window_pages, sp.page_size
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp, plan=oracle.PLAN_FLAT, budget_pages=k), s + w + k)
    for b in range(sp.batch):
        L = int(sl[b]); P = -(-L // B)
        for h in range(sp.n_kv_heads):
            probe = bf16_to_f64(Q[b, h * sp.group:(h + 1) * sp.group]).sum(0)
            Kl, _ = logical_kv(K, V, bt, L, b, h)
            ts = Kl @ probe
            page_scores = np.array([ts[j * B:min(L, (j + 1) * B)].mean() for j in range(P)])
            cand = np.arange(s, P - w)
            order = cand[np.argsort(-page_scores[cand], kind="stable")]
            gap = page_scores[order[k - 1]] - page_scores[order[k]]
            assert gap > 1e-4, "seed gives a near-tie at the cut; pick another"
            expect = sorted(list(range(s)) + order[:k].tolist() + list(range(P - w, P)))
            assert nsel[b, h] == s + k + w
            assert ids[b, h, :s + k + w].tolist() == expect


def test_softmax_is_stable_for_large_logits():
    """Logits near +-3000: exp() of the raw logits overflows; the result must still be the textbook one."""
    rng = np.random.default_rng(8)
    L, d = 64, 16
    Klog = (rng.standard_normal((L, 1, d)) * 40).astype(np.float32)
    Vlog = rng.standard_normal((L, 1, d)).astype(np.float32)
    K, V, bt = pack_pools(Klog, Vlog, 8)
    g = oracle.Geometry(1, 1, d, 8, 2, 2, 8)
    Q = f32_to_bf16_bits((rng.standard_normal((1, 1, d)) * 40).astype(np.float32))
    sl = np.array([L], np.int32)
    out = oracle.attend(Q, K, V, bt, sl, g)
    Kl, Vl = logical_kv(K, V, bt, L, 0, 0)
    z = Kl @ bf16_to_f64(Q[0, 0]) / np.sqrt(d)
    assert z.max() > 800
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out[0, 0], softmax_attention(bf16_to_f64(Q[0, 0]), Kl, Vl, 1 / np.sqrt(d)), atol=1e-6)


def _exact_cascade(a, Nc, Ng, plan, rho=None, k=None, threshold=False):
    """Brute-force cascade on exact rational page scores ``a`` (no sink / window), written independently
    of the oracle: every level sorts (score desc, index asc) with Python's sort on Fractions.
    threshold: Alg. 1 stage 2 as printed -- a level keeps every active unit whose score is >= the kk-th largest."""
    P = len(a)
    nc, ng = -(-P // Nc), -(-(-(-P // Nc)) // Ng)
    ps = [Fraction(x) for x in a]
    cs = [sum(ps[c * Nc:min(P, (c + 1) * Nc)]) / len(ps[c * Nc:min(P, (c + 1) * Nc)]) for c in range(nc)]
    gs = [sum(cs[u * Ng:min(nc, (u + 1) * Ng)]) / len(cs[u * Ng:min(nc, (u + 1) * Ng)]) for u in range(ng)]

    def top(cands, sc, kk):
        order = sorted(cands, key=lambda i: (-sc[i], i))
        if threshold and 0 < kk <= len(order):
            tau = sc[order[kk - 1]]
            return {i for i in cands if sc[i] >= tau}
        return set(order[:kk])

    def cnt(n, bp):
        return max(1, min(n, -(-n * bp // 10000)))
    if plan == "flat":
        return sorted(top(range(P), ps, k))
    G = top(range(ng), gs, cnt(ng, rho[0]))
    cc = [c for c in range(nc) if c // Ng in G]
    C = top(cc, cs, cnt(len(cc), rho[1]))
    pp = [p for p in range(P) if p // Nc in C]
    return sorted(top(pp, ps, cnt(len(pp), rho[2])))


def _one_hot_problem(a, Nc, Ng):
    """One-token pages; page i's key is a_i * e_i and the single query row is all ones, so S(page i) = a_i
    exactly and every chunk / grid score is an exact dyadic mean."""
    P = len(a)
    Klog = np.zeros((P, 1, P), np.float32)
    Klog[np.arange(P), 0, np.arange(P)] = a
    Vlog = np.arange(P * P, dtype=np.float32).reshape(P, 1, P) % 7
    K, V, bt = pack_pools(Klog, Vlog, 1)
    g = oracle.Geometry(1, 1, P, 1, Nc, Ng, P)
    Q = f32_to_bf16_bits(np.ones((1, 1, P), np.float32))
    sl = np.array([P], np.int32)
    return K, V, Q, bt, sl, g


def test_cascade_matches_hand_worked_example():
    lines = [l.split("#")[0].strip() for l in open(os.path.join(GOLDEN, "cascade_worked.txt"))]
    lines = [l for l in lines if l]
    a = [int(x) for x in lines[0].split()[1:]]
    K, V, Q, bt, sl, g = _one_hot_problem(a, 2, 2)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    checked = 0
    for l in lines[1:]:
        lhs, rhs = l.split("->")
        want = [int(x) for x in rhs.split()]
        f = lhs.split()
        if f[0] == "ratio":
            plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=0, window_pages=0, rho_g_bp=int(f[1]),
                               rho_c_bp=int(f[2]), rho_p_bp=int(f[3]))
            assert _exact_cascade(a, 2, 2, "ratio", rho=[int(x) for x in f[1:4]]) == want
        else:
            plan = oracle.Plan(plan=oracle.PLAN_FLAT, sink_pages=0, window_pages=0, budget_pages=int(f[1]))
            assert _exact_cascade(a, 2, 2, "flat", k=int(f[1])) == want
        ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, 16)
        assert ids[0, 0, :nsel[0, 0]].tolist() == want, l
        checked += 1
    assert checked == 4


@pytest.mark.parametrize("seed", range(6))
def test_cascade_matches_exact_bruteforce_with_many_ties(seed):
    """Small integer scores -> many exact ties at every level, ragged hierarchy; exact rational brute force."""
    rng = np.random.default_rng(seed)
    P = int(rng.integers(9, 60))
    Nc, Ng = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    a = rng.integers(-3, 4, size=P).tolist()
    K, V, Q, bt, sl, g = _one_hot_problem(a, Nc, Ng)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    # means of <= 4 small integers with denominators 3 are not dyadic; keep the exact cases only
    rho = [int(x) for x in rng.choice([2500, 3300, 5000, 7500, 10000], 3)]
    plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=0, window_pages=0, rho_g_bp=rho[0], rho_c_bp=rho[1], rho_p_bp=rho[2])
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, P)
    if Nc in (1, 2, 4) and Ng in (1, 2, 4) and P % Nc == 0 and (P // Nc) % Ng == 0:
        assert ids[0, 0, :nsel[0, 0]].tolist() == _exact_cascade(a, Nc, Ng, "ratio", rho=rho)
    k = int(rng.integers(1, P))
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, oracle.Plan(plan=oracle.PLAN_FLAT, sink_pages=0, window_pages=0,
                                                                 budget_pages=k), P)
    assert ids[0, 0, :nsel[0, 0]].tolist() == _exact_cascade(a, Nc, Ng, "flat", k=k)


# ------------------------------------------------------------------ Alg. 1 stage 2 as printed: S >= tau keeps every tie
@pytest.mark.parametrize("seed", range(8))
def test_threshold_rule_matches_exact_bruteforce_with_many_ties(seed):
    """Small integer scores, so every level has ties at its cut: under the threshold rule all of them survive, and
    the next level counts its active units from that larger set.  Exact rational brute force (dyadic cases)."""
    rng = np.random.default_rng(100 + seed)
    Nc, Ng = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4]))
    P = Nc * Ng * int(rng.integers(2, 9))
    a = rng.integers(-2, 3, size=P).tolist()
    K, V, Q, bt, sl, g = _one_hot_problem(a, Nc, Ng)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    rho = [int(x) for x in rng.choice([2500, 3300, 5000, 7500], 3)]
    plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=0, window_pages=0, rho_g_bp=rho[0], rho_c_bp=rho[1],
                       rho_p_bp=rho[2], cut_rule=oracle.CUT_THRESHOLD)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, P)
    want = _exact_cascade(a, Nc, Ng, "ratio", rho=rho, threshold=True)
    assert ids[0, 0, :nsel[0, 0]].tolist() == want
    exact_count = _exact_cascade(a, Nc, Ng, "ratio", rho=rho)
    assert len(want) >= len(exact_count)
    k = int(rng.integers(1, P))
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, oracle.Plan(plan=oracle.PLAN_FLAT, sink_pages=0, window_pages=0,
                                                                 budget_pages=k, cut_rule=oracle.CUT_THRESHOLD), P)
    want = _exact_cascade(a, Nc, Ng, "flat", k=k, threshold=True)
    assert ids[0, 0, :nsel[0, 0]].tolist() == want and len(want) >= k
    kth = sorted(a, reverse=True)[k - 1]
    assert want == [i for i in range(P) if a[i] >= kth]


def test_threshold_rule_special_cases(ragged):
    """No ties (continuous scores): the threshold rule keeps exactly the count rule's units.  All keys identical:
    every level's units all tie at tau, so every candidate page survives (the list is every page).  Negative
    scores: tau is taken over the active units only (an inactive unit is never ranked, not even as a zero)."""
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    for kw in (dict(), dict(plan=oracle.PLAN_RATIO, rho_g_bp=6000, rho_c_bp=5000, rho_p_bp=2000)):
        a = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp, **kw), sp.max_pages, detail=True)
        b = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp, cut_rule=oracle.CUT_THRESHOLD, **kw), sp.max_pages, detail=True)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
    # identical keys
    L, d, B = 48 * 4, 16, 4
    rng = np.random.default_rng(3)
    Klog = np.tile(rng.standard_normal((1, 1, d)).astype(np.float32), (L, 1, 1))
    K2, V2, bt2 = pack_pools(Klog, Klog, B)
    g2 = oracle.Geometry(1, 1, d, B, 2, 2, 48)
    Q2 = f32_to_bf16_bits(rng.standard_normal((1, 1, d)).astype(np.float32))
    sl2 = np.array([L], np.int32)
    s2 = oracle.summarize(K2, bt2, sl2, g2)
    plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=1, window_pages=2, rho_g_bp=3000, rho_c_bp=3000, rho_p_bp=3000,
                       cut_rule=oracle.CUT_THRESHOLD)
    ids, nsel, kg, kc, cnt = oracle.select(Q2, *s2, sl2, g2, plan, 48, detail=True)
    assert nsel[0, 0] == 48 and ids[0, 0].tolist() == list(range(48)) and cnt[0, 0].tolist() == [12, 24, 45]
    # negative scores (every page scores below zero; half of the grids are inactive at chunk level)
    a = [-5, -6, -1, -2, -9, -9, -7, -8]
    K3, V3, Q3, bt3, sl3, g3 = _one_hot_problem(a, 2, 2)
    s3 = oracle.summarize(K3, bt3, sl3, g3)
    plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=0, window_pages=0, rho_g_bp=5000, rho_c_bp=5000, rho_p_bp=5000,
                       cut_rule=oracle.CUT_THRESHOLD)
    ids, nsel = oracle.select(Q3, *s3, sl3, g3, plan, 8)
    assert ids[0, 0, :nsel[0, 0]].tolist() == [2]          # grid 0 (mean -3.5) -> chunk 1 (-1.5) -> page 2 (-1)


# ------------------------------------------------------------------ per-sequence budgets
def test_per_sequence_budgets(ragged):
    """budget_per_seq[b] > 0 is sequence b's page budget k; an entry <= 0 falls back to the plan's own budget.
    Flat plan: brute-force top-k_b per sequence (numpy); budget plan: the same lists as one call per sequence with
    that fixed budget."""
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    per = (7, 0, 3)
    s, w = sp.sink_pages, sp.window_pages
    ps, _, _ = oracle.scores(Q, pv, cv, gv, sl, g)
    flat = plan_of(sp, plan=oracle.PLAN_FLAT, budget_per_seq=per)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, flat, sp.max_pages)
    for b in range(sp.batch):
        P = -(-int(sl[b]) // sp.page_size)
        k = per[b] if per[b] > 0 else max(1, -(-P * sp.budget_bp // 10000))
        for h in range(sp.n_kv_heads):
            cand = np.arange(s, P - w)
            top = cand[np.argsort(-ps[b, h, cand], kind="stable")][:k]
            assert ids[b, h, :nsel[b, h]].tolist() == list(range(s)) + sorted(top.tolist()) + list(range(P - w, P))
    both = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp, budget_per_seq=per), sp.max_pages, detail=True)
    for b in range(sp.batch):
        one = oracle.select(Q[b:b + 1], pv[b:b + 1], cv[b:b + 1], gv[b:b + 1], sl[b:b + 1], g,
                            plan_of(sp, budget_pages=max(per[b], 0)), sp.max_pages, detail=True)
        assert all(np.array_equal(x[b:b + 1], y) for x, y in zip(both, one))
    # the model-wide scope takes the same per-sequence budgets
    probes = [oracle.anchor(pv, sl, g, w)]
    sids, sn, scnt = oracle.select_shared(probes, [pv], [cv], [gv], sl, g, plan_of(sp, budget_per_seq=per), sp.max_pages, detail=True)
    for b in range(sp.batch):
        P = -(-int(sl[b]) // sp.page_size)
        k = per[b] if per[b] > 0 else max(1, -(-P * sp.budget_bp // 10000))
        assert sn[b] == s + w + min(k, scnt[b, 2]) and scnt[b, 2] <= k


# ------------------------------------------------------------------ P7: Table 1 budgets
def test_ratio_plan_reproduces_table1_budgets():
    P, Nc, Ng = 6400, 8, 8
    rng = np.random.default_rng(3)
    Klog = rng.standard_normal((P, 1, 8)).astype(np.float32)
    K, V, bt = pack_pools(Klog, Klog, 1)
    g = oracle.Geometry(1, 1, 8, 1, Nc, Ng, P)
    Q = f32_to_bf16_bits(rng.standard_normal((1, 1, 8)).astype(np.float32))
    sl = np.array([P], np.int32)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    for line in open(os.path.join(GOLDEN, "table1_budgets.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        name, rg, rc, rp, printed = line[0], float(line[1]), float(line[2]), float(line[3]), int(line[4])
        plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=0, window_pages=0, rho_g_bp=round(rg * 1e4),
                           rho_c_bp=round(rc * 1e4), rho_p_bp=round(rp * 1e4))
        ids, nsel, kg, kc, cnt = oracle.select(Q, pv, cv, gv, sl, g, plan, P, detail=True)
        share = 100.0 * nsel[0, 0] / P
        assert abs(share - printed) < 1.0, (name, share)            # as printed (rounded to a percent)
        assert abs(share - 100 * rg * rc * rp) < 0.02, (name, share)  # the product of the ratios
        assert cnt[0, 0].tolist() == [round(100 * rg), round(800 * rg * rc), nsel[0, 0]]


# ------------------------------------------------------------------ P5 / P6: invariants of the page list
@pytest.mark.parametrize("plan_kw", [
    dict(plan=oracle.PLAN_BUDGET), dict(plan=oracle.PLAN_BUDGET, budget_pages=9, over_chunk=2, over_grid=1),
    dict(plan=oracle.PLAN_RATIO, rho_g_bp=5000, rho_c_bp=2000, rho_p_bp=1000),
    dict(plan=oracle.PLAN_RATIO, rho_g_bp=8000, rho_c_bp=7000, rho_p_bp=7000), dict(plan=oracle.PLAN_FLAT)])
def test_page_list_invariants(ragged, plan_kw):
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    plan = plan_of(sp, **plan_kw)
    ids, nsel, kg, kc, cnt = oracle.select(Q, pv, cv, gv, sl, g, plan, sp.max_pages, detail=True)
    s, w, Nc, Ng = plan.sink_pages, plan.window_pages, sp.pages_per_chunk, sp.chunks_per_grid
    for b in range(sp.batch):
        P = -(-int(sl[b]) // sp.page_size)
        for h in range(sp.n_kv_heads):
            row = ids[b, h, :nsel[b, h]]
            assert (ids[b, h, nsel[b, h]:] == -1).all()
            assert (np.diff(row) > 0).all() and row[0] >= 0 and row[-1] < P
            assert set(range(s)) <= set(row) and set(range(P - w, P)) <= set(row)      # safety pages
            k_g, k_c, k_p = cnt[b, h]
            assert nsel[b, h] == s + k_p + w
            assert kg[b, h].sum() == k_g and kc[b, h].sum() == k_c
            for j in row:
                if s <= j < P - w:                                                     # containment
                    assert kc[b, h, j // Nc] and kg[b, h, j // Nc // Ng]
            for c in np.flatnonzero(kc[b, h]):
                assert kg[b, h, c // Ng]
            if plan.plan == oracle.PLAN_BUDGET:
                k = plan.budget_pages or max(1, -(-P * plan.budget_bp // 10000))
                t = -(-plan.over_chunk * k // Nc)
                assert k_g == min(-(-(-(-P // Nc)) // Ng), -(-plan.over_grid * t // Ng))
                assert k_c <= t and k_p <= k


def test_budget_plan_counts_at_benchmark_shapes():
    """Keep-counts of the budget plan: 1 % of 8192 pages with factors 10 / 5 is the Aggressive setting
    (0.5, 0.2, 0.1) of Table 1 up to ceilings: k=82, k_c=103 (10 % of chunks), k_g=65 (half the grids)."""
    P = 8192
    rng = np.random.default_rng(5)
    Klog = rng.standard_normal((P, 1, 4)).astype(np.float32)
    K, V, bt = pack_pools(Klog, Klog, 1)
    g = oracle.Geometry(1, 1, 4, 1, 8, 8, P)
    Q = f32_to_bf16_bits(rng.standard_normal((1, 1, 4)).astype(np.float32))
    sl = np.array([P], np.int32)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    plan = oracle.Plan(plan=oracle.PLAN_BUDGET, sink_pages=1, window_pages=4, budget_bp=100)
    ids, nsel, kg, kc, cnt = oracle.select(Q, pv, cv, gv, sl, g, plan, 128, detail=True)
    assert cnt[0, 0].tolist() == [65, 103, 82] and nsel[0, 0] == 87


def test_safety_pages_cover_short_sequences():
    sp = workload.WorkloadSpec("short", 4, (0, 96), 4, 2, 16, ("fixed", 32), (1, 1), 2, 3, budget_pages=2,
                               pages_per_chunk=2, chunks_per_grid=2)
    wl = workload.generate(sp, 5, seq_lens=[0, 1, 80, 96])
    K, V, Q, bt, sl = host_arrays(wl)
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp), 7)
    assert nsel[:, 0].tolist() == [0, 1, 5, 6]               # P = 0, 1, 5 (<= s+w), 6 (one candidate page)
    assert ids[2, 0, :5].tolist() == [0, 1, 2, 3, 4] and ids[3, 1, :6].tolist() == [0, 1, 2, 3, 4, 5]
    out = oracle.attend(Q, K, V, bt, sl, g, ids, nsel)
    assert not out[0].any() and np.isfinite(out).all()       # empty sequence -> zeros
    _, Vl = logical_kv(K, V, bt, 1, 1, 0)
    np.testing.assert_allclose(out[1, 0], Vl[0], atol=1e-7)  # one token -> its value row


# ------------------------------------------------------------------ P8: zero-copy / physical placement
def test_physical_placement_does_not_matter(ragged):
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    rng = np.random.default_rng(0)
    perm = rng.permutation(K.shape[0])                      # new home of every physical page
    K2, V2 = np.empty_like(K), np.empty_like(V)
    K2[perm], V2[perm] = K, V
    bt2 = np.where(bt >= 0, perm[np.maximum(bt, 0)], -1).astype(np.int32)
    a = oracle.summarize(K, bt, sl, g)
    b = oracle.summarize(K2, bt2, sl, g)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    ids, nsel = oracle.select(Q, *a, sl, g, plan_of(sp), sp.max_selected)
    assert np.array_equal(oracle.attend(Q, K, V, bt, sl, g, ids, nsel), oracle.attend(Q, K2, V2, bt2, sl, g, ids, nsel))


# ------------------------------------------------------------------ P10: all keys equal
def test_identical_keys_tie_to_lowest_indices_and_uniform_softmax():
    L, H, d, B = 40 * 4, 1, 16, 4
    rng = np.random.default_rng(1)
    Klog = np.tile(rng.standard_normal((1, H, d)).astype(np.float32), (L, 1, 1))
    Vlog = rng.standard_normal((L, H, d)).astype(np.float32)
    K, V, bt = pack_pools(Klog, Vlog, B, perm=rng.permutation(40))
    g = oracle.Geometry(2, 1, d, B, 2, 2, 40)
    Q = f32_to_bf16_bits(rng.standard_normal((1, 2, d)).astype(np.float32))
    sl = np.array([L], np.int32)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=1, window_pages=2, rho_g_bp=5000, rho_c_bp=5000, rho_p_bp=5000)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, 40)
    # 10 grids -> 5 lowest; 10 chunks -> 5 lowest (0..4); candidate pages 1..9 -> ceil(4.5)=5 lowest: 1..5
    assert ids[0, 0, :nsel[0, 0]].tolist() == [0, 1, 2, 3, 4, 5, 38, 39]
    out = oracle.attend(Q, K, V, bt, sl, g, ids, nsel)
    toks = listed_tokens(ids[0, 0], nsel[0, 0], L, B)
    Vbf = bf16_to_f64(f32_to_bf16_bits(Vlog))[:, 0]
    np.testing.assert_allclose(out[0, 0], Vbf[toks].mean(0), atol=1e-6)
    np.testing.assert_allclose(out[0, 1], Vbf[toks].mean(0), atol=1e-6)


# ------------------------------------------------------------------ P11: planted topic
def test_planted_topic_is_recovered():
    """Low noise, a one-topic query, budget = the segment's pages: the selection is exactly that segment."""
    sp = workload.WorkloadSpec("planted", 2, (4096, 4096), 4, 2, 16, ("fixed", 128), (1, 1), 1, 4, budget_pages=8,
                               noise_std=0.05)
    wl = workload.generate(sp, 11)
    K, V, Q, bt, sl = host_arrays(wl)
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp), sp.max_selected)
    for b in range(2):
        for h in range(2):
            topics = {wl.q_topics[b][hq][0] for hq in (2 * h, 2 * h + 1)}
            if len(topics) != 1:
                continue                                    # the group's two rows chose different topics
            seg = topics.pop()
            want = set(range(seg * 8, seg * 8 + 8)) - {0} - set(range(252, 256))
            got = set(ids[b, h, :nsel[b, h]].tolist()) - {0} - set(range(252, 256))
            assert want <= got


# ------------------------------------------------------------------ Eq. 3: the key-derived query anchor
def test_anchor_probe_is_the_mean_of_the_window_page_vectors(ragged):
    """Scores under the anchor probe against the definition written with numpy from the raw keys:
    anchor = mean over the last w pages of (mean of the page's key rows); S(u) = anchor . v_u.  With w = 1 the
    anchor is the tail page's vector, so S(tail page) = |v_tail|^2; sum_{p in W} S(p) / |W| = |anchor|^2 >= 0."""
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    B = sp.page_size
    for w in (1, 2, 5):
        plan = plan_of(sp, window_pages=w, probe=oracle.PROBE_ANCHOR)
        ps, cs, gs = oracle.scores(Q, pv, cv, gv, sl, g, plan)
        for b in range(sp.batch):
            L = int(sl[b]); P = -(-L // B); W = min(w, P)
            for h in range(sp.n_kv_heads):
                Kl, _ = logical_kv(K, V, bt, L, b, h)
                page_means = np.stack([Kl[j * B:min((j + 1) * B, L)].mean(0) for j in range(P)])
                anchor = page_means[P - W:].mean(0)
                np.testing.assert_allclose(ps[b, h, :P], page_means @ anchor, rtol=2e-6, atol=2e-6)
                np.testing.assert_allclose(ps[b, h, P - W:P].mean(), anchor @ anchor, rtol=2e-6, atol=2e-6)
                if w == 1:
                    np.testing.assert_allclose(ps[b, h, P - 1], page_means[P - 1] @ page_means[P - 1], rtol=2e-6)
                nc = -(-P // sp.pages_per_chunk)
                np.testing.assert_allclose(cs[b, h, :nc], cv[b, h, :nc].astype(np.float64) @ anchor, rtol=2e-6, atol=2e-6)


def test_anchor_selection_ignores_the_query_and_the_scale_of_the_keys(ragged):
    """Eq. 3-4 use keys only: another query gives the same pages; doubling every key multiplies all scores by 4
    and gives the same pages; and the list differs from the query probe's (so the switch is not a no-op)."""
    sp, wl, (K, V, Q, bt, sl) = ragged
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    plan = plan_of(sp, probe=oracle.PROBE_ANCHOR)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, sp.max_selected)
    Q2 = f32_to_bf16_bits(np.random.default_rng(5).standard_normal(Q.shape).astype(np.float32))
    ids2, nsel2 = oracle.select(Q2, pv, cv, gv, sl, g, plan, sp.max_selected)
    assert np.array_equal(ids, ids2) and np.array_equal(nsel, nsel2)
    ids3, nsel3 = oracle.select(Q, 2 * pv, 2 * cv, 2 * gv, sl, g, plan, sp.max_selected)
    assert np.array_equal(ids, ids3) and np.array_equal(nsel, nsel3)
    idq, _ = oracle.select(Q, pv, cv, gv, sl, g, plan_of(sp), sp.max_selected)
    assert not np.array_equal(ids, idq)
    # brute force under the flat plan: stable argsort of the anchor's page scores
    flat = plan_of(sp, plan=oracle.PLAN_FLAT, budget_pages=7, probe=oracle.PROBE_ANCHOR)
    idf, nf = oracle.select(Q, pv, cv, gv, sl, g, flat, sp.max_pages)
    ps, _, _ = oracle.scores(Q, pv, cv, gv, sl, g, flat)
    for b in range(sp.batch):
        P = -(-int(sl[b]) // sp.page_size)
        for h in range(sp.n_kv_heads):
            cand = np.arange(flat.sink_pages, P - flat.window_pages)
            order = cand[np.argsort(-ps[b, h, cand], kind="stable")][:7]
            want = sorted(set(range(flat.sink_pages)) | set(order.tolist()) | set(range(P - flat.window_pages, P)))
            assert idf[b, h, :nf[b, h]].tolist() == want


# ------------------------------------------------------------------ Eq. 1 Flatten: one page set for all layers and heads
@pytest.fixture(scope="module")
def layers():
    """Three 'layers' of the ragged workload: same lengths, independent keys and block tables."""
    sp = workload.WorkloadSpec("ragged", 3, (64, 3000), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_bp=300,
                               pages_per_chunk=4, chunks_per_grid=4)
    out = []
    for seed in (77, 78, 79):
        wl = workload.generate(sp, seed, seq_lens=[3000, 1237, 641])
        out.append(host_arrays(wl))
    return sp, out


def test_anchor_output_is_the_mean_of_the_window_page_means(layers):
    """oracle.anchor against Eq. 3 written with numpy from the raw keys."""
    sp, ls = layers
    g = geom_of(sp)
    K, V, Q, bt, sl = ls[0]
    pv, _, _ = oracle.summarize(K, bt, sl, g)
    B = sp.page_size
    for w in (1, 3, 400):
        a = oracle.anchor(pv, sl, g, w)
        for b in range(sp.batch):
            L = int(sl[b]); P = -(-L // B); W = min(w, P)
            for h in range(sp.n_kv_heads):
                Kl, _ = logical_kv(K, V, bt, L, b, h)
                means = np.stack([Kl[j * B:min((j + 1) * B, L)].mean(0) for j in range(P - W, P)])
                np.testing.assert_allclose(a[b, h], means.mean(0), rtol=3e-6, atol=3e-6)


def test_shared_scope_scores_the_flattened_vectors(layers):
    """Eq. 1 concatenates the per-layer, per-head page means into one vector per page, Eq. 3 averages those over
    the window and Eq. 4 is their dot product.  Built here with numpy from the raw keys (one long vector per page),
    stable argsort, first k: the flat plan of the shared scope must return exactly these pages."""
    sp, ls = layers
    g = geom_of(sp)
    B, s, w, k = sp.page_size, sp.sink_pages, sp.window_pages, 9
    summ = [oracle.summarize(K, bt, sl, g) for (K, V, Q, bt, sl) in ls]
    sl = ls[0][4]
    probes = [oracle.anchor(pv, sl, g, w) for (pv, cv, gv) in summ]
    plan = plan_of(sp, plan=oracle.PLAN_FLAT, budget_pages=k)
    ids, nsel = oracle.select_shared(probes, [x[0] for x in summ], [x[1] for x in summ], [x[2] for x in summ], sl, g,
                                     plan, s + w + k)
    for b in range(sp.batch):
        L = int(sl[b]); P = -(-L // B)
        flat = []
        for (K, V, Q, bt, _) in ls:
            for h in range(sp.n_kv_heads):
                Kl, _ = logical_kv(K, V, bt, L, b, h)
                flat.append(np.stack([Kl[j * B:min((j + 1) * B, L)].mean(0) for j in range(P)]))
        flat = np.concatenate(flat, axis=1)                   # [P, layers * heads * d]
        assert flat.shape == (P, 3 * sp.n_kv_heads * sp.head_dim)
        score = flat @ flat[P - w:].mean(0)
        cand = np.arange(s, P - w)
        order = cand[np.argsort(-score[cand], kind="stable")]
        gap = score[order[k - 1]] - score[order[k]]
        assert gap > 1e-4, "seed gives a near-tie at the cut; pick another"
        want = sorted(list(range(s)) + order[:k].tolist() + list(range(P - w, P)))
        assert nsel[b] == s + k + w and ids[b, :nsel[b]].tolist() == want
    # and it is not what any single layer would pick
    one, _ = oracle.select_shared(probes[:1], [summ[0][0]], [summ[0][1]], [summ[0][2]], sl, g, plan, s + w + k)
    assert not np.array_equal(one, ids)


def test_shared_scope_of_one_layer_and_one_head_is_the_per_head_cascade():
    """With a single layer and a single KV head the flattened vector is that head's vector: the shared cascade
    (all three levels, budget and ratio plans) must return the per-head cascade's list."""
    sp = workload.WorkloadSpec("onehead", 2, (64, 4000), 4, 1, 16, ("fixed", 128), (2, 2), 1, 3, budget_bp=200,
                               pages_per_chunk=4, chunks_per_grid=4)
    wl = workload.generate(sp, 5, seq_lens=[4000, 1733])
    K, V, Q, bt, sl = host_arrays(wl)
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    for kw in (dict(), dict(plan=oracle.PLAN_RATIO, rho_g_bp=5000, rho_c_bp=4000, rho_p_bp=3000)):
        plan = plan_of(sp, probe=oracle.PROBE_ANCHOR, **kw)
        ids, nsel, _, _, cnt = oracle.select(Q, pv, cv, gv, sl, g, plan, sp.max_pages, detail=True)
        probe = oracle.anchor(pv, sl, g, plan.window_pages)
        ids_s, nsel_s, cnt_s = oracle.select_shared([probe], [pv], [cv], [gv], sl, g, plan, sp.max_pages, detail=True)
        assert np.array_equal(ids[:, 0], ids_s) and np.array_equal(nsel[:, 0], nsel_s)
        assert np.array_equal(cnt[:, 0], cnt_s)
        if kw:
            assert (cnt_s[:, 0] < -(-(-(-sl // 16) // 4) // 4)).all(), "the grid level must actually prune"


def test_shared_scope_is_linear_in_the_layers(layers):
    """The score is a sum over layers: listing every layer twice doubles all scores (same pages), a layer whose
    probe is zero changes nothing, and the order of the layers does not matter beyond rounding."""
    sp, ls = layers
    g = geom_of(sp)
    summ = [oracle.summarize(K, bt, sl, g) for (K, V, Q, bt, sl) in ls]
    sl = ls[0][4]
    plan = plan_of(sp)
    probes = [oracle.anchor(x[0], sl, g, plan.window_pages) for x in summ]
    cols = lambda idx: ([probes[i] for i in idx], [summ[i][0] for i in idx], [summ[i][1] for i in idx], [summ[i][2] for i in idx])
    base = oracle.select_shared(*cols([0, 1, 2]), sl, g, plan, sp.max_selected, detail=True)
    twice = oracle.select_shared(*cols([0, 1, 2, 0, 1, 2]), sl, g, plan, sp.max_selected, detail=True)
    swapped = oracle.select_shared(*cols([2, 0, 1]), sl, g, plan, sp.max_selected, detail=True)
    for other in (twice, swapped):
        assert all(np.array_equal(a, b) for a, b in zip(base, other))
    pr, pg, ch, gr = cols([0, 1, 2])
    muted = oracle.select_shared(pr[:2] + [np.zeros_like(pr[2])], pg, ch, gr, sl, g, plan, sp.max_selected, detail=True)
    two = oracle.select_shared(*cols([0, 1]), sl, g, plan, sp.max_selected, detail=True)
    assert all(np.array_equal(a, b) for a, b in zip(muted, two))
    assert not np.array_equal(two[0], base[0])
    # list invariants: safety pages present, ascending, counts as the plan's integer formulas say
    ids, nsel, cnt = base
    for b in range(sp.batch):
        P = -(-int(sl[b]) // sp.page_size)
        row = ids[b, :nsel[b]].tolist()
        assert row == sorted(set(row)) and set(range(plan.sink_pages)) <= set(row)
        assert set(range(P - plan.window_pages, P)) <= set(row) and (ids[b, nsel[b]:] == -1).all()
        k = max(1, -(-P * plan.budget_bp // 10000))
        assert nsel[b] == plan.sink_pages + plan.window_pages + min(k, cnt[b, 2]) and cnt[b, 2] <= k


def test_shared_scope_never_draws_safety_pages_from_the_budget():
    """Sec. 3.2 unites the sink and recent-window pages with the selection; they are not drawn from it.  Two cases
    in which a safety page WOULD take a budget slot if it were a candidate at page level:
    (1) every key row identical in both layers: all scores tie, ties go to the lowest index, so the kept pages are
        the lowest pages AFTER the sinks;
    (2) the sink pages and the window pages carry the anchor's own direction (planted), so they outscore every
        other page: the kept pages must still be the top k of the pages between them (brute force, numpy)."""
    L, H, d, B, Nc, Ng, s, w, k = 128 * 16, 2, 128, 16, 4, 4, 2, 3, 6
    P = L // B
    g = oracle.Geometry(4, H, d, B, Nc, Ng, P)
    sl = np.array([L], np.int32)
    rng = np.random.default_rng(20732)

    def layer(Klog):
        K, _, bt = pack_pools(Klog, np.zeros_like(Klog), B, perm=rng.permutation(P))
        return oracle.summarize(K, bt, sl, g)

    def run(summ, plan):
        probes = [oracle.anchor(pv, sl, g, w) for (pv, cv, gv) in summ]
        return probes, oracle.select_shared(probes, [x[0] for x in summ], [x[1] for x in summ], [x[2] for x in summ],
                                            sl, g, plan, s + k + w)

    # (1) exact ties at every level
    row = np.linspace(-1, 1, d, dtype=np.float32)
    summ = [layer(np.tile(row, (L, H, 1))) for _ in range(2)]
    for kw in (dict(plan=oracle.PLAN_BUDGET), dict(plan=oracle.PLAN_FLAT)):
        _, (ids, nsel) = run(summ, oracle.Plan(sink_pages=s, window_pages=w, budget_pages=k, **kw))
        assert ids[0, :nsel[0]].tolist() == list(range(s)) + list(range(s, s + k)) + list(range(P - w, P))

    # (2) planted: sinks and window along one direction t, everything else small noise
    t = rng.standard_normal((H, d)).astype(np.float32)
    summ = []
    for _ in range(2):
        Klog = 0.05 * rng.standard_normal((L, H, d)).astype(np.float32)
        Klog[:s * B] += t
        Klog[(P - w) * B:] += t
        summ.append(layer(Klog))
    plan = oracle.Plan(plan=oracle.PLAN_FLAT, sink_pages=s, window_pages=w, budget_pages=k)
    probes, (ids, nsel) = run(summ, plan)
    flat = np.concatenate([pv[0].astype(np.float64).transpose(1, 0, 2).reshape(P, H * d) for (pv, _, _) in summ], axis=1)
    probe = np.concatenate([p[0].astype(np.float64).reshape(H * d) for p in probes])
    score = flat @ probe
    assert score[:s].min() > score[s:P - w].max() and score[P - w:].min() > score[s:P - w].max(), "the plant must dominate"
    cand = np.arange(s, P - w)
    top = cand[np.argsort(-score[cand], kind="stable")][:k]
    assert nsel[0] == s + k + w
    assert ids[0, :nsel[0]].tolist() == list(range(s)) + sorted(top.tolist()) + list(range(P - w, P))
    # the per-head cascade on the same plant (one layer, anchor probe): the same rule
    pv, cv, gv = summ[0]
    Q = np.zeros((1, 4, d), np.uint16)
    hplan = oracle.Plan(plan=oracle.PLAN_FLAT, sink_pages=s, window_pages=w, budget_pages=k, probe=oracle.PROBE_ANCHOR)
    hid, hn = oracle.select(Q, pv, cv, gv, sl, g, hplan, s + k + w)
    a = oracle.anchor(pv, sl, g, w)
    for h in range(H):
        sc = pv[0, h].astype(np.float64) @ a[0, h].astype(np.float64)
        top = cand[np.argsort(-sc[cand], kind="stable")][:k]
        assert hid[0, h, :hn[0, h]].tolist() == list(range(s)) + sorted(top.tolist()) + list(range(P - w, P))


# ------------------------------------------------------------------ Sec. 3.3: entropy / variance of the entropy per page
def test_entropy_closed_forms_and_library_routine():
    """Uniform logits: log V.  One logit far above the rest: ~0.  Two levels: the closed form
    H = log Z - (a e^a n_a + b e^b n_b) / Z.  Random rows: scipy's entropy of scipy's softmax.  Adding a constant to a
    row changes nothing; 0 <= H <= log V."""
    from scipy.special import softmax
    from scipy.stats import entropy as sp_entropy
    V = 1000
    rows = np.zeros((5, V), np.float32)
    rows[1, 7] = 100.0
    rows[2, :250] = 2.0                                   # two levels: 250 logits at 2, 750 at 0
    rng = np.random.default_rng(0)
    rows[3] = rng.standard_normal(V) * 3
    rows[4] = -rows[3]
    bits = f32_to_bf16_bits(rows)
    H = oracle.entropy(bits)
    z = bf16_to_f64(bits)
    assert abs(H[0] - np.log(V)) < 1e-12
    assert 0 <= H[1] < 1e-38
    Z = 250 * np.exp(2.0) + 750
    assert abs(H[2] - (np.log(Z) - 2.0 * 250 * np.exp(2.0) / Z)) < 1e-12
    for r in (3, 4):
        assert abs(H[r] - sp_entropy(softmax(z[r]))) < 1e-10
    half = np.round(rng.uniform(-4, 4, V) * 2) / 2          # half-integers: they and their shift by 8 are exact in bf16
    pair = f32_to_bf16_bits(np.stack([half, half + 8.0]).astype(np.float32))
    assert np.array_equal(bf16_to_f64(pair[1]) - 8.0, bf16_to_f64(pair[0]))
    Hs = oracle.entropy(pair)
    assert abs(Hs[0] - Hs[1]) < 1e-12, "softmax is shift invariant"
    assert (H >= 0).all() and (H <= np.log(V) + 1e-12).all()
    # only the first `vocab` entries of a row count
    wide = np.concatenate([bits[3:4], f32_to_bf16_bits(np.full((1, 24), 50.0, np.float32))], axis=1)
    assert abs(oracle.entropy(wide, vocab=V)[0] - H[3]) == 0


def test_page_trigger_is_mean_and_population_variance_with_an_or_rule():
    rng = np.random.default_rng(1)
    H = rng.uniform(0.5, 3.0, 16).astype(np.float32)
    mean, var, fire = oracle.page_trigger(H, 10.0, 10.0)
    assert abs(mean - H.astype(np.float64).mean()) < 1e-12 and abs(var - H.astype(np.float64).var()) < 1e-12 and not fire
    assert oracle.page_trigger(H, mean - 1e-6, 10.0)[2] and oracle.page_trigger(H, 10.0, var - 1e-6)[2]
    assert not oracle.page_trigger(H, mean + 1e-6, var + 1e-6)[2]
    const = np.full(16, 2.5, np.float32)
    assert oracle.page_trigger(const, 2.4, 0.0)[:2] == (2.5, 0.0)
    assert not oracle.page_trigger(const, 2.5, 0.0)[2], "strictly above, not at, the threshold"
    assert oracle.page_trigger(np.array([1.0, 3.0], np.float32), 5.0, 0.5)[:2] == (2.0, 1.0)


# ------------------------------------------------------------------ P12: degenerate hierarchy
def test_one_token_pages_give_token_level_topk_attention():
    rng = np.random.default_rng(4)
    L, d = 50, 8
    Klog = rng.standard_normal((L, 1, d)).astype(np.float32)
    Vlog = rng.standard_normal((L, 1, d)).astype(np.float32)
    K, V, bt = pack_pools(Klog, Vlog, 1, perm=rng.permutation(L))
    g = oracle.Geometry(1, 1, d, 1, 1, 1, L)
    qf = rng.standard_normal((1, 1, d)).astype(np.float32)
    Q = f32_to_bf16_bits(qf)
    sl = np.array([L], np.int32)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    np.testing.assert_array_equal(pv[0, 0], bf16_to_f64(f32_to_bf16_bits(Klog))[:, 0].astype(np.float32))
    np.testing.assert_array_equal(cv, pv)
    np.testing.assert_array_equal(gv, pv)
    tok = bf16_to_f64(f32_to_bf16_bits(Klog))[:, 0] @ bf16_to_f64(Q)[0, 0]
    for k in (1, 5):
        plan = oracle.Plan(plan=oracle.PLAN_BUDGET, sink_pages=0, window_pages=0, budget_pages=k, over_chunk=L, over_grid=L)
        ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, k)
        assert ids[0, 0].tolist() == sorted(np.argsort(-tok, kind="stable")[:k].tolist())
    out = oracle.attend(Q, K, V, bt, sl, g, ids[:, :, :1] * 0 + int(np.argmax(tok)), np.ones((1, 1), np.int32))
    np.testing.assert_array_equal(out[0, 0], bf16_to_f64(f32_to_bf16_bits(Vlog))[int(np.argmax(tok)), 0].astype(np.float32))


def test_negative_scores_are_not_outranked_by_inactive_units():
    """All scores negative: zero-filling inactive units (Alg. 1 as printed) would rank them first; the
    cascade must still return children of kept parents only."""
    a = [-5, -6, -1, -2, -9, -9, -3, -4]
    K, V, Q, bt, sl, g = _one_hot_problem(a, 2, 2)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    plan = oracle.Plan(plan=oracle.PLAN_RATIO, sink_pages=0, window_pages=0, rho_g_bp=5000, rho_c_bp=5000, rho_p_bp=5000)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, 8)
    # grids: (-5.5-1.5)/2=-3.5, (-9-3.5)/2=-6.25 -> grid 0; chunks -5.5, -1.5 -> chunk 1; pages -1,-2 -> page 2
    assert ids[0, 0, :nsel[0, 0]].tolist() == [2]


def test_generator_recipe_statistics():
    """The workload module follows the stated recipe: unit-variance topics, noise std 0.5, unit values."""
    sp = workload.spec("cfg1")
    wl = workload.generate(sp, 123)
    K, V, Q, bt, sl = host_arrays(wl)
    Kl, Vl = logical_kv(K, V, bt, sl[0], 0, 0)
    assert abs(Vl.std() - 1.0) < 0.02 and abs(Vl.mean()) < 0.02
    seg = Kl.reshape(32, 128, 128)
    assert abs((seg - seg.mean(1, keepdims=True)).std() - 0.5) < 0.02
    assert abs(seg.mean(1).std() - 1.0) < 0.05
    assert np.isnan(bf16_to_f64(K[bt.max() + 1:])).all() or K.shape[0] == bt.max() + 1
