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
from gpu_common import config_of, gpu_plan, to_device
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
            pv, cv, gv = (t[:3].cpu().numpy() for t in lib.summary_views(summ))
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
