"""chess_sparse_decode_static: the allocation-free variant of chess_sparse_decode (its split partials and arrival
counters live in a device array the library owns).  Called through the C ABI, checked bit for bit against
chess_sparse_decode on the same lists, and against the oracle, on calls in a row that share the one array:
a batch, then a smaller batch with shorter lists, then another context with another geometry."""
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
SUMMARY_DTYPE_SWEEP = False       # nothing here reads or writes summary vectors


def _lists(lib, d, plan, batch, sp):
    summ, ws = lib.new_summaries(), lib.new_workspace()
    ids = torch.full((batch, sp.n_kv_heads, lib.cfg.max_selected_pages), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((batch, sp.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
    lib.select(d.q, summ, d.seq_lens, gpu_plan(plan), ids, nsel, ws)
    return ids, nsel, ws


def _both(lib, d, ids, nsel, ws, sp):
    batch = d.seq_lens.shape[0]
    a = torch.full((batch, sp.n_q_heads, 128), float("nan"), device="cuda")
    b = torch.full_like(a, float("nan"))
    lib.sparse_decode(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, ids, nsel, a, ws)
    lib.sparse_decode_static(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, ids, nsel, b)
    torch.cuda.synchronize()
    return a, b


def test_static_scratch_variant_equals_sparse_decode():
    sp = workload.WorkloadSpec("ragged", 5, (0, 3000), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_bp=900,
                               pages_per_chunk=4, chunks_per_grid=4)
    lens = [3000, 1237, 641, 16, 0]
    wl = workload.generate(sp, 81, seq_lens=lens)
    d = to_device(wl)
    lib = pk.Chess(config_of(sp, max_selected=sp.max_pages))
    plan = plan_of(sp)
    ids, nsel, ws = _lists(lib, d, plan, sp.batch, sp)
    for forced in (0, 7):                                            # the automatic split shape, and several splits per row
        lib.debug_force_splits(forced)
        a, b = _both(lib, d, ids, nsel, ws, sp)
        assert torch.equal(a, b), "first call"
        K, V, Q, bt, sl = host_arrays(wl)
        ref = oracle.attend(Q, K, V, bt, sl, geom_of(sp), ids.cpu().numpy(), nsel.cpu().numpy())
        assert np.abs(b.cpu().numpy() - ref).max() <= 1e-2

        # second call, smaller: two of the sequences, lists cut to a third
        sub = [1, 2]
        d2 = workload.Workload(sp, wl.seed, wl.layer, d.k_pool, d.v_pool, d.block_table[sub].contiguous(),
                               d.seq_lens[sub].contiguous(), d.q[sub].contiguous(), wl.segments, wl.q_topics)
        ids2 = ids[sub].contiguous()
        nsel2 = (nsel[sub] // 3).clamp_(min=1).contiguous()
        a2, b2 = _both(lib, d2, ids2, nsel2, ws, sp)
        assert torch.equal(a2, b2), "second, smaller call"
        ref2 = oracle.attend(Q[sub], K, V, bt[sub], sl[sub], geom_of(sp), ids2.cpu().numpy(), nsel2.cpu().numpy())
        assert np.abs(b2.cpu().numpy() - ref2).max() <= 1e-2

    # another context, another geometry (group of 7, 32-token pages), on the same device array
    sp3 = workload.spec("cfg5", scale=1 / 16)
    wl3 = workload.generate(sp3, workload.default_seed("cfg5"))
    d3 = to_device(wl3)
    lib3 = pk.Chess(config_of(sp3))
    ids3, nsel3, ws3 = _lists(lib3, d3, plan_of(sp3), sp3.batch, sp3)
    a3, b3 = _both(lib3, d3, ids3, nsel3, ws3, sp3)
    assert torch.equal(a3, b3), "other context"
    # and the first context again, after the other one used the array
    lib.debug_force_splits(0)
    a, b = _both(lib, d, ids, nsel, ws, sp)
    assert torch.equal(a, b), "first context after the other one"
    lib.close()
    lib3.close()


def test_static_scratch_variant_in_a_hip_graph():
    """The call allocates nothing and clears its counters with a fill kernel (not a memset node), so it can be captured:
    every replay of the graph, with eager calls of the workspace variant and synchronisations in between and a different
    query each time, gives the eager result bit for bit."""
    sp = workload.spec("cfg2", scale=1 / 4)
    wl = to_device(workload.generate(sp, workload.default_seed("cfg2")))
    lib = pk.Chess(config_of(sp))
    ids, nsel, ws = _lists(lib, wl, plan_of(sp), sp.batch, sp)
    qs = [wl.q] + [workload.extra_queries(wl, v) for v in range(1, 4)]
    eager = []
    for q in qs:
        out = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
        lib.sparse_decode(q, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, ids, nsel, out, ws)
        torch.cuda.synchronize()
        eager.append(out.clone())
    q_in = torch.empty_like(wl.q)
    out_g = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        q_in.copy_(qs[0])
        lib.sparse_decode_static(q_in, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, ids, nsel, out_g)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            lib.sparse_decode_static(q_in, wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, ids, nsel, out_g)
        for rep in range(6):
            i = rep % len(qs)
            q_in.copy_(qs[i])
            out_g.fill_(float("nan"))
            graph.replay()
            stream.synchronize()
            assert torch.equal(out_g, eager[i]), f"replay {rep}"
            scratch = torch.full((1, sp.n_q_heads, 128), float("nan"), device="cuda")      # eager work between the replays
            lib.sparse_decode(qs[(i + 1) % len(qs)], wl.k_pool, wl.v_pool, wl.block_table, wl.seq_lens, ids, nsel, scratch, ws)
            stream.synchronize()
    lib.close()


def test_static_scratch_variant_rejects_what_does_not_fit():
    """A shape whose partials exceed the array (16 query heads per KV head, 8 rows, 64 splits forced: 4.26 MB) is
    refused with CHESS_ESCRATCH before anything is launched; so are null pointers (CHESS_EINVAL)."""
    lib = pk.Chess(pk.Config(n_q_heads=16, n_kv_heads=1, page_size=16, max_batch=8, max_pages_per_seq=256,
                             max_selected_pages=64))
    z = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    sl = torch.zeros(8, dtype=torch.int32, device="cuda")
    lib.debug_force_splits(64)
    with pytest.raises(pk.ChessError, match="-5"):
        lib.sparse_decode_static(z, z, z, z, sl, z, z, z)
    with pytest.raises(pk.ChessError, match="-1"):
        lib.sparse_decode_static(None, z, z, z, sl, z, z, z)
    lib.debug_force_splits(0)
    out = torch.full((8, 16, 128), float("nan"), device="cuda")
    lib.sparse_decode_static(z, z, z, z, sl, z, z, out)          # empty sequences: defined, zero output
    torch.cuda.synchronize()
    assert not out.any()
    lib.close()
