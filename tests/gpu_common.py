"""Helpers of the GPU parity tests: run the HIP path through the Python binding (which only marshals
arguments for the C ABI) and the CPU oracle on the same seeded workload."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

import oracle
import paper_2602_20732_amd as pk
import workload
import helpers
from helpers import geom_of, host_arrays


def config_of(sp: workload.WorkloadSpec, max_selected=None, max_batch=None) -> pk.Config:
    return pk.Config(n_q_heads=sp.n_q_heads, n_kv_heads=sp.n_kv_heads, page_size=sp.page_size,
                     max_batch=sp.batch if max_batch is None else max_batch, max_pages_per_seq=sp.max_pages,
                     max_selected_pages=sp.max_selected if max_selected is None else max_selected,
                     pages_per_chunk=sp.pages_per_chunk, chunks_per_grid=sp.chunks_per_grid,
                     summary_dtype=helpers.SUMMARY_DTYPE)


def host_views(lib: pk.Chess, summaries, n=None):
    """The three summary arrays of a buffer as float32 numpy arrays (a bf16 value converts exactly)."""
    return tuple((t if n is None else t[:n]).float().cpu().numpy() for t in lib.summary_views(summaries))


def gpu_plan(op: oracle.Plan) -> pk.SelectPlan:
    kw = {f: getattr(op, f) for f in op.__dataclass_fields__}
    if kw["budget_per_seq"] is not None:                     # the library takes the per-sequence budgets from device memory
        kw["budget_per_seq"] = torch.as_tensor(list(kw["budget_per_seq"]), dtype=torch.int32, device="cuda")
    return pk.SelectPlan(**kw)


@dataclass
class GpuRun:
    pages: np.ndarray
    chunks: np.ndarray
    grids: np.ndarray
    ids: np.ndarray
    nsel: np.ndarray
    out: np.ndarray
    dense: np.ndarray
    step_ids: np.ndarray = None      # the same step through the single-launch entry point
    step_nsel: np.ndarray = None
    step_out: np.ndarray = None


def to_device(wl: workload.Workload):
    return wl if wl.k_pool.is_cuda else workload.Workload(
        wl.spec, wl.seed, wl.layer, wl.k_pool.cuda(), wl.v_pool.cuda(), wl.block_table.cuda(), wl.seq_lens.cuda(),
        wl.q.cuda(), wl.segments, wl.q_topics)


def run_gpu(lib: pk.Chess, wl: workload.Workload, plan: oracle.Plan, dense: bool = True, ids_override=None,
            cluster: int = 0) -> GpuRun:
    """summarize -> select -> sparse decode (+ dense decode) on the GPU; results as numpy arrays."""
    d = to_device(wl)
    c = lib.cfg
    batch = d.seq_lens.shape[0]
    summ = lib.new_summaries()
    ws = lib.new_workspace()
    ids = torch.full((batch, c.n_kv_heads, c.max_selected_pages), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((batch, c.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    out = torch.full((batch, c.n_q_heads, c.head_dim), float("nan"), dtype=torch.float32, device="cuda")
    dn = torch.full_like(out, float("nan"))
    lib.summarize(d.k_pool, d.block_table, d.seq_lens, summ)
    lib.debug_force_cluster(cluster)
    lib.select(d.q, summ, d.seq_lens, gpu_plan(plan), ids, nsel, ws)
    torch.cuda.synchronize()
    P = (-(-d.seq_lens.long() // c.page_size)).view(-1, 1, 1)            # the list must be safe to walk
    assert bool(((nsel >= 0) & (nsel <= c.max_selected_pages)).all()), "n_selected out of range"
    live = torch.arange(c.max_selected_pages, device="cuda").view(1, 1, -1) < nsel.unsqueeze(-1)
    assert bool((((ids >= 0) & (ids < P)) | ~live).all()), "page id out of range"
    if ids_override is not None:
        ids.copy_(torch.as_tensor(ids_override[0]).cuda())
        nsel.copy_(torch.as_tensor(ids_override[1]).cuda())
    lib.sparse_decode(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, ids, nsel, out, ws)
    if dense:
        lib.dense_decode(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, dn, ws)
    # the fused entry point: selection and attention in one launch, on a workspace of its own
    ws2 = lib.new_workspace()
    ids2 = torch.full_like(ids, -7)
    nsel2 = torch.full_like(nsel, -7)
    out2 = torch.full_like(out, float("nan"))
    lib.decode_step(d.q, d.k_pool, d.v_pool, d.block_table, d.seq_lens, summ, gpu_plan(plan), ids2, nsel2, out2, ws2)
    torch.cuda.synchronize()
    assert lib.workspace_error(ws) == 0 and lib.workspace_error(ws2) == 0, "a kernel gave up a bounded wait"
    pv, cv, gv = host_views(lib, summ, batch)
    return GpuRun(pv, cv, gv, ids.cpu().numpy(), nsel.cpu().numpy(), out.cpu().numpy(), dn.cpu().numpy(),
                  ids2.cpu().numpy(), nsel2.cpu().numpy(), out2.cpu().numpy())


@dataclass
class OracleRun:
    pages: np.ndarray
    chunks: np.ndarray
    grids: np.ndarray
    ids: np.ndarray
    nsel: np.ndarray
    out: np.ndarray
    dense: np.ndarray
    host: tuple


def run_oracle(wl: workload.Workload, plan: oracle.Plan, max_sel: int, dense: bool = True) -> OracleRun:
    sp = wl.spec
    K, V, Q, bt, sl = host = host_arrays(wl)
    g = geom_of(sp)
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    ids, nsel = oracle.select(Q, pv, cv, gv, sl, g, plan, max_sel)
    out = oracle.attend(Q, K, V, bt, sl, g, ids, nsel)
    dn = oracle.attend(Q, K, V, bt, sl, g) if dense else None
    return OracleRun(pv, cv, gv, ids, nsel, out, dn, host)


def assert_summaries_equal(gpu: GpuRun, ref: OracleRun, sp, seq_lens):
    """Bit-exact on every unit that exists (both sides add in the same order in fp64, round once)."""
    B, Nc, Ng = sp.page_size, sp.pages_per_chunk, sp.chunks_per_grid
    for b, L in enumerate(seq_lens):
        P = -(-int(L) // B); nc = -(-P // Nc); ng = -(-nc // Ng)
        assert np.array_equal(gpu.pages[b, :, :P].view(np.uint32), ref.pages[b, :, :P].view(np.uint32)), f"page vectors, seq {b}"
        assert np.array_equal(gpu.chunks[b, :, :nc].view(np.uint32), ref.chunks[b, :, :nc].view(np.uint32)), f"chunk vectors, seq {b}"
        assert np.array_equal(gpu.grids[b, :, :ng].view(np.uint32), ref.grids[b, :, :ng].view(np.uint32)), f"grid vectors, seq {b}"


def classify_selection(gpu_ids, gpu_n, ref: OracleRun, wl, plan: oracle.Plan):
    """Compare page lists row by row.  Returns (hard, near): rows whose sets differ, split into
    near-ties (every page in the symmetric difference has an fp64 score within 1e-5 * max(1, |cut|) of the
    oracle's cut score at page level) and hard mismatches."""
    sp = wl.spec
    K, V, Q, bt, sl = ref.host
    g = geom_of(sp)
    ps, cs, gs = oracle.scores(Q, ref.pages, ref.chunks, ref.grids, sl, g, plan)
    hard, near = [], []
    for b in range(gpu_ids.shape[0]):
        for h in range(gpu_ids.shape[1]):
            a = gpu_ids[b, h, :max(gpu_n[b, h], 0)].tolist()
            r = ref.ids[b, h, :ref.nsel[b, h]].tolist()
            if a == r and (gpu_ids[b, h, max(gpu_n[b, h], 0):] == -1).all():
                continue
            diff = set(a) ^ set(r)
            kept = [p for p in r if plan.sink_pages <= p < -(-int(sl[b]) // sp.page_size) - plan.window_pages]
            cut = min(ps[b, h, kept]) if kept else 0.0
            ok = bool(diff) and gpu_n[b, h] == ref.nsel[b, h] and all(
                0 <= p < ps.shape[2] and abs(ps[b, h, p] - cut) < 1e-5 * max(1.0, abs(cut)) for p in diff)
            (near if ok else hard).append((b, h, sorted(diff)))
    return hard, near


def host_subset(wl: workload.Workload, seqs):
    """Host arrays (K bits, V bits, Q bits, block table, seq lens) of the chosen sequences only, with their pages
    gathered into a compact pool (the oracle does not care where pages live)."""
    sp = wl.spec
    bt = wl.block_table.cpu().numpy()
    sl = wl.seq_lens.cpu().numpy()[list(seqs)]
    P = [-(-int(n) // sp.page_size) for n in sl]
    phys = np.concatenate([bt[b, :P[i]] for i, b in enumerate(seqs)]) if sum(P) else np.zeros(0, np.int64)
    idx = torch.as_tensor(phys, dtype=torch.long, device=wl.k_pool.device)
    K = workload.bf16_bits(wl.k_pool[idx])
    V = workload.bf16_bits(wl.v_pool[idx])
    Q = workload.bf16_bits(wl.q[list(seqs)])
    bt2 = np.full((len(seqs), sp.max_pages), -1, np.int32)
    off = 0
    for i in range(len(seqs)):
        bt2[i, :P[i]] = np.arange(off, off + P[i])
        off += P[i]
    return K, V, Q, bt2, sl.astype(np.int32)
