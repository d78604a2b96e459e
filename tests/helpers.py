"""Test-side utilities: independent unpacking of the paged pools into logical rows, small hand-built
inputs, and the bookkeeping shared by the oracle pins and the GPU parity tests.  None of this is used by
the product path."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import workload


SUMMARY_DTYPE = 0     # storage type of the summaries in the running test (0 = fp32, 1 = bf16); tests/conftest.py sets it


def geom_of(sp: workload.WorkloadSpec, max_pages=None, summary_dtype=None) -> oracle.Geometry:
    return oracle.Geometry(sp.n_q_heads, sp.n_kv_heads, sp.head_dim, sp.page_size, sp.pages_per_chunk,
                           sp.chunks_per_grid, sp.max_pages if max_pages is None else max_pages,
                           SUMMARY_DTYPE if summary_dtype is None else summary_dtype)


def plan_of(sp: workload.WorkloadSpec, **kw) -> oracle.Plan:
    base = dict(sink_pages=sp.sink_pages, window_pages=sp.window_pages, budget_pages=sp.budget_pages,
                budget_bp=sp.budget_bp)
    base.update(kw)
    return oracle.Plan(**base)


def host_arrays(wl: workload.Workload):
    """(K bits, V bits, Q bits, block table, seq lens) as numpy arrays for the oracle."""
    return (workload.bf16_bits(wl.k_pool), workload.bf16_bits(wl.v_pool), workload.bf16_bits(wl.q),
            wl.block_table.cpu().numpy(), wl.seq_lens.cpu().numpy())


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (via torch, independent of both implementations)."""
    return torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def logical_kv(K, V, bt, seq_len, b, h):
    """Rows of sequence b, KV head h in token order: (Kl [L,d], Vl [L,d]) as fp64.
    K pool is [phys][H][B][d], V pool is [phys][H][d][B]."""
    B = K.shape[2]
    L = int(seq_len)
    P = -(-L // B)
    phys = bt[b, :P]
    Kl = bf16_to_f64(K[phys, h]).reshape(P * B, -1)[:L]
    Vl = bf16_to_f64(V[phys, h]).transpose(0, 2, 1).reshape(P * B, -1)[:L]
    return Kl, Vl


def pack_pools(Klog: np.ndarray, Vlog: np.ndarray, B: int, perm=None):
    """Pack logical fp32 rows [L,H,d] of ONE sequence into pools; returns (K bits, V bits, block table [1,P]).
    Unused tail slots hold bf16 NaN."""
    L, H, d = Klog.shape
    P = -(-L // B)
    pad = P * B - L
    nanpad = np.full((pad, H, d), np.nan, np.float32)
    Kp = np.concatenate([Klog.astype(np.float32), nanpad]).reshape(P, B, H, d).transpose(0, 2, 1, 3)
    Vp = np.concatenate([Vlog.astype(np.float32), nanpad]).reshape(P, B, H, d).transpose(0, 2, 3, 1)
    if perm is None:
        perm = np.arange(P)
    perm = np.asarray(perm)
    Kpool = np.empty_like(Kp)
    Vpool = np.empty_like(Vp)
    Kpool[perm] = Kp
    Vpool[perm] = Vp
    return f32_to_bf16_bits(Kpool), f32_to_bf16_bits(Vpool), perm.astype(np.int32)[None, :]


def listed_tokens(ids_row, n, seq_len, B):
    """Token indices covered by the first n listed pages, in listed order."""
    toks = []
    for j in ids_row[:n]:
        toks.extend(range(int(j) * B, min(int(seq_len), (int(j) + 1) * B)))
    return np.asarray(toks, dtype=np.int64)


def softmax_attention(qrow: np.ndarray, Kl: np.ndarray, Vl: np.ndarray, scale: float) -> np.ndarray:
    """Textbook single-query attention with numpy's matmul (fp64)."""
    z = (Kl @ qrow) * scale
    p = np.exp(z - z.max())
    p /= p.sum()
    return p @ Vl
