"""Seeded synthetic inputs for the CHESS decode hot path.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds none of the method's floating-point arithmetic: no
summaries, no scores, no selection, no attention -- only random numbers, the
topic-segment recipe of the benchmark configurations, and the packing of
logical K/V rows into the paged pool layout.  One integer formula of the
method is restated here, ``WorkloadSpec.budget_for`` (the page budget of a
sequence, k = max(1, ceil(P * bp / 10^4))): it sizes the ``page_ids`` rows a
configuration needs and serves as a length check in the tests and the
benchmark; neither the oracle nor the kernels call it.

Random numbers come from a stateless counter-based generator (a 64-bit
multiply-xorshift finaliser applied to ``key + counter``), written with integer
torch ops only, so the same (seed, index) gives the same bf16 value on the CPU
and on the GPU.  A standard normal is approximated by the centred sum of twelve
16-bit uniforms (Irwin-Hall), exact in fp32.

Pool layouts (one layer):
  K pool  bf16 [physical page][H_kv][B tokens][d]
  V pool  bf16 [physical page][H_kv][d][B tokens]      (token-minor inside a page)
  block table int32 [batch][max_pages]  logical page -> physical page, a seeded
  random permutation of the pool (never the identity), -1 past a sequence's pages
Unused pool pages and the unused slots of a partial tail page are filled with
bf16 NaN so that any read of them shows up in the result.

The paper's efficiency runs use "synthetic data of varying lengths" and give no
value distribution (Sec. 5, Sec. 5.3); the five shapes below are the benchmark
configurations this repository is measured on and stand in for that workload.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np
import torch

_MASK64 = (1 << 64) - 1
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_GOLD = 0x9E3779B97F4A7C15

STREAM_TOPIC, STREAM_KNOISE, STREAM_V, STREAM_QNOISE, STREAM_PICK, STREAM_SEG, STREAM_LEN, STREAM_PERM = range(8)


def _signed(x: int) -> int:
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def mix_int(x: int) -> int:
    """64-bit finaliser on a Python int (same function as ``_mix`` below)."""
    x &= _MASK64
    x ^= x >> 30
    x = (x * _C1) & _MASK64
    x ^= x >> 27
    x = (x * _C2) & _MASK64
    x ^= x >> 31
    return x


def stream_key(seed: int, stream: int, *coords: int) -> int:
    k = mix_int(seed * _GOLD + stream)
    for c in coords:
        k = mix_int(k ^ ((c + 1) * _GOLD))
    return k


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    x = x ^ _lsr(x, 30)
    x = x * _signed(_C1)
    x = x ^ _lsr(x, 27)
    x = x * _signed(_C2)
    x = x ^ _lsr(x, 31)
    return x


def normal_from_counter(key: int, idx: torch.Tensor) -> torch.Tensor:
    """Approximate N(0,1) for int64 counters ``idx`` under ``key``; fp32, multiples of 2^-16."""
    acc = torch.zeros_like(idx)
    base = idx * 3 + _signed(key)
    for r in range(3):
        h = _mix((base + r) * _signed(_GOLD))
        acc += (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)
    return (acc - 393210).to(torch.float32) * (1.0 / 65536.0)


def uniform_int(key: int, counter: int, n: int) -> int:
    """Integer in [0, n) from (key, counter), Python-side."""
    return mix_int((key + counter * 3) * _GOLD) % n


def uniform_unit(key: int, counter: int) -> float:
    return ((mix_int((key + counter * 3) * _GOLD) >> 11) + 0.5) / float(1 << 53)


# ----------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    batch: int
    ctx: Tuple[int, int]               # (lo, hi) inclusive; lo == hi for a fixed length
    n_q_heads: int
    n_kv_heads: int
    page_size: int
    segment: Tuple[str, int]           # ("equal", count) | ("fixed", tokens) | ("geometric", mean tokens)
    topics_per_q: Tuple[int, int]      # (lo, hi) inclusive
    sink_pages: int = 1
    window_pages: int = 4
    budget_pages: int = 0              # > 0: fixed page budget
    budget_bp: int = 100               # else basis points of the sequence's pages
    head_dim: int = 128
    pages_per_chunk: int = 8
    chunks_per_grid: int = 8
    noise_std: float = 0.5
    equal_norm: bool = False           # rescale every topic vector to norm sqrt(d)
    n_layers: int = 1

    @property
    def max_pages(self) -> int:
        return -(-self.ctx[1] // self.page_size)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def budget_for(self, pages: int) -> int:
        """Page budget k of a sequence of `pages` pages (buffer sizing and length checks only)."""
        if self.budget_pages > 0:
            return self.budget_pages
        return max(1, -(-pages * self.budget_bp // 10000))

    @property
    def max_selected(self) -> int:
        return self.sink_pages + self.window_pages + self.budget_for(self.max_pages)


def spec(name: str, scale: float = 1.0) -> WorkloadSpec:
    """The benchmark configurations (cfg1..cfg5, cfg4b = 5 % budget, cfg5adv = equal-norm topics).
    ``scale`` < 1 shrinks the context (and cfg3's batch / layer count) for CPU-sized tests."""
    def L(n):
        return max(64, int(round(n * scale)))
    if name == "cfg1":
        return WorkloadSpec(name, 1, (L(4096), L(4096)), 8, 8, 16, ("equal", 32), (2, 2), 1, 4, budget_pages=16)
    if name == "cfg2":
        return WorkloadSpec(name, 1, (L(32768), L(32768)), 32, 8, 16, ("fixed", 128), (3, 3), 1, 4)
    if name == "cfg3":
        nb = 32 if scale >= 1 else max(2, int(32 * scale * 4))
        nl = 32 if scale >= 1 else 2
        return WorkloadSpec(name, nb, (L(16384), L(32768)), 32, 8, 16, ("fixed", 128), (3, 3), 1, 4, n_layers=nl)
    if name in ("cfg4a", "cfg4b"):
        nb = 8 if scale >= 1 else 2
        return WorkloadSpec(name, nb, (L(131072), L(131072)), 32, 8, 16, ("geometric", 256), (1, 4), 1, 4,
                            budget_bp=100 if name == "cfg4a" else 500)
    if name in ("cfg5", "cfg5adv"):
        return WorkloadSpec(name, 1, (L(262144), L(262144)), 28, 4, 32, ("geometric", 256), (3, 3), 1, 2,
                            equal_norm=(name == "cfg5adv"))
    raise KeyError(name)


@dataclass
class Workload:
    spec: WorkloadSpec
    seed: int
    layer: int
    k_pool: torch.Tensor        # bf16 [n_phys][H_kv][B][d]
    v_pool: torch.Tensor        # bf16 [n_phys][H_kv][d][B]
    block_table: torch.Tensor   # int32 [batch][max_pages]
    seq_lens: torch.Tensor      # int32 [batch]
    q: torch.Tensor             # bf16 [batch][H_q][d]
    segments: List[List[int]] = field(default_factory=list)        # per sequence: segment start tokens
    q_topics: List[List[List[int]]] = field(default_factory=list)  # [b][hq] -> segment ids the query mixes


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of a bf16 tensor as a numpy uint16 array (host copy)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _segment_starts(sp: WorkloadSpec, seed: int, layer: int, b: int, L: int) -> List[int]:
    kind, val = sp.segment
    if kind == "equal":
        n = min(val, L)
        return [(i * L) // n for i in range(n)]
    if kind == "fixed":
        return list(range(0, L, val))
    key = stream_key(seed, STREAM_SEG, b)      # segments are shared by layers and heads
    p = 1.0 / float(val)
    starts, pos, c = [], 0, 0
    while pos < L:
        starts.append(pos)
        u = uniform_unit(key, c)
        c += 1
        pos += 1 + int(math.floor(math.log(u) / math.log1p(-p)))
    return starts


def seq_lengths(sp: WorkloadSpec, seed: int) -> List[int]:
    lo, hi = sp.ctx
    key = stream_key(seed, STREAM_LEN)
    return [lo + uniform_int(key, b, hi - lo + 1) for b in range(sp.batch)]


def _topic_vectors(sp: WorkloadSpec, seed: int, layer: int, b: int, n_seg: int, dev) -> torch.Tensor:
    """Topic vectors [n_seg][H_kv][d] of sequence b: one per (segment, kv head)."""
    H, d = sp.n_kv_heads, sp.head_dim
    tkey = stream_key(seed, STREAM_TOPIC, layer, b)
    tidx = torch.arange(n_seg * H * d, dtype=torch.int64, device=dev)
    topics = normal_from_counter(tkey, tidx).view(n_seg, H, d)
    if sp.equal_norm:
        topics = topics * (math.sqrt(d) / topics.norm(dim=-1, keepdim=True))
    return topics


def _query_rows(sp: WorkloadSpec, seed: int, layer: int, b: int, variant: int, topics, n_seg: int,
                q: torch.Tensor, dev) -> List[List[int]]:
    """Fill q[b]: every q head = sum of its chosen topic vectors (of its KV head) + noise.  ``variant``
    draws another query for the same keys.  Returns the chosen segment ids per q head."""
    d, G = sp.head_dim, sp.group
    pkey = stream_key(seed, STREAM_PICK, layer, b, variant)
    qkey = stream_key(seed, STREAM_QNOISE, layer, b, variant)
    picks_b = []
    for hq in range(sp.n_q_heads):
        lo, hi = sp.topics_per_q
        T = lo + uniform_int(pkey, hq * 64, hi - lo + 1)
        chosen: List[int] = []
        c = 1
        while n_seg and len(chosen) < min(T, n_seg):
            s_id = uniform_int(pkey, hq * 64 + c, n_seg)
            c += 1
            if s_id not in chosen:
                chosen.append(s_id)
        picks_b.append(chosen)
        noise = normal_from_counter(qkey, torch.arange(hq * d, (hq + 1) * d, dtype=torch.int64, device=dev))
        row = noise * sp.noise_std
        for s_id in chosen:
            row = row + topics[s_id, hq // G]
        q[b, hq] = row.to(torch.bfloat16)
    return picks_b


def extra_queries(wl: "Workload", variant: int) -> torch.Tensor:
    """Another seeded query batch [batch][H_q][d] for the keys of ``wl`` (same recipe, other topic picks)."""
    sp, dev = wl.spec, wl.k_pool.device
    q = torch.empty_like(wl.q)
    for b in range(sp.batch):
        n_seg = len(wl.segments[b])
        topics = _topic_vectors(sp, wl.seed, wl.layer, b, n_seg, dev) if n_seg else None
        _query_rows(sp, wl.seed, wl.layer, b, variant, topics, n_seg, q, dev)
    return q


def generate(sp: WorkloadSpec, seed: int, layer: int = 0, device="cpu", spare_pages: int = 3,
             seq_lens: Optional[List[int]] = None, block_elems: int = 1 << 24) -> Workload:
    """Build one layer's K/V pools, block table, lengths and query for ``sp``."""
    dev = torch.device(device)
    H, d, B, G = sp.n_kv_heads, sp.head_dim, sp.page_size, sp.group
    lens = list(seq_lens) if seq_lens is not None else seq_lengths(sp, seed)
    assert len(lens) == sp.batch and all(0 <= n <= sp.ctx[1] for n in lens)
    pages = [-(-n // B) for n in lens]
    n_phys = sum(pages) + spare_pages

    # logical -> physical: seeded permutation of the pool, shifted so it is never the identity
    perm_gen = torch.Generator(device="cpu")
    perm_gen.manual_seed(stream_key(seed, STREAM_PERM, layer) & 0x7FFFFFFFFFFFFFFF)
    perm = torch.randperm(n_phys, generator=perm_gen)
    perm = (perm + 1) % n_phys if n_phys > 1 and bool((perm == torch.arange(n_phys)).all()) else perm
    bt = torch.full((sp.batch, sp.max_pages), -1, dtype=torch.int32)
    off = 0
    for b, P in enumerate(pages):
        bt[b, :P] = perm[off:off + P].to(torch.int32)
        off += P

    nan16 = torch.tensor(float("nan"), dtype=torch.bfloat16, device=dev)
    k_pool = nan16.repeat(n_phys * H * B * d).view(n_phys, H, B, d)
    v_pool = nan16.repeat(n_phys * H * d * B).view(n_phys, H, d, B)
    q = torch.empty(sp.batch, sp.n_q_heads, d, dtype=torch.bfloat16, device=dev)

    segments, q_topics = [], []
    hd = torch.arange(H * d, dtype=torch.int64, device=dev)
    pages_per_block = max(1, block_elems // (B * H * d))
    for b, Lb in enumerate(lens):
        starts = _segment_starts(sp, seed, layer, b, Lb) if Lb > 0 else []
        segments.append(starts)
        n_seg = len(starts)
        topics = _topic_vectors(sp, seed, layer, b, n_seg, dev) if n_seg else None
        picks_b = _query_rows(sp, seed, layer, b, 0, topics if n_seg else None, n_seg, q, dev)
        q_topics.append(picks_b)
        if Lb == 0:
            continue
        # keys and values, a block of pages at a time
        bounds = torch.tensor(starts, dtype=torch.int64, device=dev)
        kkey = stream_key(seed, STREAM_KNOISE, layer, b)
        vkey = stream_key(seed, STREAM_V, layer, b)
        P = pages[b]
        phys_all = bt[b, :P].to(torch.int64).to(dev)
        for p0 in range(0, P, pages_per_block):
            p1 = min(P, p0 + pages_per_block)
            tok = torch.arange(p0 * B, p1 * B, dtype=torch.int64, device=dev)
            idx = tok[:, None] * (H * d) + hd[None, :]                       # [tokens][H*d]
            seg = torch.searchsorted(bounds, tok, right=True) - 1
            seg = seg.clamp_(0, n_seg - 1)
            kk = topics[seg] + normal_from_counter(kkey, idx).view(-1, H, d) * sp.noise_std
            vv = normal_from_counter(vkey, idx).view(-1, H, d)
            valid = (tok < Lb)[:, None, None]
            kk = torch.where(valid, kk, torch.full_like(kk, float("nan"))).to(torch.bfloat16)
            vv = torch.where(valid, vv, torch.full_like(vv, float("nan"))).to(torch.bfloat16)
            k_pool[phys_all[p0:p1]] = kk.view(p1 - p0, B, H, d).permute(0, 2, 1, 3)
            v_pool[phys_all[p0:p1]] = vv.view(p1 - p0, B, H, d).permute(0, 2, 3, 1)
    return Workload(sp, seed, layer, k_pool, v_pool, bt.to(dev),
                    torch.tensor(lens, dtype=torch.int32, device=dev), q, segments, q_topics)


def default_seed(name: str) -> int:
    base = {"cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4a": 4, "cfg4b": 4, "cfg5": 5, "cfg5adv": 5}
    return 0xC4E55 + base.get(name, 9)
