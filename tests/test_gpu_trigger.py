"""GPU parity of the Sec. 3.3 monitor: chess_entropy against the oracle's fp64 entropy (fp32 arithmetic on the GPU:
absolute tolerance 2e-4 nats, derived from ~150K fp32 exponentials at 1e-6 relative each with random signs, times
log V), and chess_trigger_update -- fp64 arithmetic in step order on both sides -- bit-exact on the same inputs."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2602_20732_amd as pk
import workload
from helpers import f32_to_bf16_bits

pytestmark = pytest.mark.gpu
SUMMARY_DTYPE_SWEEP = False       # nothing here reads or writes summary vectors
ATOL = 2e-4


def make_lib(max_batch):
    return pk.Chess(pk.Config(n_q_heads=8, n_kv_heads=8, page_size=16, max_batch=max_batch, max_pages_per_seq=64,
                              max_selected_pages=16))


@pytest.mark.parametrize("batch,vocab,stride", [(1, 151936, 151936), (32, 151936, 151936), (5, 1000, 1024), (3, 7, 8),
                                                (64, 32003, 32008)])
def test_entropy_matches_the_oracle(batch, vocab, stride):
    lib = make_lib(64)
    rng = np.random.default_rng(vocab + batch)
    z = (rng.standard_normal((batch, stride)) * rng.uniform(0.2, 6.0, (batch, 1))).astype(np.float32)
    z[:, vocab:] = 80.0                                    # padding beyond the vocabulary must not count
    if batch >= 3:
        z[1, :vocab] = 1.5                                 # uniform row: log V
        z[2, :vocab] = -30.0; z[2, vocab // 2] = 40.0      # one dominant token: ~0
    bits = f32_to_bf16_bits(z)
    d = torch.as_tensor(bits.view(np.int16)).cuda().view(torch.bfloat16)
    H = torch.full((batch,), float("nan"), device="cuda")
    ws = lib.new_workspace()
    for _ in range(2):                                     # the arrival counters re-arm themselves
        lib.entropy(d, H, ws, vocab=vocab)
        torch.cuda.synchronize()
        ref = oracle.entropy(bits, vocab=vocab)
        got = H.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all() and np.abs(got - ref).max() <= ATOL, np.abs(got - ref).max()
    if batch >= 3:
        assert abs(got[1] - np.log(vocab)) <= ATOL and abs(got[2]) <= ATOL
    lib.close()


def test_masked_logits_count_as_probability_zero():
    lib = make_lib(2)
    z = np.full((2, 4096), -np.inf, np.float32)
    z[0, [5, 77, 4000]] = 0.25                             # three equally likely tokens: log 3
    z[1, 9] = 3.0                                          # one token: 0
    bits = f32_to_bf16_bits(z)
    d = torch.as_tensor(bits.view(np.int16)).cuda().view(torch.bfloat16)
    H = torch.full((2,), float("nan"), device="cuda")
    lib.entropy(d, H, lib.new_workspace())
    got = H.cpu().numpy()
    assert abs(got[0] - np.log(3)) <= 1e-6 and got[1] == 0.0
    assert np.abs(oracle.entropy(bits) - got).max() <= 1e-6
    lib.close()


def test_trigger_update_is_bit_exact_and_fires_on_either_threshold():
    lib = make_lib(6)
    batch, page = 6, 16
    rng = np.random.default_rng(3)
    steps = 3 * page + 5
    Hs = rng.uniform(0.5, 3.0, (steps, batch)).astype(np.float32)
    Hs[page:2 * page, 1] += 2.0                            # a page of high entropy for sequence 1
    Hs[2 * page:3 * page:2, 2] += 3.0                      # an unstable page for sequence 2
    tau_h, tau_v = 3.0, 1.5
    hist = torch.zeros((batch, page), device="cuda")
    count = torch.zeros((batch,), dtype=torch.int32, device="cuda")
    fire = torch.full((batch,), -1, dtype=torch.int32, device="cuda")
    stats = torch.zeros((batch, 2), dtype=torch.float64, device="cuda")
    fired = []
    for t in range(steps):
        lib.trigger_update(torch.as_tensor(Hs[t]).cuda(), page, tau_h, tau_v, hist, count, fire, stats)
        f = fire.cpu().numpy()
        if (t + 1) % page:
            assert not f.any() and int(count[0]) == (t + 1) % page
            continue
        st = stats.cpu().numpy()
        for b in range(batch):
            mean, var, fr = oracle.page_trigger(Hs[t + 1 - page:t + 1, b], tau_h, tau_v)
            assert st[b, 0] == mean and st[b, 1] == var and bool(f[b]) == fr, (t, b)
        fired.append(f.copy())
    assert fired[1][1] == 1 and fired[2][2] == 1 and fired[0].sum() == 0, fired
    with pytest.raises(pk.ChessError):
        lib.trigger_update(torch.as_tensor(Hs[0]).cuda(), 0, tau_h, tau_v, hist, count, fire, stats)
    lib.close()


def test_monitor_step_equals_the_two_calls():
    """chess_monitor_step (entropy + page statistics in one launch) against chess_entropy + chess_trigger_update on
    the same logits, step by step over three pages: entropies, flags, statistics and counters identical."""
    lib = make_lib(8)
    batch, page, vocab = 8, 4, 50000
    gen = torch.Generator(device="cuda").manual_seed(11)
    ws = lib.new_workspace()

    def state():
        return dict(H=torch.zeros((batch,), device="cuda"), hist=torch.zeros((batch, page), device="cuda"),
                    count=torch.zeros((batch,), dtype=torch.int32, device="cuda"),
                    fire=torch.full((batch,), -1, dtype=torch.int32, device="cuda"),
                    stats=torch.zeros((batch, 2), dtype=torch.float64, device="cuda"))
    A, B = state(), state()
    fired = 0
    for t in range(3 * page):
        scale = torch.rand((batch, 1), device="cuda", generator=gen) * 4 + 0.1
        logits = (torch.randn((batch, vocab), device="cuda", generator=gen) * scale).to(torch.bfloat16)
        lib.entropy(logits, A["H"], ws)
        lib.trigger_update(A["H"], page, 9.5, 0.6, A["hist"], A["count"], A["fire"], A["stats"])
        lib.monitor_step(logits, page, 9.5, 0.6, B["H"], B["hist"], B["count"], B["fire"], ws, stats=B["stats"])
        torch.cuda.synchronize()
        for k in A:
            assert torch.equal(A[k], B[k]), (t, k)
        fired += int(A["fire"].sum())
    assert 0 < fired < 3 * batch, "thresholds chosen so that some pages fire and some do not"
    ref = oracle.entropy(logits.view(torch.int16).cpu().numpy().view(np.uint16))
    assert np.abs(B["H"].cpu().numpy() - ref).max() <= ATOL
    with pytest.raises(pk.ChessError):
        lib.monitor_step(logits, 0, 1.0, 1.0, B["H"], B["hist"], B["count"], B["fire"], ws)
    lib.close()
