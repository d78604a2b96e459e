"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only; no GPU involved).

``oracle/chess_oracle.c`` is compiled, with ``tests/oracle_sanitized_driver.c``, into an executable with
``-fsanitize=address,undefined`` (the runtime linked statically, so nothing has to be preloaded), run on a ragged
workload that exercises every oracle function -- both cut rules, all three plans, both probes, per-sequence budgets,
the model-wide scope, sparse and dense attention, the entropy monitor -- and its results must equal those of the
ordinary build bit for bit.  Any sanitizer report fails the run (``-fno-sanitize-recover=all``)."""
from __future__ import annotations

import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
import workload
from helpers import geom_of, host_arrays, plan_of

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _records(path):
    out, raw = [], open(path, "rb").read()
    at = 0
    while at < len(raw):
        (n,) = struct.unpack_from("<q", raw, at)
        out.append(raw[at + 8:at + 8 + n])
        at += 8 + n
    return out


@pytest.mark.parametrize("summary_dtype", [oracle.SUMMARY_F32, oracle.SUMMARY_BF16])
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path, summary_dtype):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-fno-fast-math", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           os.path.join(ROOT, "oracle", "chess_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitized_driver.c"),
           "-o", exe, "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0 and "static-lib" in res.stderr:
        pytest.skip("this gcc has no static sanitizer runtimes")
    assert res.returncode == 0, res.stderr

    sp = workload.WorkloadSpec("ragged", 3, (64, 3000), 8, 2, 16, ("fixed", 128), (2, 2), 1, 2, budget_bp=300,
                               pages_per_chunk=4, chunks_per_grid=4)
    wl = workload.generate(sp, 77, seq_lens=[3000, 1237, 16])          # the last one is covered by its safety pages
    K, V, Q, bt, sl = host_arrays(wl)
    g = geom_of(sp, summary_dtype=summary_dtype)
    per = (9, 0, 2)
    plans = [plan_of(sp),
             plan_of(sp, plan=oracle.PLAN_RATIO, rho_g_bp=5000, rho_c_bp=4000, rho_p_bp=3000, cut_rule=oracle.CUT_THRESHOLD),
             plan_of(sp, plan=oracle.PLAN_FLAT, budget_pages=11, probe=oracle.PROBE_ANCHOR),
             plan_of(sp, budget_per_seq=per, cut_rule=oracle.CUT_THRESHOLD)]
    rng = np.random.default_rng(5)
    logits = workload.bf16_bits(__import__("torch").as_tensor(rng.standard_normal((2, 1000)).astype(np.float32) * 4).bfloat16())
    H = rng.random(16).astype(np.float32)

    def rec(a):
        b = np.ascontiguousarray(a).tobytes()
        return struct.pack("<q", len(b)) + b

    inp = tmp_path / "in.bin"
    with open(inp, "wb") as f:
        f.write(rec(np.array([g.n_q_heads, g.n_kv_heads, g.head_dim, g.page_size, g.pages_per_chunk, g.chunks_per_grid,
                              g.max_pages, g.summary_dtype], np.int32)))
        f.write(rec(np.array([[p.plan, p.sink_pages, p.window_pages, p.budget_pages, p.budget_bp, p.over_chunk, p.over_grid,
                               p.rho_g_bp, p.rho_c_bp, p.rho_p_bp, p.probe, p.cut_rule] for p in plans], np.int32)))
        f.write(rec(sl.astype(np.int32)) + rec(bt.astype(np.int32)) + rec(K) + rec(V) + rec(Q))
        f.write(rec(np.array(per, np.int32)))
        f.write(rec(logits) + rec(np.array([997, 1000], np.int32)) + rec(H))
    outp = tmp_path / "out.bin"
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, str(inp), str(outp)], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0 and "ERROR" not in run.stderr and "runtime error" not in run.stderr, run.stderr[-4000:]

    # the same calls through the ordinary build (every plan here uses the per-sequence budgets, as the driver does)
    r = iter(_records(outp))
    pv, cv, gv = oracle.summarize(K, bt, sl, g)
    for ref in (pv, cv, gv):
        assert next(r) == ref.tobytes()
    anc = oracle.anchor(pv, sl, g, plans[0].window_pages)
    assert next(r) == anc.tobytes()
    from dataclasses import replace
    for p in plans:
        p = replace(p, budget_per_seq=per)
        ps, _, _ = oracle.scores(Q, pv, cv, gv, sl, g, p)
        got = np.frombuffer(next(r), np.float64).reshape(ps.shape)
        live = ~np.isnan(ps)                                     # the wrapper pre-fills rows past a sequence's pages with NaN
        assert np.array_equal(got[live], ps[live])
        ids, nsel, _, _, cnt = oracle.select(Q, pv, cv, gv, sl, g, p, g.max_pages, detail=True)
        assert struct.unpack("<i", next(r))[0] == 0
        assert next(r) == ids.tobytes() and next(r) == nsel.tobytes() and next(r) == cnt.tobytes()
        assert next(r) == oracle.attend(Q, K, V, bt, sl, g, ids, nsel).tobytes()
        sid, sn = oracle.select_shared([anc, anc], [pv, pv], [cv, cv], [gv, gv], sl, g, p, g.max_pages)
        assert struct.unpack("<i", next(r))[0] == 0
        assert next(r) == sid.tobytes() and next(r) == sn.tobytes()
    assert next(r) == oracle.attend(Q, K, V, bt, sl, g).tobytes()
    assert next(r) == oracle.entropy(logits, vocab=997).tobytes()
    mean, var, fire = oracle.page_trigger(H, 1.0, 0.5)
    assert next(r) == struct.pack("<dd", mean, var) and struct.unpack("<i", next(r))[0] == int(fire)
