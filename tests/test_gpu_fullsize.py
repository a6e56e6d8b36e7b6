"""GPU parity at the real widths and vocabularies of the paper's models, in the launch
configuration bench.py times (bf16, skinny GEMMs for partial steps, tiled GEMMs for full steps).

* 2-layer twins of the LLaDA-8B and Dream-7B shapes (same d, heads, FFN, vocabulary, context):
  many teacher-forced steps against the live fp64 oracle, with a FULL step forced periodically so
  both launch shapes run whatever the random model's entropies are.
* Full depth: the 32-layer LLaDA-8B shape, the 28-layer Dream-7B shape (GQA 28/4, two tokens per
  step) and the long chain-of-thought shape (1280 positions, k = 4), each replaying a short stored
  oracle trace FULL, PARTIAL x 3, FULL, PARTIAL; and 16 sequences of 1024 + 512 positions side by
  side on the 2-layer twin, free-running, so that FULL and PARTIAL sequences share launches.
  The traces (tests/golden/*_trace.json / .npz) are written by tests/golden/make_traces.py,
  which calls only the oracle: per block row the 16 largest logits and 256 random columns, the
  row statistics, and K / V at sampled positions, layers and heads over the whole head dimension.
Tolerance 2e-2 of the tensor's largest magnitude (bf16 bar); the statistics and decision checks
are those of tests/gpu_harness.py."""
import json
import os

import numpy as np
import pytest

import ec_inputs
import paper_2603_18489_amd as ec
from oracle import entropycache as eco
from tests.gpu_harness import (Counters, check_against_oracle, check_own_decision,
                               check_reduction, gpu_cache, run_teacher_forced,
                               run_teacher_forced_batch)

pytestmark = pytest.mark.gpu
TOL = 2e-2
HERE = os.path.dirname(os.path.abspath(__file__))


def periodic_full(period):
    return lambda i: eco.FULL if i % period == 0 else eco.PARTIAL


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,steps,period,scale", [
    ("llada8b_l2", 72, 12, 8.0),        # 34-row partial steps, 768-row full steps, block change at 32/64
    ("dream7b_l2", 36, 12, 8.0),        # GQA 28/4, 2 tokens per step, T = 1280
    ("llada8b_fp8_l2", 36, 12, 8.0),    # matrices as e4m3 codes + row scales
])
def test_two_layer_twins(name, steps, period, scale):
    wl = ec_inputs.WORKLOADS[name]
    cfg = wl.model.replace(logit_scale=scale)
    w = ec_inputs.make_weights(cfg, wl.seed, threads=16)
    prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    eco.enable_f64_cache(True)
    try:
        s = run_teacher_forced(cfg, w, wl.decode, prompt, TOL, max_steps=steps,
                               check_cache_every=6, mode_fn=periodic_full(period), verbose=True)
    finally:
        eco.enable_f64_cache(False)
    print(s)
    assert s["steps"] == steps and s["modes"][eco.FULL] == steps // period
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0 and s["modes_exact"] > 0


@pytest.mark.timeout(900)
def test_long_cot_shape_two_layers():
    """Config-4 shape: prompt 256 + generation 1024, k = 4, tau = 0.5 on a 2-layer LLaDA twin."""
    wl = ec_inputs.WORKLOADS["llada8b_cot"]
    cfg = wl.model.replace(n_layers=2, logit_scale=8.0)
    w = ec_inputs.make_weights(cfg, wl.seed, threads=16)
    prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    eco.enable_f64_cache(True)
    try:
        s = run_teacher_forced(cfg, w, wl.decode, prompt, TOL, max_steps=40, check_cache_every=8,
                               mode_fn=periodic_full(10), verbose=True)
    finally:
        eco.enable_f64_cache(False)
    print(s)
    assert s["steps"] == 40
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0 and s["modes_exact"] > 0


@pytest.mark.timeout(900)
def test_batch_of_ragged_sequences_two_layers():
    """The many-sequence shape (ragged prompts, one row list per step) on a 2-layer LLaDA twin:
    every sequence against its own oracle run; free-running modes, so FULL and PARTIAL sequences
    share steps."""
    wl = ec_inputs.WORKLOADS["llada8b_l2"]
    cfg = wl.model.replace(logit_scale=8.0)
    w = ec_inputs.make_weights(cfg, wl.seed, threads=16)
    dec = wl.decode.replace(gen_len=64, batch=3)
    prompts = [ec_inputs.make_prompt(cfg.vocab, P, 40 + i) for i, P in enumerate((300, 77, 160))]
    eco.enable_f64_cache(True)
    try:
        s = run_teacher_forced_batch(cfg, w, dec, prompts, TOL, max_steps=10, check_cache_every=5)
    finally:
        eco.enable_f64_cache(False)
    print(s)
    assert s["steps"] == 10 and s["modes"][eco.FULL] >= 3 and s["modes"][eco.PARTIAL] >= 3
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0


# ---- stored oracle traces ---------------------------------------------------------------------
def check_trace_step(cfg, dec, gold, st, arr, key, q, g, cnt, seq, where):
    """One step of one sequence against the stored oracle samples."""
    nmb = len(st["Mb"])
    assert q["mode_run"] == st["mode"] and q["n_query_rows"] == st["n_rows"], where
    assert q["n_block_rows"] == nmb and q["step_index"] == st["t"], where
    assert q["done"] == st["done"] and q["n_recent_next"] == len(st["R"]), where
    logits = g.debug_read(ec.EC_DBG_LOGITS, count=nmb, seq=seq)
    stats = g.debug_read(ec.EC_DBG_ROW_STATS, count=nmb, seq=seq)
    cols = arr[key + "cols"].astype(np.int64)
    ref_z = arr[key + "logits"].astype(np.float64)
    diff = np.abs(np.take_along_axis(logits, cols, axis=1).astype(np.float64) - ref_z)
    e = float(diff.max() / st["logits_absmax"])
    cnt.up("logits", e)
    assert e <= TOL, f"{where}: logits rel err {e:.3e}"
    # the sampled columns hold each row's 16 largest logits: the oracle's argmax is among them
    assert [int(c) for c in cols[:, 0]] == st["tok"]
    check_reduction(cfg, logits, stats, cnt, where)
    check_own_decision(stats, st["Mb"], dec, q, where)
    # per-row logit error: measured on 272 of the V columns, doubled for the ones not sampled
    dz_row = 2.0 * diff.max(axis=1) + 0.02 * TOL * st["logits_absmax"]
    ref = {"Mb": st["Mb"], "tok": st["tok"], "conf": np.array(st["conf"]), "H": np.array(st["H"]),
           "top2gap": np.array(st["top2gap"]), "H_sens": np.array(st["H_sens"]),
           "logits_absmax": st["logits_absmax"], "own_positions": st["own_positions"],
           "own_tokens": st["own_tokens"], "E_own": st["E_own"]}
    check_against_oracle(cfg, dec, TOL, ref, q, stats, dz_row, cnt, where)
    pos = arr[key + "kv_pos"]
    for li, l in enumerate(gold["layers"]):
        for name, which in (("K", ec.EC_DBG_KCACHE), ("V", ec.EC_DBG_VCACHE)):
            c = gpu_cache(g, which, l, seq=seq)[pos][:, gold["heads"], :]
            ref_kv = arr[key + name][li]
            e = float(np.abs(c - ref_kv).max() / st[name + "_absmax"][li])
            cnt.up(name, e)
            assert e <= TOL, f"{where} layer {l}: {name} rel err {e:.3e}"
            # and every sampled (position, head) vector against its own largest magnitude: an
            # error confined to a few rows or heads cannot hide behind the layer's maximum
            ev = float((np.abs(c - ref_kv).max(axis=-1) / np.abs(ref_kv).max(axis=-1)).max())
            cnt.up(name + "_vec", ev)
            assert ev <= VEC_TOL, f"{where} layer {l}: {name} vector rel err {ev:.3e}"


# A sampled (position, head) vector's own largest magnitude can lie several times below its
# layer's, so the same absolute error reads larger against it: 4 x the tensor bar (observed:
# up to 0.041 at 32 layers, 0.01 - 0.02 on the 2-layer batch trace).
VEC_TOL = 4 * TOL


def load_trace(name):
    gold = json.load(open(os.path.join(HERE, "golden", f"{name}_trace.json")))
    arr = np.load(os.path.join(HERE, "golden", f"{name}_trace.npz"))
    wl = ec_inputs.WORKLOADS[gold["workload"]]
    cfg = wl.model.replace(logit_scale=gold["logit_scale"], n_layers=gold["n_layers"])
    return gold, arr, wl, cfg


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["llada8b", "dream7b", "llada8b_cot"])
def test_full_depth_against_stored_oracle_trace(name):
    gold, arr, wl, cfg = load_trace(name)
    w = ec_inputs.make_weights(cfg, wl.seed, threads=16)
    prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), wl.decode, prompt)
    g.keep_logits(True)
    del w
    cnt = Counters()
    try:
        for i, st in enumerate(gold["steps"]):
            q = g.step_forced(st["mode"], st["positions"], st["tokens"])
            check_trace_step(cfg, wl.decode, gold, st, arr, f"s{i}_", q, g, cnt, 0, f"step {st['t']}")
            print(f"t={st['t']} mode={st['mode']} rows={st['n_rows']} {cnt.summary()}", flush=True)
    finally:
        g.close()
    assert cnt.tokens_exact > 0 and cnt.rows_decided + cnt.modes_exact > 0


@pytest.mark.timeout(900)
def test_sixteen_sequences_against_stored_oracle_traces():
    """16 sequences of 1024 + 512 positions in one context (2-layer twin of the LLaDA-8B shape):
    each follows its own oracle run's entropy flag, so steps mix 1536-row and <= 34-row sequences
    in the same launches."""
    gold, arr, wl, cfg = load_trace("llada8b_b16")
    B = gold["batch"]
    w = ec_inputs.make_weights(cfg, wl.seed, threads=16)
    prompts = [ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, s) for s in gold["prompt_seeds"]]
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), wl.decode, prompts)
    g.keep_logits(True)
    del w
    dec1 = wl.decode.replace(batch=1)
    cnt = Counters()
    mixed = 0
    try:
        for i, per_seq in enumerate(gold["steps"]):
            modes = [s["mode"] for s in per_seq]
            mixed += int(0 < sum(modes) < B)
            q = g.step_forced_batch(modes, [s["positions"] for s in per_seq],
                                    [s["tokens"] for s in per_seq])
            for b, st in enumerate(per_seq):
                check_trace_step(cfg, dec1, gold, st, arr, f"s{i}_b{b}_", q[b], g, cnt, b,
                                 f"seq {b} step {st['t']}")
            print(f"step {i + 1} modes {modes} {cnt.summary()}", flush=True)
    finally:
        g.close()
    assert mixed >= 2
    assert cnt.tokens_exact > 0 and cnt.rows_decided > 0 and cnt.modes_exact > 0
