"""Pins of the oracle's optional decoding rules (no GPU): confidence-based parallel decoding
(the paper's experimental setup: threshold 0.9) and the alternative thresholding variables of
the ablation "Choice of thresholding variable" (entropy sum, max confidence).  Every expectation
is rebuilt from the per-row confidences and entropies a step reports, or from limiting cases
that reduce to the fixed-n rule pinned elsewhere."""
import numpy as np
import pytest

import ec_inputs
from oracle import entropycache as eco


def model_and_prompt(scale=6.0, seed=21):
    cfg = ec_inputs.ModelCfg(n_layers=2, d_model=32, n_heads=4, n_kv_heads=2, head_dim=8,
                             d_ffn=48, vocab=61, mask_id=60, rms_eps=1e-5, rope_base=10000.0,
                             logit_scale=scale, dtype="f32")
    w = ec_inputs.make_weights(cfg, seed, std=0.3, gain_jitter=0.2, threads=1)
    prompt = (ec_inputs.make_prompt(cfg.vocab + 96, 7, seed) % (cfg.vocab - 1)).astype(np.int32)
    return eco.OracleModel(cfg, w), prompt


def run(model, prompt, **kw):
    dec = ec_inputs.DecodeCfg(gen_len=24, block=8, k_recent=2, tokens_per_step=1, tau=1.0, **kw)
    st = eco.eco_init(model, dec, prompt)
    return st, eco.eco_generate(st)


def test_threshold_decoding_commits_exactly_the_rows_above_the_threshold():
    model, prompt = model_and_prompt()
    thr = 0.35
    st, trace = run(model, prompt, conf_threshold=thr)
    saw_many = False
    for r in trace:
        conf, Mb, D = r["conf"], list(r["Mb"]), r["positions"]
        above = [int(p) for p, c in zip(Mb, conf) if c > thr]
        if above:
            assert sorted(D) == sorted(above)          # all of them, nothing else
        else:
            assert D == [int(Mb[int(np.argmax(conf))])]  # none confident: the single best row
        saw_many |= len(D) > 1
        assert len(D) <= eco.MAX_TOKENS_PER_STEP
    assert saw_many, "seed never decodes several tokens at once: the test would be vacuous"
    assert not st.masked.any()


def test_threshold_limits_reduce_to_known_schedules():
    model, prompt = model_and_prompt()
    _, fixed = run(model, prompt)
    _, high = run(model, prompt, conf_threshold=0.999999)   # nothing ever exceeds it
    assert [r["positions"] for r in high] == [r["positions"] for r in fixed]
    assert [r["tokens"] for r in high] == [r["tokens"] for r in fixed]
    _, low = run(model, prompt, conf_threshold=1e-9)        # everything exceeds it
    assert len(low) == 3 and all(len(r["positions"]) == 8 for r in low)   # one step per block
    _, mid = run(model, prompt, conf_threshold=0.35)
    assert len(low) <= len(mid) <= len(fixed)


@pytest.mark.parametrize("metric", [0, 1, 2])
def test_gate_value_and_flag_follow_the_reported_rows(metric):
    model, prompt = model_and_prompt()
    tau = {0: 0.9, 1: 1.5, 2: 0.8}[metric]
    dec = dict(conf_threshold=0.5, gate_metric=metric)
    d = ec_inputs.DecodeCfg(gen_len=24, block=8, k_recent=2, tokens_per_step=1, tau=tau, **dec)
    st = eco.eco_init(model, d, prompt)
    trace = eco.eco_generate(st)
    flags = set()
    for r in trace:
        rowof = {int(p): i for i, p in enumerate(r["Mb"])}
        H = [float(r["H"][rowof[p]]) for p in r["positions"]]
        c = [float(r["conf"][rowof[p]]) for p in r["positions"]]
        want = {0: max(H), 1: float(np.sum(H)), 2: max(c)}[metric]
        assert r["E"] == pytest.approx(want, rel=1e-12, abs=1e-15)
        assert r["skip"] == ((want >= tau) if metric == 2 else (want <= tau))
        flags.add(r["skip"])
    assert flags == {True, False}, "threshold never crossed: the test would be vacuous"


def test_entropy_sum_equals_max_entropy_when_one_token_is_decoded_per_step():
    model, prompt = model_and_prompt()
    _, a = run(model, prompt, gate_metric=0)
    _, b = run(model, prompt, gate_metric=1)
    assert [(r["mode"], r["positions"], r["tokens"], r["E"]) for r in a] == \
           [(r["mode"], r["positions"], r["tokens"], r["E"]) for r in b]


def test_sliding_window_limits_and_invariants():
    """Sliding-window schedule: with a window covering the whole generation it is the single-block
    schedule; with a window of one it decodes strictly left to right; in between the window
    always holds min(w, remaining) masked slots and nothing right of it is decoded early."""
    model, prompt = model_and_prompt()
    N = 24

    def gen(**kw):
        d = ec_inputs.DecodeCfg(gen_len=N, k_recent=2, tokens_per_step=1, tau=1.0, **kw)
        st = eco.eco_init(model, d, prompt)
        return st, eco.eco_generate(st)

    _, whole_blocks = gen(block=N, schedule=0)
    _, whole_window = gen(block=N, schedule=1)
    assert [(r["mode"], r["positions"], r["tokens"]) for r in whole_blocks] == \
           [(r["mode"], r["positions"], r["tokens"]) for r in whole_window]

    st, one = gen(block=1, schedule=1)
    assert [r["positions"][0] for r in one] == list(range(st.P, st.P + N))

    st, mid = gen(block=5, schedule=1)
    remaining = N
    decoded = set()
    for r in mid:
        Mb = [int(p) for p in r["Mb"]]
        assert len(Mb) == min(5, remaining)
        # every generation slot left of the window's last position is either in it or decoded
        for p in range(st.P, Mb[-1] + 1):
            assert p in Mb or p in decoded
        decoded.update(r["positions"])
        remaining -= len(r["positions"])
    assert remaining == 0 and len(mid) == N
    # unlike fixed blocks, the window moves before it is empty
    assert any(r["Mb"][-1] > st.P + 4 and len(r["Mb"]) == 5 for r in mid[:6])
