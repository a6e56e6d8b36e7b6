"""GPU parity: the HIP path behind the C ABI against the fp64 oracle, element by element, under
teacher forcing.  Tolerances (relative to the tensor's largest magnitude): 1e-4 for float32
models, 2e-2 for bfloat16 models; integer state, row sets and decisions are bit-exact (decisions
wherever the oracle's margins exceed the tolerance)."""
import math

import numpy as np
import pytest

import ec_inputs
import paper_2603_18489_amd as ec
from oracle import entropycache as eco
from tests.gpu_harness import run_teacher_forced, run_teacher_forced_batch, relerr

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2, "fp8w": 2e-2}


def small_cfg(dtype, hq=4, hkv=4, hd=64, d=256, f=768, vocab=4096, layers=2, scale=16.0):
    return ec_inputs.ModelCfg(n_layers=layers, d_model=d, n_heads=hq, n_kv_heads=hkv, head_dim=hd,
                              d_ffn=f, vocab=vocab, mask_id=vocab - 1, rms_eps=1e-5,
                              rope_base=10000.0, logit_scale=scale, dtype=dtype)


def test_tiny_f32_whole_generation():
    wl = ec_inputs.WORKLOADS["tiny_f32"]
    cfg = wl.model.replace(logit_scale=16.0)      # both modes occur (about half the steps FULL)
    w = ec_inputs.make_weights(cfg, wl.seed, gain_jitter=0.1)
    prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    s = run_teacher_forced(cfg, w, wl.decode, prompt, TOL["f32"])
    print(s)
    assert s["steps"] == 64 and s["modes"][eco.FULL] >= 2 and s["modes"][eco.PARTIAL] >= 10
    assert s["exact_checked"] >= 32


@pytest.mark.parametrize("dtype,hq,hkv,hd,P,N,block,k,n,tau", [
    ("f32", 4, 2, 64, 37, 45, 16, 3, 2, 2.5),       # GQA, ragged last block, T not / 16
    ("f32", 2, 1, 128, 5, 9, 32, 0, 1, 1e9),        # gen shorter than block, k = 0, head_dim 128
    ("bf16", 4, 4, 64, 64, 64, 32, 2, 1, 3.0),
    ("bf16", 4, 2, 128, 50, 70, 32, 4, 2, 2.5),     # GQA, head_dim 128, 70 = 2 blocks + 6
    ("bf16", 8, 2, 64, 100, 33, 32, 2, 3, 1e9),     # T = 133 > 128 rows: tiled GEMM in FULL
    ("bf16", 4, 2, 64, 40, 128, 32, 64, 1, 1e9),    # k = 64: partial steps of 65 .. 96 rows
])
def test_small_models_whole_generation(dtype, hq, hkv, hd, P, N, block, k, n, tau):
    cfg = small_cfg(dtype, hq, hkv, hd, d=hq * hd if hq * hd >= 256 else 256)
    w = ec_inputs.make_weights(cfg, 7, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=N, block=block, k_recent=k, tokens_per_step=n, tau=tau)
    prompt = ec_inputs.make_prompt(cfg.vocab, P, 3)
    s = run_teacher_forced(cfg, w, dec, prompt, TOL[dtype])
    print(s)
    assert s["modes"][eco.PARTIAL] >= 1
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0 and s["modes_exact"] > 0


@pytest.mark.parametrize("dtype,thr,metric,tau,scale", [
    ("f32", 0.5, ec.EC_GATE_MAX_ENTROPY, 2.5, 13.0),
    ("f32", 0.35, ec.EC_GATE_ENTROPY_SUM, 4.0, 13.0),
    ("f32", 0.5, ec.EC_GATE_MAX_CONFIDENCE, 0.3, 13.0),
    ("bf16", 0.5, ec.EC_GATE_MAX_ENTROPY, 2.5, 13.0),
    ("bf16", 0.5, ec.EC_GATE_ENTROPY_SUM, 6.0, 13.0),
])
def test_confidence_threshold_decoding_and_gate_metrics(dtype, thr, metric, tau, scale):
    """Confidence-based parallel decoding (several tokens per step, the recent set grows by ties)
    and the alternative thresholding variables, against the oracle under teacher forcing."""
    cfg = small_cfg(dtype, 4, 2, 64, scale=scale)
    w = ec_inputs.make_weights(cfg, 17, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=80, block=32, k_recent=4, tokens_per_step=1, tau=tau,
                              conf_threshold=thr, gate_metric=metric)
    prompt = ec_inputs.make_prompt(cfg.vocab, 45, 9)
    s = run_teacher_forced(cfg, w, dec, prompt, TOL[dtype])
    print(s)
    assert s["modes"][eco.PARTIAL] >= 1 and s["modes"][eco.FULL] >= 1
    assert s["steps"] < 80, "no step decoded several tokens: the threshold path did not run"
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0 and s["modes_exact"] > 0


@pytest.mark.parametrize("dtype,block,k,n,thr,tau", [
    ("f32", 16, 3, 2, 0.0, 2.5),      # window slides by two slots a step
    ("bf16", 32, 4, 1, 0.5, 2.5),     # with confidence-based parallel decoding
])
def test_sliding_window_schedule(dtype, block, k, n, thr, tau):
    """Sliding-window decoding: M^t is the leftmost `block` masked slots, so the row sets differ
    from the blockwise ones at every step."""
    cfg = small_cfg(dtype, 4, 2, 64, scale=13.0)
    w = ec_inputs.make_weights(cfg, 17, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=70, block=block, k_recent=k, tokens_per_step=n, tau=tau,
                              conf_threshold=thr, schedule=ec.EC_SCHED_SLIDING)
    prompt = ec_inputs.make_prompt(cfg.vocab, 45, 9)
    s = run_teacher_forced(cfg, w, dec, prompt, TOL[dtype])
    print(s)
    assert s["modes"][eco.PARTIAL] >= 1 and s["modes"][eco.FULL] >= 1
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0 and s["modes_exact"] > 0


@pytest.mark.parametrize("hq,hkv,hd", [(4, 4, 64), (4, 2, 128)])
def test_long_context_partial_steps(hq, hkv, hd):
    """More than 2048 keys: the partial-step attention cuts the keys into slices that different
    blocks reduce and the last one to finish adds up."""
    cfg = small_cfg("bf16", hq, hkv, hd, d=hq * hd if hq * hd >= 256 else 256)
    w = ec_inputs.make_weights(cfg, 11, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=40, block=32, k_recent=3, tokens_per_step=2, tau=1e9)
    prompt = ec_inputs.make_prompt(cfg.vocab, 2100, 5)
    s = run_teacher_forced(cfg, w, dec, prompt, TOL["bf16"], max_steps=8)
    print(s)
    assert s["modes"][eco.PARTIAL] >= 6
    assert s["tokens_exact"] > 0 and s["modes_exact"] > 0


@pytest.mark.parametrize("hq,hkv,hd,plens,N,block,k,n,tau,fast", [
    (4, 4, 64, [40, 100, 7], 40, 16, 2, 2, 3.0, None),      # ragged prompts, mixed modes
    (4, 2, 128, [70, 9, 33, 150], 36, 32, 3, 1, 2.5, 1),    # GQA; sequence 1 finishes early;
                                                             # 150 + 36 rows: a many-row sequence
])
def test_batched_sequences_match_their_own_oracle_runs(hq, hkv, hd, plens, N, block, k, n, tau, fast):
    """Sequences of a batch are independent: each must reproduce the oracle run on it alone,
    whatever modes the others are in and after some of them have finished."""
    cfg = small_cfg("bf16", hq, hkv, hd, d=hq * hd if hq * hd >= 256 else 256)
    w = ec_inputs.make_weights(cfg, 13, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=N, block=block, k_recent=k, tokens_per_step=n, tau=tau,
                              batch=len(plens))
    prompts = [ec_inputs.make_prompt(cfg.vocab, P, 20 + i) for i, P in enumerate(plens)]
    s = run_teacher_forced_batch(cfg, w, dec, prompts, TOL["bf16"], fast_seq=fast)
    print(s)
    assert s["modes"][eco.PARTIAL] >= 1 and s["modes"][eco.FULL] >= len(plens)
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0 and s["modes_exact"] > 0
    if fast is not None:
        assert s["finished_early"] >= 1


def test_tile_counts_that_do_not_divide_the_block_widths():
    """Feature counts whose 16-row tiles are not a multiple of the tiles a GEMM block owns:
    772 gate/up tiles in groups of 3, 257 vocabulary tiles in groups of 4 (the last group of the
    packed layout is partly empty, the last block's surplus tiles must be dropped)."""
    cfg = small_cfg("bf16", 4, 2, 64, f=6176, vocab=4112)
    w = ec_inputs.make_weights(cfg, 37, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=40, block=32, k_recent=2, tokens_per_step=2, tau=3.0)
    prompt = ec_inputs.make_prompt(cfg.vocab, 150, 8)    # 190 rows in FULL steps: tiled GEMMs
    s = run_teacher_forced(cfg, w, dec, prompt, TOL["bf16"])
    print(s)
    assert s["modes"][eco.PARTIAL] >= 1 and s["modes"][eco.FULL] >= 1
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0 and s["modes_exact"] > 0


def _random_case(seed):
    r = np.random.RandomState(seed)
    hkv, hd = int(r.choice([1, 2, 4])), int(r.choice([64, 128]))
    hq = hkv * int(r.choice([1, 2, 4])) if hd == 64 else hkv * int(r.choice([1, 2]))
    return dict(dtype=str(r.choice(["f32", "bf16"])), hq=hq, hkv=hkv, hd=hd,
                P=int(r.randint(0, 90)), N=int(r.randint(5, 70)), block=int(r.choice([4, 8, 16, 32])),
                k=int(r.randint(0, 12)), n=int(r.randint(1, 4)), tau=float(r.choice([1.5, 2.5, 3.5, 1e9])),
                thr=float(r.choice([0.0, 0.0, 0.4])), metric=int(r.choice([0, 0, 1, 2])),
                schedule=int(r.choice([0, 1])), scale=float(r.choice([10.0, 13.0, 16.0])))


@pytest.mark.parametrize("seed", list(range(100, 112)))
def test_random_configurations(seed):
    """Seeded sweep over head layouts, sizes, schedules and decoding rules (whole generations,
    teacher forced)."""
    c = _random_case(seed)
    d = max(256, c["hq"] * c["hd"])
    cfg = small_cfg(c["dtype"], c["hq"], c["hkv"], c["hd"], d=d, scale=c["scale"])
    w = ec_inputs.make_weights(cfg, seed, gain_jitter=0.1)
    tau = c["tau"] if c["metric"] != 2 else min(c["tau"], 0.5)
    dec = ec_inputs.DecodeCfg(gen_len=c["N"], block=c["block"], k_recent=c["k"],
                              tokens_per_step=c["n"], tau=tau, conf_threshold=c["thr"],
                              gate_metric=c["metric"], schedule=c["schedule"])
    prompt = ec_inputs.make_prompt(cfg.vocab, c["P"], seed + 1)
    s = run_teacher_forced(cfg, w, dec, prompt, TOL[c["dtype"]], max_steps=40)
    print(c, s)
    assert s["tokens_exact"] > 0


def test_largest_batch():
    """EC_MAX_BATCH sequences with ragged prompts, every one against its own oracle run."""
    cfg = small_cfg("bf16", 4, 2, 64, scale=13.0)
    w = ec_inputs.make_weights(cfg, 41, gain_jitter=0.1)
    B = ec.EC_MAX_BATCH
    dec = ec_inputs.DecodeCfg(gen_len=12, block=8, k_recent=2, tokens_per_step=2, tau=2.5, batch=B)
    prompts = [ec_inputs.make_prompt(cfg.vocab, 1 + (7 * b) % 23, 300 + b) for b in range(B)]
    s = run_teacher_forced_batch(cfg, w, dec, prompts, TOL["bf16"], check_cache_every=3)
    print(s)
    assert s["steps"] == 6 and s["modes"][eco.FULL] >= B
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0 and s["modes_exact"] > 0


def test_many_few_row_sequences_one_attention_block_per_sequence_and_head():
    """32 ragged sequences x 8 heads whose partial steps recompute up to 36 rows each: the row
    list packs them back to back (a 16-row tile holds rows of two or three sequences), and the
    batch is large enough that the attention serves all row tiles of a (sequence, head) from one
    block that reads the sequence's K/V once.  Every sequence against its own oracle run."""
    cfg = small_cfg("bf16", 8, 4, 64, scale=13.0)
    w = ec_inputs.make_weights(cfg, 59, gain_jitter=0.1)
    B = 32
    dec = ec_inputs.DecodeCfg(gen_len=40, block=32, k_recent=4, tokens_per_step=2, tau=1e9, batch=B)
    prompts = [ec_inputs.make_prompt(cfg.vocab, 5 + (11 * b) % 57, 500 + b) for b in range(B)]
    s = run_teacher_forced_batch(cfg, w, dec, prompts, TOL["bf16"], max_steps=7, check_cache_every=3)
    print(s)
    assert s["modes"][eco.PARTIAL] == 6 * B and s["tokens_exact"] > 0


def test_batched_generate_runs_every_sequence_to_the_end():
    """ec_generate on a batch: free-running, sequences in different modes side by side; every
    generation slot ends up decoded, the counters add up, and a reset reproduces the run."""
    cfg = small_cfg("bf16", 4, 2, 64, scale=13.0)
    w = ec_inputs.make_weights(cfg, 31, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=48, block=16, k_recent=2, tokens_per_step=2, tau=2.5, batch=3)
    prompts = [ec_inputs.make_prompt(cfg.vocab, P, 50 + i) for i, P in enumerate((30, 5, 64))]
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), dec, prompts)
    try:
        toks, stats = g.generate()
        assert toks.shape == (3, 48) and stats["tokens"] == 3 * 48 and stats["steps"] == 24
        assert stats["full_steps"] + stats["partial_steps"] == 3 * 24 and stats["full_steps"] >= 3
        for b in range(3):
            assert not g.debug_read(ec.EC_DBG_MASKED, seq=b).any()
            assert np.array_equal(g.debug_read(ec.EC_DBG_X, seq=b)[len(prompts[b]):], toks[b])
        g.reset(prompts)
        toks2, stats2 = g.generate()
        assert np.array_equal(toks, toks2) and stats2["full_steps"] == stats["full_steps"]
    finally:
        g.close()


def test_recompute_ratio_counter():
    """RR = rows recomputed / (steps x T), the fraction of KV states recomputed per step: 1 when
    the threshold lies below every entropy (all steps FULL); with a threshold nothing exceeds it
    is one FULL step plus |M u R| <= block + k rows per step, and equals the oracle's count."""
    cfg = small_cfg("f32", 4, 2, 64)
    w = ec_inputs.make_weights(cfg, 67, gain_jitter=0.1)
    prompt = ec_inputs.make_prompt(cfg.vocab, 40, 13)
    dw = ec.weights_to_device(cfg, w)
    T, N, block, k = 40 + 32, 32, 8, 2
    for tau in (-1.0, 1e9):
        dec = ec_inputs.DecodeCfg(gen_len=N, block=block, k_recent=k, tokens_per_step=1, tau=tau)
        g = ec.EntropyCache(cfg, dw, dec, prompt)
        try:
            _, stats = g.generate()
        finally:
            g.close()
        assert stats["steps"] == N
        rr = stats["rows_recomputed"] / (stats["steps"] * T)
        if tau < 0:
            assert stats["full_steps"] == N and rr == 1.0
        else:
            assert stats["full_steps"] == 1 and stats["partial_steps"] == N - 1
            rows_oracle = sum(len(r["S"]) for r in eco.eco_generate(
                eco.eco_init(eco.OracleModel(cfg, w), dec, prompt)))
            assert stats["rows_recomputed"] == rows_oracle
            assert T < stats["rows_recomputed"] <= T + (N - 1) * (block + k)
            assert rr < 0.25


@pytest.mark.parametrize("dtype,P,N,block,k,n,tau", [
    ("f32", 0, 20, 8, 2, 1, 2.5),          # no prompt at all
    ("bf16", 3, 40, 128, 100, 32, 1e9),    # largest block and tokens per step, k beyond the generation
    ("f32", 9, 12, 4, 1, 1, -1.0),         # threshold below any entropy: every step FULL
    ("bf16", 17, 33, 1, 0, 1, 1e9),        # block of one: strictly left to right, no recent rows
])
def test_degenerate_shapes(dtype, P, N, block, k, n, tau):
    cfg = small_cfg(dtype, 4, 2, 64)
    w = ec_inputs.make_weights(cfg, 23, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=N, block=block, k_recent=k, tokens_per_step=n, tau=tau)
    prompt = ec_inputs.make_prompt(cfg.vocab, P, 4)
    s = run_teacher_forced(cfg, w, dec, prompt, TOL[dtype])
    print(s)
    assert s["tokens_exact"] > 0 and s["rows_decided"] > 0
    if tau < 0:
        assert s["modes"][eco.PARTIAL] == 0


def test_largest_context_properties():
    """15000 positions (the largest context the library accepts) on a small model, where the
    oracle is too slow: properties that hold at any size.  A second FULL step with nothing
    committed in between is idempotent (same logits, same cache); a PARTIAL step after it sees an
    exact cache and reproduces those logits on the block rows."""
    cfg = small_cfg("bf16", 4, 2, 64)
    w = ec_inputs.make_weights(cfg, 29, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=200, block=32, k_recent=2, tokens_per_step=1, tau=1.0)
    prompt = ec_inputs.make_prompt(cfg.vocab, 14800, 6)
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), dec, prompt)
    g.keep_logits(True)
    try:
        r1 = g.step_forced(ec.EC_FULL, [], [])
        z1 = g.debug_read(ec.EC_DBG_LOGITS, count=32)
        k1 = g.debug_read(ec.EC_DBG_KCACHE, 1)
        r2 = g.step_forced(ec.EC_FULL, [], [])
        z2 = g.debug_read(ec.EC_DBG_LOGITS, count=32)
        k2 = g.debug_read(ec.EC_DBG_KCACHE, 1)
        assert r1["n_query_rows"] == r2["n_query_rows"] == 15000
        assert np.array_equal(z1, z2) and np.array_equal(k1, k2)      # same kernels, same inputs
        assert np.isfinite(z1).all() and float(np.abs(z1).max()) > 0
        r3 = g.step_forced(ec.EC_PARTIAL, [], [])
        z3 = g.debug_read(ec.EC_DBG_LOGITS, count=32)
        assert r3["n_query_rows"] == 32
        assert relerr(z3, z1) <= TOL["bf16"]
        # the partial step rewrote the block rows' K/V from the same inputs
        assert relerr(ec_bits(g.debug_read(ec.EC_DBG_KCACHE, 1)), ec_bits(k1)) <= TOL["bf16"]
    finally:
        g.close()


def ec_bits(a):
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32) if a.dtype == np.uint16 else a


def test_free_running_generation_matches_oracle_f32():
    """Without forcing: the GPU's own decisions reproduce the oracle's generation (float32 model,
    margins far above 1e-4 at every step of this seed)."""
    wl = ec_inputs.WORKLOADS["tiny_f32"]
    cfg = wl.model.replace(logit_scale=16.0)
    w = ec_inputs.make_weights(cfg, wl.seed)
    prompt = ec_inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed)
    st = eco.eco_init(eco.OracleModel(cfg, w), wl.decode, prompt)
    trace = eco.eco_generate(st)
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), wl.decode, prompt)
    toks, stats = g.generate()
    assert stats["steps"] == len(trace) and stats["full_steps"] == st.n_full
    assert stats["rows_recomputed"] == st.rows_recomputed
    assert np.array_equal(toks, st.x[st.P:].astype(np.int32))
    # reset and step by step: same sequence of modes, positions, tokens, entropies
    g.reset(prompt)
    for r in trace:
        q = g.step(ec.EC_AUTO)
        assert q["mode_run"] == r["mode"] and q["positions"] == r["positions"]
        assert q["tokens"] == r["tokens"]
        assert abs(q["max_entropy"] - r["E"]) < 1e-3
    g.close()


def test_state_errors_and_forced_mode_schedule():
    cfg = small_cfg("f32")
    w = ec_inputs.make_weights(cfg, 5)
    dec = ec_inputs.DecodeCfg(gen_len=8, block=4, k_recent=2, tokens_per_step=1, tau=1e9)
    prompt = ec_inputs.make_prompt(cfg.vocab, 6, 1)
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), dec, prompt)
    with pytest.raises(ec.EcError) as e:
        g.step(ec.EC_PARTIAL)
    assert e.value.code == ec.EC_ERR_STATE
    with pytest.raises(ec.EcError) as e:
        g.step_forced(ec.EC_FULL, [2], [1])            # a prompt position is not a masked slot
    assert e.value.code == ec.EC_ERR_ARG
    # forced all-FULL schedule vs oracle forced the same way
    st = eco.eco_init(eco.OracleModel(cfg, w), dec, prompt)
    for i in range(8):
        r = eco.eco_step(st, eco.FULL)
        q = g.step_forced(ec.EC_FULL, r["positions"], r["tokens"])
        assert q["n_query_rows"] == st.T
        assert relerr(g.debug_read(ec.EC_DBG_LOGITS, count=len(r["Mb"])), r["logits"]) < 1e-4
    assert q["done"]
    with pytest.raises(ec.EcError) as e:
        g.step(ec.EC_AUTO)
    assert e.value.code == ec.EC_ERR_STATE
    g.close()


def test_entropy_closed_forms_through_the_whole_path():
    """Zero LM head -> uniform logits: H = ln V, confidence 1/V, token 0 (lowest id on ties),
    most confident row = lowest position.  One dominant LM-head row -> H ~ 0, confidence ~ 1."""
    cfg = small_cfg("f32", scale=1.0)
    w = ec_inputs.make_weights(cfg, 9)
    dec = ec_inputs.DecodeCfg(gen_len=8, block=8, k_recent=2, tokens_per_step=2, tau=1.0)
    prompt = ec_inputs.make_prompt(cfg.vocab, 10, 2)
    w0 = dict(w); w0["lm_head"] = np.zeros_like(w["lm_head"])
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w0), dec, prompt)
    q = g.step(ec.EC_AUTO)
    assert q["positions"] == [10, 11] and q["tokens"] == [0, 0]
    assert q["max_entropy"] == pytest.approx(math.log(cfg.vocab), rel=1e-6)
    assert q["confidence"][0] == pytest.approx(1.0 / cfg.vocab, rel=1e-6)
    assert q["next_mode"] == ec.EC_FULL
    g.close()
    # dominant row: lm_head[77] = 1000 * (direction every final hidden state has a positive
    # component along): use the final norm's output sign trick by making all other rows zero and
    # row 77 and 78 equal -> exactly two equal maxima -> H = ln 2 when they dominate
    w1 = dict(w)
    lm = np.zeros_like(w["lm_head"])
    w1["lm_head"] = lm
    st = eco.eco_init(eco.OracleModel(cfg, w), dec, prompt)
    hfin = eco.forward_rows(st, np.arange(st.T), eco.current_block_masked(st))
    lm[77] = lm[78] = (200.0 * hfin[0] / np.linalg.norm(hfin[0]) ** 2).astype(np.float32)
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w1), dec, prompt)
    q = g.step(ec.EC_AUTO)
    stats = g.debug_read(ec.EC_DBG_ROW_STATS, count=8)
    assert int(stats[0, 0]) == 77                      # lowest id among the equal maxima
    assert stats[0, 2] == pytest.approx(math.log(2.0), rel=1e-4)
    assert stats[0, 1] == pytest.approx(0.5, rel=1e-4)
    g.close()


def test_large_magnitude_residual_stream():
    """Residual rows with sums of squares near 1e10 (embeddings of magnitude ~6000, as the
    massive activations of trained models): the fixed-point row sums behind the folded RMSNorm
    must neither wrap nor lose the row."""
    from tests.gpu_harness import bf16_bits_to_f32
    cfg = small_cfg("bf16", 4, 2, 64)
    w = ec_inputs.make_weights(cfg, 43, gain_jitter=0.1)
    w["tok_emb"] = ec_inputs.f32_to_bf16_bits(bf16_bits_to_f32(w["tok_emb"]) * np.float32(3e5))
    dec = ec_inputs.DecodeCfg(gen_len=40, block=32, k_recent=2, tokens_per_step=2, tau=1e9)
    prompt = ec_inputs.make_prompt(cfg.vocab, 150, 8)
    s = run_teacher_forced(cfg, w, dec, prompt, TOL["bf16"])
    print(s)
    assert s["modes"][eco.PARTIAL] >= 1 and s["rows_decided"] > 0 and s["modes_exact"] > 0


def test_long_context_ragged_batch_gqa():
    """Two sequences of more than 2048 positions with grouped-query heads of 128: the key slices
    of the partial-step attention (pieces summed by the last block to arrive) on a ragged batch."""
    cfg = small_cfg("bf16", 4, 2, 128, d=512)
    w = ec_inputs.make_weights(cfg, 47, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=24, block=16, k_recent=3, tokens_per_step=2, tau=1e9, batch=2)
    prompts = [ec_inputs.make_prompt(cfg.vocab, P, 60 + i) for i, P in enumerate((2100, 2333))]
    s = run_teacher_forced_batch(cfg, w, dec, prompts, TOL["bf16"], max_steps=6, check_cache_every=3)
    print(s)
    assert s["modes"][eco.PARTIAL] >= 8 and s["tokens_exact"] > 0


def test_logits_stay_out_of_memory_unless_asked_for():
    """The bfloat16 path reduces the vocabulary inside the LM-head kernel: by default a step
    leaves no logits behind (reading them is a state error), and switching the store on changes
    nothing else - same tokens, same statistics, bit for bit."""
    cfg = small_cfg("bf16", 4, 2, 64, scale=13.0)
    w = ec_inputs.make_weights(cfg, 53, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=48, block=16, k_recent=2, tokens_per_step=2, tau=2.5)
    prompt = ec_inputs.make_prompt(cfg.vocab, 30, 12)
    dw = ec.weights_to_device(cfg, w)
    runs = []
    for keep in (False, True):
        g = ec.EntropyCache(cfg, dw, dec, prompt)
        g.keep_logits(keep)
        trace = []
        while True:
            q = g.step(ec.EC_AUTO)
            stats = g.debug_read(ec.EC_DBG_ROW_STATS, count=q["n_block_rows"])
            trace.append((q, stats.copy()))
            if keep:
                z = g.debug_read(ec.EC_DBG_LOGITS, count=q["n_block_rows"])
                assert np.array_equal(z.max(axis=1), stats[:, 3])
            else:
                with pytest.raises(ec.EcError) as e:
                    g.debug_read(ec.EC_DBG_LOGITS, count=1)
                assert e.value.code == ec.EC_ERR_STATE
            if q["done"]:
                break
        runs.append(trace)
        g.close()
    assert len(runs[0]) == len(runs[1])
    for (qa, sa), (qb, sb) in zip(*runs):
        assert qa == qb and np.array_equal(sa, sb)


@pytest.mark.parametrize("hq,hkv,hd,P,N,block,k,n,tau,f", [
    (4, 4, 64, 64, 64, 32, 2, 1, 3.0, 768),
    (4, 2, 128, 50, 70, 32, 4, 2, 2.5, 1280),    # GQA, head_dim 128, ragged last block
    (8, 2, 64, 100, 33, 32, 2, 3, 1e9, 768),     # 133 rows in FULL steps: tiled kernels + scales
    (4, 2, 64, 40, 128, 32, 64, 1, 1e9, 6208),   # up to 96 rows; 776 gate/up tiles in groups of 3
])
def test_e4m3_weight_models_whole_generation(hq, hkv, hd, P, N, block, k, n, tau, f):
    """Matrices stored as e4m3 codes with per-row scales (EC_FP8W): partial steps stream the
    codes and widen them in registers, full steps run on their exact bf16 expansion; both apply
    the row scales to the sums.  The oracle decodes the same codes exactly."""
    cfg = small_cfg("fp8w", hq, hkv, hd, d=hq * hd if hq * hd >= 256 else 256, f=f)
    w = ec_inputs.make_weights(cfg, 7, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=N, block=block, k_recent=k, tokens_per_step=n, tau=tau)
    prompt = ec_inputs.make_prompt(cfg.vocab, P, 3)
    s = run_teacher_forced(cfg, w, dec, prompt, TOL["fp8w"])
    print(s)
    assert s["modes"][eco.PARTIAL] >= 1 and s["tokens_exact"] > 0 and s["modes_exact"] > 0


def test_e4m3_weight_batch():
    cfg = small_cfg("fp8w", 4, 2, 128, d=512)
    w = ec_inputs.make_weights(cfg, 13, gain_jitter=0.1)
    dec = ec_inputs.DecodeCfg(gen_len=36, block=32, k_recent=3, tokens_per_step=1, tau=2.5, batch=4)
    prompts = [ec_inputs.make_prompt(cfg.vocab, P, 20 + i) for i, P in enumerate((70, 9, 33, 150))]
    s = run_teacher_forced_batch(cfg, w, dec, prompts, TOL["fp8w"], max_steps=12)
    print(s)
    assert s["modes"][eco.PARTIAL] >= 1 and s["tokens_exact"] > 0


@pytest.mark.parametrize("dtype,batch", [("bf16", 1), ("f32", 1), ("bf16", 3)])
def test_rows_of_nan_logits_are_reported_and_nothing_leaves_its_buffers(dtype, batch):
    """A model whose final norm gain is NaN: every logit is NaN, so no row has a maximum.  The
    step must say so (EC_ERR_NONFINITE), the rows take token 0 (a row's token indexes the
    embedding table at the next step), further steps and a generation run to their end the same
    way, and a healthy context next to it is unaffected."""
    cfg = small_cfg(dtype, 4, 2, 64)
    good = ec_inputs.make_weights(cfg, 61, gain_jitter=0.1)
    bad = dict(good)
    bad["final_norm"] = good["final_norm"].copy()
    if dtype == "f32":
        bad["final_norm"][:] = np.nan
    else:
        bad["final_norm"][:] = 0x7FC0          # a bfloat16 NaN
    dec = ec_inputs.DecodeCfg(gen_len=24, block=8, k_recent=2, tokens_per_step=2, tau=2.5, batch=batch)
    prompts = [ec_inputs.make_prompt(cfg.vocab, 9 + 5 * b, 70 + b) for b in range(batch)]
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, bad), dec, prompts if batch > 1 else prompts[0])
    for mode in (ec.EC_AUTO, ec.EC_AUTO, ec.EC_PARTIAL, ec.EC_FULL):
        with pytest.raises(ec.EcError) as e:
            g.step(mode)
        assert e.value.code == ec.EC_ERR_NONFINITE
        x = g.debug_read(ec.EC_DBG_X)
        assert x.min() >= 0 and x.max() < cfg.vocab
    stats = g.debug_read(ec.EC_DBG_ROW_STATS, count=1)
    assert stats[0, 0] == 0 and stats[0, 1] == 0 and np.isinf(stats[0, 2])
    with pytest.raises(ec.EcError) as e:
        g.generate()
    assert e.value.code == ec.EC_ERR_NONFINITE
    g.close()
    # the same shapes with finite weights still match the oracle
    s = (run_teacher_forced(cfg, good, dec, prompts[0], TOL[dtype], max_steps=4) if batch == 1 else
         run_teacher_forced_batch(cfg, good, dec, prompts, TOL[dtype], max_steps=4))
    assert s["steps"] == 4
