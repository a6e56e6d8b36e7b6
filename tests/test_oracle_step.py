"""Pins of the oracle's step: full step == dense cache-free forward, partial-step invariants,
staleness semantics, schedule properties (no GPU).  Passages: appendix "Full EntropyCache
algorithm" (prefill branch, partial branch), Method section on recent-token recomputation."""
import math

import numpy as np
import pytest

import ec_inputs
from oracle import entropycache as eco
from tests.dense_reference import dense_forward


def small_model(dtype="f32", hq=4, hkv=2, seed=11, vocab=97, layers=2, gain_jitter=0.2):
    cfg = ec_inputs.ModelCfg(n_layers=layers, d_model=32, n_heads=hq, n_kv_heads=hkv, head_dim=8,
                             d_ffn=48, vocab=vocab, mask_id=vocab - 1, rms_eps=1e-5,
                             rope_base=10000.0, logit_scale=1.0, dtype=dtype)
    # std 0.3: far from the near-linear regime of N(0,0.02) so every non-linearity matters
    w = ec_inputs.make_weights(cfg, seed, std=0.3, gain_jitter=gain_jitter, threads=1)
    return eco.OracleModel(cfg, w)


def new_state(model, P=6, N=8, block=4, k=2, n=1, tau=1.0, seed=5):
    dec = ec_inputs.DecodeCfg(gen_len=N, block=block, k_recent=k, tokens_per_step=n, tau=tau)
    prompt = ec_inputs.make_prompt(model.cfg.vocab + 96, P, seed) % (model.cfg.vocab - 1)
    return eco.eco_init(model, dec, prompt.astype(np.int32))


@pytest.mark.parametrize("dtype,hq,hkv", [("f32", 4, 2), ("f32", 2, 2), ("bf16", 4, 1)])
def test_full_step_equals_dense_forward(dtype, hq, hkv):
    m = small_model(dtype, hq, hkv)
    st = new_state(m)
    x0 = st.x.copy()
    r = eco.eco_step(st, eco.FULL)
    hf, logits, K, V = dense_forward(m.cfg, m.w, x0)
    assert np.allclose(st.Kc, K, rtol=1e-10, atol=1e-12)
    assert np.allclose(st.Vc, V, rtol=1e-10, atol=1e-12)
    assert np.allclose(r["logits"], logits[r["Mb"]], rtol=1e-9, atol=1e-11)
    # decode: most confident row of the block, argmax token, its entropy
    import scipy.special
    p = scipy.special.softmax(logits[r["Mb"]], axis=-1)
    best = int(np.argmax(p.max(-1)))
    assert r["positions"] == [int(r["Mb"][best])]
    assert r["tokens"] == [int(np.argmax(p[best]))]
    assert r["E"] == pytest.approx(float(scipy.special.entr(p[best]).sum()), rel=1e-10)


def test_logit_scale_multiplies_logits():
    m = small_model()
    m2 = eco.OracleModel(m.cfg.replace(logit_scale=2.5), m.w)
    a = eco.eco_step(new_state(m), eco.FULL)
    b = eco.eco_step(new_state(m2), eco.FULL)
    assert np.allclose(b["logits"], 2.5 * a["logits"], rtol=1e-13)


def test_second_full_after_decode_equals_dense_of_new_x():
    m = small_model()
    st = new_state(m)
    eco.eco_step(st, eco.FULL)
    x1 = st.x.copy()
    r = eco.eco_step(st, eco.FULL)
    _, logits, K, V = dense_forward(m.cfg, m.w, x1)
    assert np.allclose(st.Kc, K, rtol=1e-10, atol=1e-12)
    assert np.allclose(r["logits"], logits[r["Mb"]], rtol=1e-9, atol=1e-11)


def test_partial_with_all_rows_is_full_bit_for_bit():
    m = small_model()
    a, b = new_state(m), new_state(m)
    for s in (a, b):
        eco.eco_step(s, eco.FULL)
    ra = eco.eco_step(a, eco.FULL)
    rb = eco.eco_step(b, eco.PARTIAL, rows_override=np.arange(b.T))
    assert np.array_equal(ra["logits"], rb["logits"])
    assert np.array_equal(a.Kc, b.Kc) and np.array_equal(a.Vc, b.Vc)
    assert ra["positions"] == rb["positions"] and ra["E"] == rb["E"]


def test_partial_with_no_rows_leaves_cache_unchanged():
    m = small_model()
    st = new_state(m)
    eco.eco_step(st, eco.FULL)
    K0, V0, x0 = st.Kc.copy(), st.Vc.copy(), st.x.copy()
    eco.eco_step(st, eco.PARTIAL, rows_override=np.array([], dtype=np.int64))
    assert np.array_equal(st.Kc, K0) and np.array_equal(st.Vc, V0) and np.array_equal(st.x, x0)


def test_partial_touches_only_its_rows_and_layer0_is_exact():
    m = small_model(layers=3)
    st = new_state(m, k=2, tau=1e9)                     # never triggers a full recompute
    eco.eco_step(st, eco.AUTO)                          # t=1 is FULL
    K_before, V_before = st.Kc.copy(), st.Vc.copy()
    x_before = st.x.copy()
    r = eco.eco_step(st, eco.AUTO)
    assert r["mode"] == eco.PARTIAL
    S = r["S"]
    notS = np.setdiff1d(np.arange(st.T), S)
    # rows outside S are bit-untouched in every layer (stale by design)
    assert np.array_equal(st.Kc[:, notS], K_before[:, notS])
    assert np.array_equal(st.Vc[:, notS], V_before[:, notS])
    # layer-0 K/V depend only on x[j] and j, so for j in S they equal the dense values for the
    # x this step ran on: pins that current embeddings and absolute positions were used
    _, _, K, V = dense_forward(m.cfg, m.w, x_before)
    assert np.allclose(st.Kc[0, S], K[0, S], rtol=1e-10, atol=1e-12)
    assert np.allclose(st.Vc[0, S], V[0, S], rtol=1e-10, atol=1e-12)
    # the token decoded at step 1 is in S (it is "recent") and its layer-0 K changed
    dec1 = [p for p in range(st.P, st.T) if st.hist[p - st.P] == 1][0]
    assert dec1 in S
    assert not np.allclose(st.Kc[0, dec1], K_before[0, dec1])
    # layer-1 K/V of rows in S are still exact: layer-0 K/V of every position depend on x alone
    # and x changed only inside S, so the layer-0 context these rows attended was exact
    assert np.allclose(st.Kc[1, S], K[1, S], rtol=1e-10, atol=1e-12)
    # but layer-1 rows outside S are stale, and from layer 2 on so is what rows in S compute
    assert not np.allclose(st.Kc[1, notS], K[1, notS], rtol=1e-6)
    assert not np.allclose(st.Kc[2, S], K[2, S], rtol=1e-6)


def test_partial_on_unchanged_x_reproduces_full():
    """FULL, then recompute the block rows again without having changed x (forced commit of the
    same token that is already there): logits and K/V of those rows equal the FULL values."""
    m = small_model()
    st = new_state(m)
    r1 = eco.eco_step(st, eco.FULL, forced={"positions": [], "tokens": []})
    assert st.masked[st.P:].all()                        # nothing was committed
    K1, V1 = st.Kc.copy(), st.Vc.copy()
    r2 = eco.eco_step(st, eco.PARTIAL, forced={"positions": [], "tokens": []})
    assert list(r2["S"]) == list(r1["Mb"])               # block rows only, no recent tokens yet
    assert np.allclose(r2["logits"], r1["logits"], rtol=1e-11, atol=1e-13)
    assert np.allclose(st.Kc, K1, rtol=1e-11, atol=1e-13)
    assert np.allclose(st.Vc, V1, rtol=1e-11, atol=1e-13)


def test_partial_before_full_is_an_error_and_step_after_done_too():
    m = small_model()
    st = new_state(m)
    with pytest.raises(RuntimeError):
        eco.eco_step(st, eco.PARTIAL)
    eco.eco_generate(st)
    with pytest.raises(RuntimeError):
        eco.eco_step(st)


@pytest.mark.parametrize("n,k,tau", [(1, 2, 1.0), (2, 2, 3.0), (1, 3, 1e9), (3, 1, -1.0)])
def test_schedule_properties(n, k, tau):
    m = small_model()
    N, w = 12, 4
    st = new_state(m, P=5, N=N, block=w, k=k, n=n, tau=tau)
    trace = eco.eco_generate(st)
    # termination in exactly ceil(w/n) * N/w steps; every slot decoded exactly once
    assert len(trace) == math.ceil(w / n) * (N // w)
    assert sorted(p for r in trace for p in r["positions"]) == list(range(st.P, st.T))
    lastfull = 0
    for i, r in enumerate(trace):
        t = i + 1
        assert r["t"] == t
        if r["mode"] == eco.FULL:
            lastfull = t
            assert len(r["S"]) == st.T
        else:
            assert len(r["S"]) <= w + k + (n - 1)        # ties of one step may exceed k by n-1
            assert set(r["Mb"]).issubset(set(r["S"]))
        assert r["dt_eff"] == t - lastfull               # paper's counter == t - last full step
        # mode follows the previous step's flag; first step is full
        assert r["mode"] == (eco.FULL if i == 0 or trace[i - 1]["E"] > tau else eco.PARTIAL)
        assert r["skip"] == (r["E"] <= tau)
        # R: decoded at or after the last full step, never more than k (+ ties)
        for p in r["R"]:
            assert st.hist[p - st.P] >= lastfull and st.hist[p - st.P] <= t
        if n == 1:
            assert len(r["R"]) <= k
        # Mb lies inside one block
        assert (r["Mb"] - st.P).min() // w == (r["Mb"] - st.P).max() // w
        assert 0.0 <= r["E"] <= math.log(m.cfg.vocab) + 1e-9
    rr = eco.recompute_ratio(st)
    if tau < 0:
        assert rr == 1.0 and st.n_full == len(trace)
    if tau > 1e8:
        assert st.n_full == 1
        assert rr == pytest.approx(sum(len(r["S"]) for r in trace) / (len(trace) * st.T))
        assert rr < 0.5


def test_forced_commit_and_mode_override():
    m = small_model()
    a = new_state(m, tau=1e9)
    tr = eco.eco_generate(a, keep_logits=True)
    b = new_state(m, tau=-5.0)                            # would always go FULL on its own
    for r in tr:
        rb = eco.eco_step(b, r["mode"], forced={"positions": r["positions"], "tokens": r["tokens"]})
        assert rb["mode"] == r["mode"] and list(rb["S"]) == list(r["S"])
        assert np.array_equal(rb["logits"], r["logits"])
        assert rb["own_positions"] == r["own_positions"] and rb["own_tokens"] == r["own_tokens"]
    assert np.array_equal(a.x, b.x) and np.array_equal(a.Kc, b.Kc)


def test_ragged_last_block_and_mask_id_can_be_decoded():
    m = small_model()
    st = new_state(m, P=3, N=10, block=4)                # blocks 4,4,2
    tr = eco.eco_generate(st)
    assert len(tr) == 10 and st.done
    # masked-ness is the explicit set, not x == mask_id: force-decode the mask id itself
    st2 = new_state(m, P=3, N=4, block=4)
    r = eco.eco_step(st2, eco.FULL, forced={"positions": [3], "tokens": [m.cfg.mask_id]})
    assert st2.x[3] == m.cfg.mask_id and not st2.masked[3] and 3 not in eco.current_block_masked(st2)
