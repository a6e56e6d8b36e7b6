"""Teacher-forced comparison of the HIP path with the CPU oracle on the same seeded inputs.
The oracle's decisions (mode, committed positions / tokens) drive both sides, because the method
keeps a stale cache by design and a single different decision would make the two runs diverge
without either being wrong."""
import numpy as np

import paper_2603_18489_amd as ec
from oracle import entropycache as eco


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32)


def relerr(a, b):
    """max |a-b| / max |b| over the tensor."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if b.size == 0:
        return 0.0
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def gpu_cache(g, which, layer):
    c = g.debug_read(which, layer)
    return bf16_bits_to_f32(c) if c.dtype == np.uint16 else c


def run_teacher_forced(cfg, w, dec, prompt, tol, max_steps=None, check_cache_every=1,
                       dev_weights=None, verbose=False, mode_fn=None, cache_layers=None):
    """Runs the oracle free (AUTO, or with the modes mode_fn(step_index) forces on both sides)
    and the GPU teacher-forced by it.  Returns a summary dict; raises AssertionError on any
    parity violation."""
    st = eco.eco_init(eco.OracleModel(cfg, w), dec, prompt)
    dw = dev_weights if dev_weights is not None else ec.weights_to_device(cfg, w)
    g = ec.EntropyCache(cfg, dw, dec, prompt)
    worst = {"logits": 0.0, "K": 0.0, "V": 0.0, "H": 0.0, "conf": 0.0}
    n_exact_checked = 0
    modes = {eco.FULL: 0, eco.PARTIAL: 0}
    steps = 0
    try:
        while not st.done and (max_steps is None or steps < max_steps):
            # the row set the GPU built for a partial step must be the oracle's M u R
            Mb = eco.current_block_masked(st)
            exp_rows = sorted(set(Mb.tolist()) | set(st.R))
            if steps > 0:
                rows = g.debug_read(ec.EC_DBG_ROWS, count=len(exp_rows))
                assert rows.tolist() == exp_rows, f"step {st.t}: row set differs"
            r = eco.eco_step(st, eco.AUTO if mode_fn is None else mode_fn(steps))
            q = g.step_forced(r["mode"], r["positions"], r["tokens"])
            steps += 1
            modes[r["mode"]] += 1
            nmb = len(r["Mb"])
            assert q["mode_run"] == r["mode"] and q["n_query_rows"] == len(r["S"])
            assert q["n_block_rows"] == nmb and q["step_index"] == r["t"]
            assert q["done"] == r["done"] and q["n_recent_next"] == len(r["R"])
            logits = g.debug_read(ec.EC_DBG_LOGITS, count=nmb)
            e = relerr(logits, r["logits"])
            worst["logits"] = max(worst["logits"], e)
            assert e <= tol, f"step {r['t']} mode {r['mode']}: logits rel err {e:.3e} > {tol}"
            stats = g.debug_read(ec.EC_DBG_ROW_STATS, count=nmb)
            lnV = np.log(cfg.vocab)
            eH = float(np.abs(stats[:, 2] - r["H"]).max() / lnV)
            eC = float(np.abs(stats[:, 1] - r["conf"]).max() / max(r["conf"].max(), 1e-30))
            worst["H"] = max(worst["H"], eH)
            worst["conf"] = max(worst["conf"], eC)
            # entropy / confidence inherit the logits' error, amplified by the logit range
            zrange = float(np.ptp(r["logits"]))
            stat_tol = max(tol, 4 * tol * max(zrange, 1.0)) if cfg.dtype == "bf16" else 2 * tol
            assert eH <= stat_tol, f"step {r['t']}: entropy err {eH:.3e} > {stat_tol:.3e}"
            assert eC <= stat_tol, f"step {r['t']}: confidence err {eC:.3e}"
            # decisions: bit-exact wherever the oracle's margins exceed the tolerance
            z = r["logits"]
            abs_tol = tol * np.abs(z).max()
            srt = np.sort(z, axis=1)
            top2gap = srt[:, -1] - srt[:, -2]
            for i in range(nmb):
                if top2gap[i] > 4 * abs_tol:
                    assert int(stats[i, 0]) == int(r["tok"][i]), f"step {r['t']} row {i}: argmax"
            csort = np.sort(r["conf"])[::-1]
            n = len(r["own_positions"])
            conf_margin_ok = (n >= nmb) or (csort[n - 1] - csort[n] > 8 * stat_tol * csort[n - 1])
            if n > 1:
                conf_margin_ok = conf_margin_ok and bool(
                    np.all(csort[:n - 1] - csort[1:n] > 8 * stat_tol * csort[:n - 1]))
            thr = getattr(dec, "conf_threshold", 0.0)
            if thr > 0:   # the number of tokens depends on which side of the threshold rows fall
                conf_margin_ok = conf_margin_ok and bool(
                    np.all(np.abs(r["conf"] - thr) > 8 * stat_tol * np.maximum(r["conf"], thr)))
            chosen_rows = [int(np.where(r["Mb"] == p)[0][0]) for p in r["own_positions"]]
            if conf_margin_ok and all(top2gap[i] > 4 * abs_tol for i in chosen_rows):
                assert q["positions"] == r["own_positions"], f"step {r['t']}: positions"
                assert q["tokens"] == r["own_tokens"], f"step {r['t']}: tokens"
                n_exact_checked += 1
                if abs(r["E_own"] - dec.tau) > 2 * stat_tol * lnV * max(1, len(r["own_positions"])):
                    skips = eco.gate_skips(r["E_own"], dec.tau, getattr(dec, "gate_metric", 0))
                    assert q["next_mode"] == (eco.PARTIAL if skips else eco.FULL)
                    assert abs(q["max_entropy"] - r["E_own"]) <= 2 * stat_tol * lnV * len(r["own_positions"])
            if check_cache_every and (steps % check_cache_every == 0 or st.done):
                for l in (range(cfg.n_layers) if cache_layers is None else cache_layers):
                    for name, which, oc in (("K", ec.EC_DBG_KCACHE, st.Kc), ("V", ec.EC_DBG_VCACHE, st.Vc)):
                        e = relerr(gpu_cache(g, which, l), oc[l])
                        worst[name] = max(worst[name], e)
                        assert e <= tol, f"step {r['t']} layer {l}: {name} cache rel err {e:.3e}"
            if verbose:
                print(f"t={r['t']} mode={r['mode']} |S|={len(r['S'])} E={r['E']:.3f} "
                      f"logits={worst['logits']:.2e}", flush=True)
        # integer state is bit-exact
        assert np.array_equal(g.debug_read(ec.EC_DBG_X), st.x.astype(np.int32))
        assert np.array_equal(g.debug_read(ec.EC_DBG_MASKED).astype(bool), st.masked)
        hist = np.array([np.iinfo(np.int32).min if h == -np.inf else int(h) for h in st.hist],
                        dtype=np.int32)
        assert np.array_equal(g.debug_read(ec.EC_DBG_HIST), hist)
    finally:
        g.close()
    return {"steps": steps, "modes": modes, "worst": worst, "exact_checked": n_exact_checked}


def run_teacher_forced_batch(cfg, w, dec, prompts, tol, max_steps=None, fast_seq=None,
                             check_cache_every=4):
    """The batched HIP path against one oracle run per sequence (sequences are independent, so
    the batch must reproduce each of them).  fast_seq: that sequence commits every masked token
    of its block at each step (with the oracle's argmax tokens), so it finishes early while the
    others go on.  Returns a summary; raises AssertionError on any parity violation."""
    B = len(prompts)
    model = eco.OracleModel(cfg, w)
    sts = [eco.eco_init(model, dec, p) for p in prompts]
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), dec, prompts)
    worst = {"logits": 0.0, "K": 0.0, "V": 0.0}
    steps, modes = 0, {eco.FULL: 0, eco.PARTIAL: 0}
    finished_early = 0
    try:
        while not all(st.done for st in sts) and (max_steps is None or steps < max_steps):
            res = [None] * B
            for b, st in enumerate(sts):
                if st.done:
                    continue
                Mb = eco.current_block_masked(st)
                exp_rows = sorted(set(Mb.tolist()) | set(st.R))
                if steps > 0:
                    rows = g.debug_read(ec.EC_DBG_ROWS, count=len(exp_rows), seq=b)
                    assert rows.tolist() == exp_rows, f"seq {b} step {st.t}: row set differs"
                if b == fast_seq:
                    # look at the step's own tokens first, then commit the whole block
                    import copy
                    probe = eco.eco_step(copy.deepcopy(st), eco.AUTO)
                    forced = {"positions": [int(p) for p in probe["Mb"]],
                              "tokens": [int(v) for v in probe["tok"]]}
                    res[b] = eco.eco_step(st, probe["mode"], forced=forced)
                else:
                    res[b] = eco.eco_step(st, eco.AUTO)
            mlist = [r["mode"] if r else ec.EC_AUTO for r in res]
            plist = [r["positions"] if r else [] for r in res]
            tlist = [r["tokens"] if r else [] for r in res]
            q = g.step_forced_batch(mlist, plist, tlist)
            steps += 1
            for b, r in enumerate(res):
                if r is None:
                    assert q[b]["done"], f"seq {b}: finished sequence must report done"
                    finished_early += 1
                    continue
                modes[r["mode"]] += 1
                nmb = len(r["Mb"])
                assert q[b]["mode_run"] == r["mode"] and q[b]["n_query_rows"] == len(r["S"])
                assert q[b]["n_block_rows"] == nmb and q[b]["step_index"] == r["t"]
                assert q[b]["done"] == r["done"] and q[b]["n_recent_next"] == len(r["R"])
                logits = g.debug_read(ec.EC_DBG_LOGITS, count=nmb, seq=b)
                e = relerr(logits, r["logits"])
                worst["logits"] = max(worst["logits"], e)
                assert e <= tol, f"seq {b} step {r['t']} mode {r['mode']}: logits rel err {e:.3e}"
                stats = g.debug_read(ec.EC_DBG_ROW_STATS, count=nmb, seq=b)
                zrange = float(np.ptp(r["logits"]))
                stat_tol = max(tol, 4 * tol * max(zrange, 1.0))
                assert float(np.abs(stats[:, 2] - r["H"]).max() / np.log(cfg.vocab)) <= stat_tol
                if steps % check_cache_every == 0 or sts[b].done:
                    for l in range(cfg.n_layers):
                        for name, which, oc in (("K", ec.EC_DBG_KCACHE, sts[b].Kc),
                                                ("V", ec.EC_DBG_VCACHE, sts[b].Vc)):
                            c = g.debug_read(which, l, seq=b)
                            e = relerr(bf16_bits_to_f32(c) if c.dtype == np.uint16 else c, oc[l])
                            worst[name] = max(worst[name], e)
                            assert e <= tol, f"seq {b} step {r['t']} layer {l}: {name} cache {e:.3e}"
        for b, st in enumerate(sts):
            assert np.array_equal(g.debug_read(ec.EC_DBG_X, seq=b), st.x.astype(np.int32))
            assert np.array_equal(g.debug_read(ec.EC_DBG_MASKED, seq=b).astype(bool), st.masked)
            hist = np.array([np.iinfo(np.int32).min if h == -np.inf else int(h) for h in st.hist],
                            dtype=np.int32)
            assert np.array_equal(g.debug_read(ec.EC_DBG_HIST, seq=b), hist)
    finally:
        g.close()
    return {"steps": steps, "modes": modes, "worst": worst, "finished_early": finished_early}
