"""Teacher-forced comparison of the HIP path with the CPU oracle on the same seeded inputs.
The oracle's decisions (mode, committed positions / tokens) drive both sides, because the method
keeps a stale cache by design and a single different decision would make the two runs diverge
without either being wrong.

What is compared at every step (tol = 2e-2 for bfloat16 models, 1e-4 for float32 ones):

 1. logits of the block's masked rows and the K / V caches: max |a - b| <= tol * max |b|;
 2. the vocabulary reduction on its own (Eq. 1): the oracle's softmax statistics evaluated on the
    GPU's OWN float32 logits must give the GPU's token (exact), confidence and entropy (float32
    accumulation over V: REDUCE_TOL) - no logit error enters here, whatever the vocabulary;
 3. the decision on its own: decode(), the gate value and the next mode recomputed on the host
    from the GPU's per-row statistics in float32 must equal what the step reports, bit for bit;
 4. statistics against the oracle: |H_gpu - H_oracle| within what the row's measured logit error
    allows (and never more than 2 STAT_TOL ln V; rows beyond STAT_TOL ln V are counted), and
    ln conf_gpu inside the interval that the row's measured logit error dz allows (entropy, first
    order: |dH| <= sum_j p_j |ln p_j + H| * dz; confidence, exactly: ln conf moves by
    -ln(p + (1-p) e^(+-2 dz)) while the argmax stays, by at most 2 dz otherwise);
 5. decisions against the oracle, bit-exact wherever the oracle's margins exceed the tolerance:
    the argmax token of a row when its top-2 logit gap exceeds tol * max|z| (and twice the row's
    measured logit error).  For the unmasked positions every row gets the interval its
    confidence can lie in given its measured logit error: a row that fewer than n others can
    reach must be unmasked, a row that n others certainly beat must not be, and when that
    settles the whole choice the position lists must be equal.  The next mode is compared when
    every choice those intervals allow puts the gate value on the same side of tau by more than
    tol * ln V.
 6. integer state (x, mask set, history, row sets, counters): bit-exact.
"""
import math

import numpy as np

import paper_2603_18489_amd as ec
from oracle import entropycache as eco

REDUCE_TOL = 4e-6     # float32 sums over the vocabulary against float64 ones, relative
STAT_TOL = 2e-2       # entropy against the oracle, in units of ln V (bfloat16); float32: tol


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32)


def relerr(a, b):
    """max |a-b| / max |b| over the tensor."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if b.size == 0:
        return 0.0
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def gpu_cache(g, which, layer, seq=0):
    c = g.debug_read(which, layer, seq=seq)
    return bf16_bits_to_f32(c) if c.dtype == np.uint16 else c


class Counters:
    """What a run checked bit-exactly, and the largest deviations it saw."""

    def __init__(self):
        self.tokens_exact = 0      # block rows whose argmax token was compared with the oracle's
        self.choices_exact = 0     # steps whose unmasked positions / tokens were compared
        self.modes_exact = 0       # steps whose next mode was compared
        self.rows_decided = 0      # rows that had to be (or could not be) unmasked, and were checked
        self.rows_stat = 0         # rows whose entropy was compared with the oracle's ...
        self.rows_stat_beyond = 0  # ... and how many of them were off by more than STAT_TOL * ln V
        self.worst = {"logits": 0.0, "K": 0.0, "V": 0.0, "H_lnV": 0.0, "H_vs_bound": 0.0,
                      "lnconf_vs_bound": 0.0, "reduce_H": 0.0, "reduce_conf": 0.0}

    def up(self, key, v):
        self.worst[key] = max(self.worst.get(key, 0.0), float(v))

    def summary(self):
        return {"tokens_exact": self.tokens_exact, "choices_exact": self.choices_exact,
                "modes_exact": self.modes_exact, "rows_decided": self.rows_decided,
                "rows_stat": self.rows_stat, "rows_stat_beyond": self.rows_stat_beyond,
                "worst": self.worst}


def check_reduction(cfg, logits_gpu, stats, cnt, where=""):
    """Check 2: Eq. 1 evaluated by the oracle on the GPU's own logits."""
    lnV = math.log(cfg.vocab)
    for i in range(logits_gpu.shape[0]):
        tok, conf, H = eco.softmax_stats(logits_gpu[i].astype(np.float64))
        assert int(stats[i, 0]) == tok, f"{where} row {i}: token {int(stats[i, 0])} != argmax {tok}"
        assert stats[i, 3] == logits_gpu[i].max(), f"{where} row {i}: max logit"
        eC = abs(float(stats[i, 1]) - conf) / conf
        eH = abs(float(stats[i, 2]) - H) / lnV
        cnt.up("reduce_conf", eC)
        cnt.up("reduce_H", eH)
        assert eC <= REDUCE_TOL, f"{where} row {i}: confidence {stats[i, 1]} vs {conf} ({eC:.2e})"
        assert eH <= REDUCE_TOL, f"{where} row {i}: entropy {stats[i, 2]} vs {H} ({eH:.2e} ln V)"


def own_decision_from_stats(stats, Mb, dec):
    """decode(), gate value and next mode from per-row float32 statistics, in float32, with the
    tie rules of the method's readings (most confident first, ties to the lowest position)."""
    f32 = np.float32
    conf = stats[:, 1].astype(f32)
    H = stats[:, 2].astype(f32)
    nmb = len(Mb)
    n = min(dec.tokens_per_step, nmb)
    thr = f32(getattr(dec, "conf_threshold", 0.0))
    if thr > 0:
        n = min(max(n, int(np.sum(conf > thr))), ec.EC_MAX_N, nmb)
    order = sorted(range(nmb), key=lambda i: (-float(conf[i]), int(Mb[i])))[:n]
    metric = getattr(dec, "gate_metric", 0)
    if n == 0:
        gate = f32(np.inf) if metric == 2 else f32(-np.inf)
    elif metric == 0:
        gate = max(H[i] for i in order)
    elif metric == 1:
        gate = H[order[0]]
        for i in order[1:]:
            gate = f32(gate + H[i])
    else:
        gate = max(conf[i] for i in order)
    tau = f32(dec.tau)
    skips = bool(gate >= tau) if metric == 2 else bool(gate <= tau)
    return {"positions": [int(Mb[i]) for i in order], "tokens": [int(stats[i, 0]) for i in order],
            "entropy": [float(H[i]) for i in order], "confidence": [float(conf[i]) for i in order],
            "gate": float(gate), "next_mode": ec.EC_PARTIAL if skips else ec.EC_FULL}


def check_own_decision(stats, Mb, dec, q, where=""):
    """Check 3: what the step reports equals the decision rule applied to its own statistics."""
    d = own_decision_from_stats(stats, Mb, dec)
    assert q["n_unmasked"] == len(d["positions"]), f"{where}: number of unmasked tokens"
    assert q["positions"] == d["positions"], f"{where}: positions {q['positions']} vs {d['positions']}"
    assert q["tokens"] == d["tokens"], f"{where}: tokens"
    assert np.array_equal(np.float32(q["entropy"]), np.float32(d["entropy"])), f"{where}: entropies"
    assert np.array_equal(np.float32(q["confidence"]), np.float32(d["confidence"])), f"{where}: confidences"
    assert np.float32(q["max_entropy"]) == np.float32(d["gate"]), \
        f"{where}: gate value {q['max_entropy']} vs {d['gate']}"
    assert q["next_mode"] == d["next_mode"], f"{where}: next mode"


def oracle_reference(r, dec):
    """The oracle-side quantities of one step that checks 4 and 5 need (also what the stored
    traces hold)."""
    z = r["logits"]
    srt = np.sort(z, axis=1)
    m = z.max(axis=1)
    lse = m + np.log(np.exp(z - m[:, None]).sum(axis=1))
    lp = z - lse[:, None]
    p = np.exp(lp)
    return {"Mb": [int(v) for v in r["Mb"]], "tok": [int(v) for v in r["tok"]],
            "conf": np.asarray(r["conf"]), "H": np.asarray(r["H"]),
            "top2gap": srt[:, -1] - srt[:, -2],
            "H_sens": (p * np.abs(lp + np.asarray(r["H"])[:, None])).sum(axis=1),
            "logits_absmax": float(np.abs(z).max()),
            "own_positions": list(r["own_positions"]), "own_tokens": list(r["own_tokens"]),
            "E_own": float(r["E_own"])}


def check_against_oracle(cfg, dec, tol, ref, q, stats, dz_row, cnt, where=""):
    """Checks 4 and 5.  dz_row: per block row, the largest |z_gpu - z_oracle| that was measured."""
    lnV = math.log(cfg.vocab)
    nmb = len(ref["Mb"])
    conf, H = np.asarray(ref["conf"]), np.asarray(ref["H"])
    dz = np.asarray(dz_row, dtype=np.float64)
    gaps = np.asarray(ref["top2gap"])
    stat_tol = STAT_TOL if cfg.dtype != "f32" else tol
    # Interval that a row's log-confidence can lie in, given |dz| <= dz_i on every logit: with p
    # the oracle's confidence and the argmax unchanged, ln conf moves by -ln(p + (1-p) e^(+-2 dz));
    # in any case by at most 2 dz.
    lcf = np.log(conf)
    up = np.where(gaps > 2.0 * dz, -np.log(conf + (1.0 - conf) * np.exp(-2.0 * dz)), 2.0 * dz)
    down = np.where(gaps > 2.0 * dz, np.log(conf + (1.0 - conf) * np.exp(2.0 * dz)), 2.0 * dz)
    hi, lo = lcf + up + 4 * REDUCE_TOL, lcf - down - 4 * REDUCE_TOL
    # ---- 4. statistics ---------------------------------------------------------------------------
    for i in range(nmb):
        eH = abs(float(stats[i, 2]) - H[i])
        bound_H = (1.5 * float(ref["H_sens"][i]) + dz[i]) * dz[i] + REDUCE_TOL * lnV
        cnt.up("H_lnV", eH / lnV)
        cnt.up("H_vs_bound", eH / bound_H)
        # (the nominal bar of stat_tol * ln V is what small logit errors give; a row whose measured
        # logit error allows more is held to what that error allows, never to more than twice the bar)
        assert eH <= bound_H, f"{where} row {i}: entropy error {eH:.3e} > bound {bound_H:.3e} from dz {dz[i]:.3e}"
        assert eH <= 2 * stat_tol * lnV, f"{where} row {i}: entropy {stats[i, 2]} vs {H[i]}"
        cnt.rows_stat += 1
        cnt.rows_stat_beyond += int(eH > stat_tol * lnV)
        lc_gpu = math.log(float(stats[i, 1]))
        cnt.up("lnconf_vs_bound", max((lc_gpu - lcf[i]) / (hi[i] - lcf[i]), (lcf[i] - lc_gpu) / (lcf[i] - lo[i])))
        assert lo[i] <= lc_gpu <= hi[i], f"{where} row {i}: confidence {stats[i, 1]} vs {conf[i]}"
    # ---- 5. decisions ----------------------------------------------------------------------------
    # argmax token: cannot differ when the row's top-2 gap exceeds twice its logit error
    row_ok = gaps > np.maximum(tol * ref["logits_absmax"], 2.0 * dz)
    for i in range(nmb):
        if row_ok[i]:
            assert int(stats[i, 0]) == ref["tok"][i], f"{where} row {i}: argmax token"
            cnt.tokens_exact += 1
    own = ref["own_positions"]
    n = len(own)
    chosen_rows = [ref["Mb"].index(p) for p in own]
    thr = getattr(dec, "conf_threshold", 0.0)
    n_known = True
    if thr > 0:      # how many tokens a step unmasks depends on the side of the threshold
        lt = math.log(thr)
        n_known = bool(np.all((lo > lt) | (hi < lt)))
    metric = getattr(dec, "gate_metric", 0)
    got = set(q["positions"])
    if n_known:
        assert q["n_unmasked"] == n, f"{where}: number of unmasked tokens"
        # Whatever the logit errors within dz did, a row that fewer than n others can reach is
        # unmasked, and a row that n others certainly beat is not.
        surely_in = [i for i in range(nmb)
                     if sum(1 for j in range(nmb) if j != i and hi[j] >= lo[i]) < n]
        surely_out = [i for i in range(nmb)
                      if sum(1 for j in range(nmb) if j != i and lo[j] > hi[i]) >= n]
        for i in surely_in:
            assert ref["Mb"][i] in got, f"{where}: position {ref['Mb'][i]} must be unmasked"
            assert i in chosen_rows
        for i in surely_out:
            assert ref["Mb"][i] not in got, f"{where}: position {ref['Mb'][i]} cannot be unmasked"
        cnt.rows_decided += len(surely_in) + len(surely_out)
        for p_, t_ in zip(q["positions"], q["tokens"]):     # tokens of whatever rows it chose
            i = ref["Mb"].index(p_)
            if row_ok[i]:
                assert t_ == ref["tok"][i], f"{where}: token at position {p_}"
        if len(surely_in) == n:      # the whole choice is determined
            order_ok = all(lo[a] > hi[b] for a, b in zip(chosen_rows[:-1], chosen_rows[1:]))
            if order_ok:
                assert q["positions"] == own, f"{where}: positions {q['positions']} vs {own}"
            else:
                assert sorted(q["positions"]) == sorted(own), f"{where}: positions (as a set)"
            cnt.choices_exact += 1
            if metric != 2 and n > 0 and all(row_ok[i] for i in chosen_rows):
                assert abs(q["max_entropy"] - ref["E_own"]) <= stat_tol * lnV * (n if metric == 1 else 1), \
                    f"{where}: gate value {q['max_entropy']} vs {ref['E_own']}"
        # the next mode, when every choice the errors allow lands on the same side of tau
        possible = [i for i in range(nmb) if i not in surely_out]
        decided = None
        if metric == 0 and n > 0:
            m_ = stat_tol * lnV
            if all(H[i] < dec.tau - m_ for i in possible):
                decided = eco.PARTIAL
            elif any(H[i] > dec.tau + m_ for i in surely_in) or all(H[i] > dec.tau + m_ for i in possible):
                decided = eco.FULL
        elif metric == 1 and n > 0 and len(surely_in) == n:
            m_ = stat_tol * lnV * n
            if abs(ref["E_own"] - dec.tau) > m_:
                decided = eco.PARTIAL if ref["E_own"] <= dec.tau else eco.FULL
        elif metric == 2 and n > 0:
            lt = math.log(max(dec.tau, 1e-300))
            if any(lo[i] > lt for i in surely_in):
                decided = eco.PARTIAL
            elif all(hi[i] < lt for i in possible):
                decided = eco.FULL
        if decided is not None:
            assert q["next_mode"] == decided, f"{where}: next mode"
            cnt.modes_exact += 1


def check_row_set(g, exp_rows, seq=0, where=""):
    """The row set M u R the GPU built for its next partial step: size first, then content."""
    try:
        g.debug_read(ec.EC_DBG_ROWS, count=len(exp_rows) + 1, seq=seq)
        raise AssertionError(f"{where}: the GPU's row set holds more than {len(exp_rows)} rows")
    except ec.EcError as e:
        assert e.code == ec.EC_ERR_ARG
    rows = g.debug_read(ec.EC_DBG_ROWS, count=len(exp_rows), seq=seq)
    assert rows.tolist() == exp_rows, f"{where}: row set differs"


def check_step(cfg, dec, tol, r, q, g, cnt, seq=0, where=""):
    """All per-step checks of one sequence against a live oracle result r."""
    nmb = len(r["Mb"])
    assert q["mode_run"] == r["mode"] and q["n_query_rows"] == len(r["S"]), where
    assert q["n_block_rows"] == nmb and q["step_index"] == r["t"], where
    assert q["done"] == r["done"] and q["n_recent_next"] == len(r["R"]), where
    logits = g.debug_read(ec.EC_DBG_LOGITS, count=nmb, seq=seq)
    stats = g.debug_read(ec.EC_DBG_ROW_STATS, count=nmb, seq=seq)
    e = relerr(logits, r["logits"])
    cnt.up("logits", e)
    assert e <= tol, f"{where} mode {r['mode']}: logits rel err {e:.3e} > {tol}"
    check_reduction(cfg, logits, stats, cnt, where)
    check_own_decision(stats, [int(v) for v in r["Mb"]], dec, q, where)
    dz_row = np.abs(logits.astype(np.float64) - r["logits"]).max(axis=1)
    check_against_oracle(cfg, dec, tol, oracle_reference(r, dec), q, stats, dz_row, cnt, where)


def hist_i32(st):
    return np.array([np.iinfo(np.int32).min if h == -np.inf else int(h) for h in st.hist],
                    dtype=np.int32)


def run_teacher_forced(cfg, w, dec, prompt, tol, max_steps=None, check_cache_every=1,
                       dev_weights=None, verbose=False, mode_fn=None, cache_layers=None):
    """Runs the oracle free (AUTO, or with the modes mode_fn(step_index) forces on both sides)
    and the GPU teacher-forced by it.  Returns a summary dict; raises AssertionError on any
    parity violation."""
    st = eco.eco_init(eco.OracleModel(cfg, w), dec, prompt)
    dw = dev_weights if dev_weights is not None else ec.weights_to_device(cfg, w)
    g = ec.EntropyCache(cfg, dw, dec, prompt)
    g.keep_logits(True)
    cnt = Counters()
    modes = {eco.FULL: 0, eco.PARTIAL: 0}
    steps = 0
    try:
        while not st.done and (max_steps is None or steps < max_steps):
            # the row set the GPU built for a partial step must be the oracle's M u R
            Mb = eco.current_block_masked(st)
            if steps > 0:
                check_row_set(g, sorted(set(Mb.tolist()) | set(st.R)), where=f"step {st.t}")
            r = eco.eco_step(st, eco.AUTO if mode_fn is None else mode_fn(steps))
            q = g.step_forced(r["mode"], r["positions"], r["tokens"])
            steps += 1
            modes[r["mode"]] += 1
            check_step(cfg, dec, tol, r, q, g, cnt, where=f"step {r['t']}")
            if check_cache_every and (steps % check_cache_every == 0 or st.done):
                for l in (range(cfg.n_layers) if cache_layers is None else cache_layers):
                    for name, which, oc in (("K", ec.EC_DBG_KCACHE, st.Kc), ("V", ec.EC_DBG_VCACHE, st.Vc)):
                        e = relerr(gpu_cache(g, which, l), oc[l])
                        cnt.up(name, e)
                        assert e <= tol, f"step {r['t']} layer {l}: {name} cache rel err {e:.3e}"
            if verbose:
                print(f"t={r['t']} mode={r['mode']} |S|={len(r['S'])} E={r['E']:.3f} "
                      f"logits={cnt.worst['logits']:.2e} H={cnt.worst['H_lnV']:.2e}lnV "
                      f"exact tok/choice/mode {cnt.tokens_exact}/{cnt.choices_exact}/{cnt.modes_exact}",
                      flush=True)
        # integer state is bit-exact
        assert np.array_equal(g.debug_read(ec.EC_DBG_X), st.x.astype(np.int32))
        assert np.array_equal(g.debug_read(ec.EC_DBG_MASKED).astype(bool), st.masked)
        assert np.array_equal(g.debug_read(ec.EC_DBG_HIST), hist_i32(st))
    finally:
        g.close()
    out = cnt.summary()
    out.update({"steps": steps, "modes": modes, "exact_checked": cnt.choices_exact})
    return out


def run_teacher_forced_batch(cfg, w, dec, prompts, tol, max_steps=None, fast_seq=None,
                             check_cache_every=4):
    """The batched HIP path against one oracle run per sequence (sequences are independent, so
    the batch must reproduce each of them).  fast_seq: that sequence commits every masked token
    of its block at each step (with the oracle's argmax tokens), so it finishes early while the
    others go on.  Returns a summary; raises AssertionError on any parity violation."""
    import copy
    B = len(prompts)
    model = eco.OracleModel(cfg, w)
    dec1 = dec.replace(batch=1)
    sts = [eco.eco_init(model, dec1, p) for p in prompts]
    g = ec.EntropyCache(cfg, ec.weights_to_device(cfg, w), dec, prompts)
    g.keep_logits(True)
    cnt = Counters()
    steps, modes = 0, {eco.FULL: 0, eco.PARTIAL: 0}
    finished_early = 0
    try:
        while not all(st.done for st in sts) and (max_steps is None or steps < max_steps):
            res = [None] * B
            for b, st in enumerate(sts):
                if st.done:
                    continue
                Mb = eco.current_block_masked(st)
                if steps > 0:
                    check_row_set(g, sorted(set(Mb.tolist()) | set(st.R)), seq=b,
                                  where=f"seq {b} step {st.t}")
                if b == fast_seq:
                    # look at the step's own tokens first, then commit the whole block
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
                check_step(cfg, dec1, tol, r, q[b], g, cnt, seq=b, where=f"seq {b} step {r['t']}")
                if steps % check_cache_every == 0 or sts[b].done:
                    for l in range(cfg.n_layers):
                        for name, which, oc in (("K", ec.EC_DBG_KCACHE, sts[b].Kc),
                                                ("V", ec.EC_DBG_VCACHE, sts[b].Vc)):
                            e = relerr(gpu_cache(g, which, l, seq=b), oc[l])
                            cnt.up(name, e)
                            assert e <= tol, f"seq {b} step {r['t']} layer {l}: {name} cache {e:.3e}"
        for b, st in enumerate(sts):
            assert np.array_equal(g.debug_read(ec.EC_DBG_X, seq=b), st.x.astype(np.int32))
            assert np.array_equal(g.debug_read(ec.EC_DBG_MASKED, seq=b).astype(bool), st.masked)
            assert np.array_equal(g.debug_read(ec.EC_DBG_HIST, seq=b), hist_i32(st))
    finally:
        g.close()
    out = cnt.summary()
    out.update({"steps": steps, "modes": modes, "finished_early": finished_early,
                "exact_checked": cnt.choices_exact})
    return out
