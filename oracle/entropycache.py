"""CPU oracle for one EntropyCache denoising step (TEST INFRASTRUCTURE, not the product).

Plain numpy, float64 throughout.  It executes the algorithm of the paper's appendix
"Full EntropyCache algorithm" step by step, with the definitions of the Method section
(entropy-based skipping, Eq. 1; decode history, Eq. 2; top-k recent selection, Eq. 3; recency
threshold tau_R and recent mask R).  The method keeps a *stale* KV cache by design, so there is
no closed-form result to fall back on: every step is carried out as stated, with no blocking,
fusion or reordering.  numpy's matmul / einsum serve as the contraction primitive.

Only tests, the smoke check and the bench's cpu_baseline leg may import this module.  It shares
no code with the HIP path.  Weights arrive in their storage type (float32, bfloat16 bit patterns
as uint16, or 8-bit e4m3 codes with a float32 scale per row) and are up-cast exactly; all
activations are float64.

Readings taken where the paper is silent or inconsistent (each is listed in the design notes):
  * entropy uses the natural logarithm, 0*ln 0 := 0 (Eq. 1);
  * full recompute iff E > tau strictly (Eq. 1 text and both algorithms);
  * the mask set M^t of a step is the masked positions of the current fixed block of `block`
    generation slots (blockwise semi-autoregressive decoding of the related-work section);
  * decode() unmasks min(n, |M^t|) positions ranked by maximum softmax probability, token =
    argmax; ties go to the lowest token id / lowest position;
  * the history H has one entry per generation slot; "-inf" marks never decoded;
  * Delta t_recompute starts at 0 and is read before it is updated (appendix algorithm order);
  * the first step is a full forward over prompt and masks together;
  * H^{t,0} is the embedding of the current x for every recomputed row, taken once before
    layer 1;
  * new K/V rows are written into the cache before the rows attend (K_[I]^{t,l} in the
    appendix carries the current step's values for the recomputed rows);
  * model details: pre-norm Llama block without biases, untied embedding / LM head, rotate-half
    RoPE on absolute positions, softmax scale 1/sqrt(head_dim), grouped-query head a uses KV
    head a // (Hq/Hkv), the cache holds post-RoPE keys, logits only for the rows of M^t;
  * `logit_scale` multiplies the LM-head output (1.0 reproduces the paper's model);
  * optional decoding rules (defaults off): confidence-based parallel decoding unmasks every
    block row whose confidence is strictly above `conf_threshold`, the n most confident in any
    case (the experimental setup names the rule and the threshold 0.9, not its details);
    `gate_metric` selects the thresholding variable of the ablation (entropy sum, max
    confidence; a confidence skips at or above tau); `schedule` = 1 is sliding-window decoding
    with M^t = the leftmost `block` still-masked slots (the paper gives no advance rule).

Pins (tests/test_oracle_*.py): closed forms of the entropy, RoPE identities, a dense
no-cache forward written independently with explicit T x T scores, partial-step invariants,
brute-force enumeration of Eq. 3 / tau_R on tiny histories, and for the optional rules their
limiting cases and the per-row statistics a step reports.
End-to-end generations are "parity unpinned" against the paper: it prints no token-level
values and its weights and datasets are not available.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

FULL, PARTIAL, AUTO = 0, 1, 2
POS_INF = float("inf")
NEG_INF = -math.inf


# ----------------------------------------------------------------------------------------------
# storage decoding
# ----------------------------------------------------------------------------------------------
def e4m3_values() -> np.ndarray:
    """The 256 values of the 8-bit e4m3 format (1 sign bit, 4 exponent bits with bias 7, 3
    mantissa bits; exponent 0 = subnormals m/8 * 2^-6; no infinities; S.1111.111 = NaN), written
    out from the format's definition."""
    v = np.empty(256, dtype=np.float64)
    for c in range(256):
        sgn, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            x = math.nan
        elif e == 0:
            x = (m / 8.0) * 2.0 ** -6
        else:
            x = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        v[c] = -x if sgn else x
    return v


_E4M3 = e4m3_values()


def to_f64(w) -> np.ndarray:
    """Exact up-cast of a stored tensor: float32/float64 as is, uint16 = bfloat16 bit pattern, an
    object with `codes` (uint8 e4m3) and `scale` (float32 per row) = scale[row] * e4m3(code)."""
    if hasattr(w, "codes"):
        return _E4M3[w.codes] * w.scale.astype(np.float64)[:, None]
    if w.dtype == np.uint16:
        return (w.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return w.astype(np.float64)


# Optional memo of up-cast matrices, keyed by the stored array's identity.  Tests that run many
# steps on a model whose float64 copy fits in memory switch it on to skip the repeated
# conversion; it changes no arithmetic.  Off by default (the 8B-shaped models would not fit).
_F64_CACHE: Optional[dict] = None


def enable_f64_cache(on: bool) -> None:
    global _F64_CACHE
    _F64_CACHE = {} if on else None


def _w64(w: np.ndarray) -> np.ndarray:
    if _F64_CACHE is None or w.ndim < 2:
        return to_f64(w)
    key = id(w)
    hit = _F64_CACHE.get(key)
    if hit is None or hit[0] is not w:
        hit = (w, to_f64(w))
        _F64_CACHE[key] = hit
    return hit[1]


# ----------------------------------------------------------------------------------------------
# building blocks of the transformer layer ("W(.)" and "TransformerBlock" of the appendix)
# ----------------------------------------------------------------------------------------------
def rmsnorm(h: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """h / sqrt(mean(h^2) + eps) * gain, row-wise."""
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * gain


def rope(v: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing.

    v: [R, n_heads, hd]; pos: [R] absolute positions.  Pair (j, j+hd/2) is rotated by the angle
    pos * base^(-2j/hd).
    """
    hd = v.shape[-1]
    half = hd // 2
    j = np.arange(half, dtype=np.float64)
    inv_freq = base ** (-2.0 * j / hd)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]          # [R, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def attend(q: np.ndarray, kc: np.ndarray, vc: np.ndarray) -> np.ndarray:
    """Bidirectional attention of the rows in q against ALL cached positions.

    q: [R, Hq, hd]; kc, vc: [T, Hkv, hd].  No mask.  Returns [R, Hq, hd].
    """
    r, hq, hd = q.shape
    hkv = kc.shape[1]
    group = hq // hkv
    out = np.empty_like(q)
    for a in range(hq):
        kv = a // group
        s = q[:, a, :] @ kc[:, kv, :].T / math.sqrt(hd)                # [R, T]
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=1, keepdims=True)
        out[:, a, :] = p @ vc[:, kv, :]
    return out


def softmax_stats(z: np.ndarray):
    """For one row of logits: (argmax token, max probability, entropy in nats).  Eq. 1."""
    m = z.max()
    tok = int(np.argmax(z))                       # first maximum = lowest token id on ties
    e = np.exp(z - m)
    p = e / e.sum()
    with np.errstate(divide="ignore", invalid="ignore"):
        plogp = np.where(p > 0.0, p * np.log(p), 0.0)
    return tok, float(p.max()), float(-plogp.sum())


# ----------------------------------------------------------------------------------------------
# history / recent-token selection (Eq. 2, Eq. 3, tau_R, R)
# ----------------------------------------------------------------------------------------------
def kth_largest(hist: Sequence[float], k: int) -> float:
    """min over the k entries with the largest history values (Eq. 3); -inf if k exceeds the
    number of finite entries, because the selected set then contains a never-decoded slot."""
    if k <= 0:
        return math.inf                            # empty selection: nothing qualifies by rank
    srt = sorted(hist, reverse=True)
    if k > len(srt):
        return NEG_INF
    return srt[k - 1]


def recent_set(hist: Sequence[float], k: int, t: int, dt_recompute: int) -> List[int]:
    """Indices i (generation-slot numbering) with H_i >= tau_R,
    tau_R = max(min_{j in K} H_j, t - dt_recompute)."""
    tau_r = max(kth_largest(hist, k), t - dt_recompute)
    return [i for i, h in enumerate(hist) if h >= tau_r]


# ----------------------------------------------------------------------------------------------
# model + state
# ----------------------------------------------------------------------------------------------
@dataclass
class OracleModel:
    cfg: object                    # ec_inputs.ModelCfg-like: attributes only
    w: Dict[str, object]           # stored tensors (see ec_inputs.make_weights)


@dataclass
class OracleState:
    model: OracleModel
    dec: object                    # DecodeCfg-like
    P: int
    T: int
    x: np.ndarray                  # [T] int64 token ids
    masked: np.ndarray             # [T] bool: the explicit mask set
    hist: List[float]              # [N] decode step or -inf
    Kc: np.ndarray                 # [L, T, Hkv, hd] float64, NaN until first written
    Vc: np.ndarray
    t: int = 1
    dt: int = 0                    # Delta t_recompute (the paper's counter)
    t_lastfull: int = 0            # index of the last step that ran FULL
    skip: bool = False
    blk: int = 0
    R: List[int] = field(default_factory=list)   # absolute positions of recent tokens
    mode_forced: bool = False      # a caller has replaced the algorithm's branch at least once
    rows_recomputed: int = 0       # sum of |S| over steps (recompute ratio numerator)
    steps: int = 0
    n_full: int = 0

    @property
    def done(self) -> bool:
        return not bool(self.masked.any())


def eco_init(model: OracleModel, dec, prompt: np.ndarray) -> OracleState:
    cfg = model.cfg
    P = int(len(prompt))
    N = int(dec.gen_len)
    T = P + N
    x = np.full(T, cfg.mask_id, dtype=np.int64)
    x[:P] = prompt
    masked = np.zeros(T, dtype=bool)
    masked[P:] = True
    shape = (cfg.n_layers, T, cfg.n_kv_heads, cfg.head_dim)
    return OracleState(model=model, dec=dec, P=P, T=T, x=x, masked=masked,
                       hist=[NEG_INF] * N, Kc=np.full(shape, np.nan), Vc=np.full(shape, np.nan))


def current_block_masked(st: OracleState) -> np.ndarray:
    """The step's M^t.  Blockwise decoding: the masked positions of the current fixed block.
    Sliding-window decoding (the experiments' default, "window size = 32"; the paper states no
    advance rule - reading: the window always holds the leftmost `block` still-masked
    generation slots, so it slides on as its positions are decoded)."""
    w = st.dec.block
    if getattr(st.dec, "schedule", 0) == 1:
        idx = np.arange(st.P, st.T)
        return idx[st.masked[st.P:]][:w]
    lo = st.P + st.blk * w
    hi = min(st.T, lo + w)
    idx = np.arange(lo, hi)
    return idx[st.masked[lo:hi]]


def forward_rows(st: OracleState, S: np.ndarray, want_rows: np.ndarray) -> np.ndarray:
    """Recompute the rows S through every layer against the cache, scattering their new K/V
    first; return the final hidden state of `want_rows` (a subset of S), after the final norm.
    """
    cfg, w = st.model.cfg, st.model.w
    hq, hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    S = np.asarray(S, dtype=np.int64)
    if S.size == 0:
        return np.zeros((0, cfg.d_model))
    h = to_f64(w["tok_emb"][st.x[S]])                                    # H^{t,0} = Emb[x^t]
    for l in range(cfg.n_layers):
        u = rmsnorm(h, to_f64(w["attn_norm"][l]), cfg.rms_eps)
        q = (u @ _w64(w["wq"][l]).T).reshape(-1, hq, hd)
        k = (u @ _w64(w["wk"][l]).T).reshape(-1, hkv, hd)
        v = (u @ _w64(w["wv"][l]).T).reshape(-1, hkv, hd)
        q = rope(q, S, cfg.rope_base)
        k = rope(k, S, cfg.rope_base)
        st.Kc[l, S] = k                                                  # scatter, then attend
        st.Vc[l, S] = v
        o = attend(q, st.Kc[l], st.Vc[l]).reshape(-1, hq * hd)
        h = h + o @ _w64(w["wo"][l]).T
        u = rmsnorm(h, to_f64(w["mlp_norm"][l]), cfg.rms_eps)
        act = silu(u @ _w64(w["w_gate"][l]).T) * (u @ _w64(w["w_up"][l]).T)
        h = h + act @ _w64(w["w_down"][l]).T
    sel = np.searchsorted(S, np.asarray(want_rows, dtype=np.int64))
    return rmsnorm(h[sel], to_f64(w["final_norm"]), cfg.rms_eps)


MAX_TOKENS_PER_STEP = 32   # what one step result of the C ABI can report


def gate_value(H_dec, conf_dec, metric: int) -> float:
    """The quantity compared with tau over the step's newly decoded tokens: 0 = their maximum
    entropy (Eq. 1, the method's choice), 1 = the sum of their entropies, 2 = their maximum
    confidence (the two alternatives of the ablation "Choice of thresholding variable").
    No token decoded: the value that always skips."""
    if len(H_dec) == 0:
        return POS_INF if metric == 2 else NEG_INF
    if metric == 0:
        return float(max(H_dec))
    if metric == 1:
        return float(sum(H_dec))
    return float(max(conf_dec))


def gate_skips(value: float, tau: float, metric: int) -> bool:
    """Skip the full recomputation iff the step was certain: entropy metrics at most tau (Eq. 1,
    strict > recomputes); the confidence metric at least tau (reading: the paper does not say
    which side of the threshold a confidence is compared on; high confidence = certain)."""
    return value >= tau if metric == 2 else value <= tau


def eco_step(st: OracleState, mode: int = AUTO, forced: Optional[dict] = None,
             keep_logits: bool = True, rows_override: Optional[np.ndarray] = None) -> dict:
    """One denoising step.

    mode: AUTO follows the flag of the previous step (first step is FULL); FULL / PARTIAL
          replace the algorithm's branch (teacher forcing, benchmarks).
    forced: {"positions": [...], "tokens": [...]} commits these instead of the step's own
          decode() choice (the own choice is still reported).
    rows_override: test hook - recompute exactly these rows (must contain M^t) instead of
          M^t u R; used by the invariants "all rows == full" and "no rows == no change".
    """
    if st.done:
        raise RuntimeError("step after generation finished")
    cfg, dec = st.model.cfg, st.dec
    t = st.t
    if mode == AUTO:
        mode = FULL if (t == 1 or not st.skip) else PARTIAL
    else:
        st.mode_forced = True
    if mode == PARTIAL and st.t_lastfull == 0:
        raise RuntimeError("partial step before any full step: the cache is empty")

    Mb = current_block_masked(st)
    if mode == FULL:
        S = np.arange(st.T)
        st.t_lastfull = t
    else:
        S = np.array(sorted(set(Mb.tolist()) | set(st.R)), dtype=np.int64)
    if rows_override is not None:
        S = np.asarray(rows_override, dtype=np.int64)
    # Delta t_recompute: the paper's counter, read before this step updates it.  It equals
    # t - (index of the last FULL step) as long as the flag alone chooses the branch; once a
    # caller forces modes the counter has no meaning of its own and that identity defines it.
    dt_eff = (t - st.t_lastfull) if st.mode_forced else st.dt

    hfin = forward_rows(st, S, Mb if S.size else Mb[:0])
    st.rows_recomputed += int(S.size)
    st.steps += 1
    st.n_full += int(mode == FULL)

    res = {"t": t, "mode": mode, "S": S, "Mb": Mb}
    if S.size == 0:                                  # test hook only: nothing decoded
        return res
    z = cfg.logit_scale * (hfin @ _w64(st.model.w["lm_head"]).T)       # [|Mb|, V]
    stats = [softmax_stats(z[i]) for i in range(len(Mb))]
    tok = np.array([s[0] for s in stats], dtype=np.int64)
    conf = np.array([s[1] for s in stats])
    H = np.array([s[2] for s in stats])

    # decode(): the min(n, |Mb|) rows with largest confidence; ties -> lowest position.
    # Confidence-based parallel decoding (experimental setup, threshold 0.9): every row of the
    # block whose confidence exceeds the threshold is unmasked in the same step, the n most
    # confident ones in any case; one step reports at most MAX_TOKENS_PER_STEP tokens.
    n = min(dec.tokens_per_step, len(Mb))
    if dec.conf_threshold > 0:
        n = min(max(n, int(np.sum(conf > dec.conf_threshold))), MAX_TOKENS_PER_STEP, len(Mb))
    order = sorted(range(len(Mb)), key=lambda i: (-conf[i], Mb[i]))[:n]
    own_pos = [int(Mb[i]) for i in order]
    own_tok = [int(tok[i]) for i in order]
    own_H = [float(H[i]) for i in order]
    own_conf = [float(conf[i]) for i in order]
    E_own = gate_value(own_H, own_conf, dec.gate_metric)

    if forced is not None:
        D_pos = [int(p) for p in forced["positions"]]
        D_tok = [int(v) for v in forced["tokens"]]
        rowof = {int(p): i for i, p in enumerate(Mb)}
        # an empty commit never asks for a recomputation: nothing new entered the sequence
        E = (gate_value([float(H[rowof[p]]) for p in D_pos], [float(conf[rowof[p]]) for p in D_pos],
                        dec.gate_metric)
             if all(p in rowof for p in D_pos) else E_own)
    else:
        D_pos, D_tok, E = own_pos, own_tok, E_own

    for p, v in zip(D_pos, D_tok):
        st.x[p] = v
        st.masked[p] = False
        st.hist[p - st.P] = t                                            # Eq. 2

    Ri = recent_set(st.hist, dec.k_recent, t, dt_eff)                    # Eq. 3, tau_R, R
    st.R = [st.P + i for i in Ri]

    if gate_skips(E, dec.tau, dec.gate_metric):
        st.skip = True
        st.dt = st.dt + 1
    else:
        st.skip = False
        st.dt = 0

    nblocks = -(-dec.gen_len // dec.block)
    while st.blk < nblocks and current_block_masked(st).size == 0:
        st.blk += 1
    st.t = t + 1

    res.update({
        "logits": z if keep_logits else None, "tok": tok, "conf": conf, "H": H,
        "own_positions": own_pos, "own_tokens": own_tok, "own_entropy": own_H,
        "own_confidence": own_conf, "E_own": E_own,
        "positions": D_pos, "tokens": D_tok, "E": E, "skip": st.skip,
        "next_mode": PARTIAL if st.skip else FULL, "R": list(st.R), "done": st.done,
        "dt_paper": st.dt, "dt_eff": dt_eff,
    })
    return res


def eco_generate(st: OracleState, keep_logits: bool = False) -> List[dict]:
    """Run steps until no masked position is left; returns the per-step results."""
    trace = []
    while not st.done:
        trace.append(eco_step(st, AUTO, keep_logits=keep_logits))
    return trace


def recompute_ratio(st: OracleState) -> float:
    """Fraction of KV rows recomputed per step, averaged over the steps run so far."""
    return st.rows_recomputed / (st.steps * st.T) if st.steps else 0.0
