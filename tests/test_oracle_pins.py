"""Pins of the oracle's building blocks against what the mathematics fixes (no GPU).

Each test names the passage of the paper whose quantity it pins.  A pin never re-types the
oracle's own formula: it uses a closed form, an invariant, or an independent library routine.
"""
import itertools
import math

import numpy as np
import pytest
import scipy.special

from oracle import entropycache as eco


# ------------------------------------------------------------------ Eq. 1: decoded-token entropy
def test_entropy_uniform_is_ln_v():
    for v in (2, 7, 4096, 126464):
        tok, conf, h = eco.softmax_stats(np.full(v, 3.25))
        assert tok == 0                                  # lowest id on a tie
        assert conf == pytest.approx(1.0 / v, rel=1e-12)
        assert h == pytest.approx(math.log(v), rel=1e-12)


def test_entropy_two_equal_maxima_rest_minus_inf_is_ln2():
    z = np.full(50, -np.inf)
    z[7] = z[31] = 1.5
    tok, conf, h = eco.softmax_stats(z)
    assert tok == 7 and conf == pytest.approx(0.5) and h == pytest.approx(math.log(2.0), rel=1e-14)


def test_entropy_dominant_logit_goes_to_zero():
    z = np.zeros(1000)
    z[123] = 800.0                                       # exp underflows everywhere else
    tok, conf, h = eco.softmax_stats(z)
    assert tok == 123 and conf == 1.0 and h == 0.0


def test_entropy_two_point_closed_form():
    # logits (a, 0): p = sigmoid(a); H = binary entropy
    for a in (0.3, 1.0, 4.0, -2.0):
        p = 1.0 / (1.0 + math.exp(-a))
        hb = -(p * math.log(p) + (1 - p) * math.log(1 - p))
        tok, conf, h = eco.softmax_stats(np.array([a, 0.0]))
        assert tok == (0 if a > 0 else 1)
        assert conf == pytest.approx(max(p, 1 - p), rel=1e-13)
        assert h == pytest.approx(hb, rel=1e-12)


def test_entropy_matches_library_two_pass_and_invariants():
    rng = np.random.default_rng(0)
    for v, scale in ((17, 1.0), (4096, 0.3), (4096, 5.0), (126464, 4.8)):
        z = rng.standard_normal(v) * scale
        tok, conf, h = eco.softmax_stats(z)
        p = scipy.special.softmax(z)
        assert tok == int(np.argmax(p))
        assert conf == pytest.approx(p.max(), rel=1e-12)
        assert h == pytest.approx(scipy.special.entr(p).sum(), rel=1e-11)
        assert 0.0 <= h <= math.log(v) + 1e-12           # bounds
        tok2, conf2, h2 = eco.softmax_stats(z + 11.0)    # shift invariance
        assert tok2 == tok and conf2 == pytest.approx(conf, rel=1e-12)
        assert h2 == pytest.approx(h, rel=1e-11)


# ------------------------------------------------------------------ RoPE (model detail)
def test_rope_position_zero_is_identity_and_norm_preserved():
    rng = np.random.default_rng(1)
    v = rng.standard_normal((5, 3, 16))
    assert np.array_equal(eco.rope(v, np.zeros(5, dtype=np.int64), 10000.0), v)
    r = eco.rope(v, np.arange(5) * 37, 10000.0)
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(v, axis=-1), rtol=1e-13)


def test_rope_head_dim_two_is_a_plane_rotation():
    v = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    r = eco.rope(v, np.array([3, 3]), 10000.0)            # theta_0 = 1 -> angle 3 rad
    assert np.allclose(r[0, 0], [math.cos(3.0), math.sin(3.0)], atol=1e-15)
    assert np.allclose(r[1, 0], [-math.sin(3.0), math.cos(3.0)], atol=1e-15)


def test_rope_relative_position_property_and_frequencies():
    rng = np.random.default_rng(2)
    hd, base = 64, 500000.0
    q = rng.standard_normal((1, 1, hd))
    k = rng.standard_normal((1, 1, hd))
    def dot(m, n):
        return float((eco.rope(q, np.array([m]), base) * eco.rope(k, np.array([n]), base)).sum())
    assert dot(10, 3) == pytest.approx(dot(107, 100), rel=1e-10)
    assert dot(10, 3) != pytest.approx(dot(3, 10), rel=1e-6)      # direction matters
    # pair j rotates by pos * base^(-2j/hd): check through a complex-number formulation
    pos = np.array([12345])
    z = (q[0, 0, :hd // 2] + 1j * q[0, 0, hd // 2:]) * np.exp(
        1j * pos[0] * np.array([base ** (-(2.0 * j) / hd) for j in range(hd // 2)]))
    r = eco.rope(q, pos, base)[0, 0]
    assert np.allclose(r[:hd // 2], z.real, rtol=1e-11, atol=1e-12)
    assert np.allclose(r[hd // 2:], z.imag, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ RMSNorm, SiLU
def test_rmsnorm_unit_mean_square_and_scale_invariance():
    rng = np.random.default_rng(3)
    h = rng.standard_normal((4, 96)) * 7.0
    g = np.ones(96)
    u = eco.rmsnorm(h, g, 0.0)
    assert np.allclose((u * u).mean(-1), 1.0, rtol=1e-13)
    assert np.allclose(eco.rmsnorm(3.5 * h, g, 0.0), u, rtol=1e-13)
    g2 = rng.standard_normal(96)
    assert np.allclose(eco.rmsnorm(h, g2, 0.0), u * g2, rtol=1e-13)
    # eps enters under the root, added to the mean square
    one = np.full((1, 8), 2.0)
    assert np.allclose(eco.rmsnorm(one, np.ones(8), 5.0), 2.0 / math.sqrt(4.0 + 5.0))


def test_silu_is_x_times_logistic():
    x = np.linspace(-30, 30, 241)
    assert np.allclose(eco.silu(x), x * scipy.special.expit(x), rtol=1e-13, atol=1e-300)
    assert eco.silu(np.array([0.0]))[0] == 0.0


# ------------------------------------------------------------------ attention
def test_attend_matches_explicit_loops_with_gqa():
    rng = np.random.default_rng(4)
    R, T, hq, hkv, hd = 3, 7, 4, 2, 8
    q = rng.standard_normal((R, hq, hd))
    kc = rng.standard_normal((T, hkv, hd))
    vc = rng.standard_normal((T, hkv, hd))
    out = eco.attend(q, kc, vc)
    for r in range(R):
        for a in range(hq):
            kv = a // 2
            s = [sum(q[r, a, c] * kc[j, kv, c] for c in range(hd)) / math.sqrt(hd) for j in range(T)]
            p = scipy.special.softmax(np.array(s))
            ref = sum(p[j] * vc[j, kv] for j in range(T))
            assert np.allclose(out[r, a], ref, rtol=1e-12, atol=1e-14)


def test_attend_uniform_keys_average_values():
    # all keys identical -> softmax uniform -> output is the mean value, whatever the query
    T, hd = 9, 4
    q = np.random.default_rng(5).standard_normal((2, 1, hd))
    kc = np.tile(np.array([0.3, -1.0, 2.0, 0.5]), (T, 1, 1))
    vc = np.random.default_rng(6).standard_normal((T, 1, hd))
    out = eco.attend(q, kc, vc)
    assert np.allclose(out[:, 0], vc[:, 0].mean(0), rtol=1e-13)


# ------------------------------------------------------------------ Eq. 3, tau_R, R
def _literal_recent(hist, k, t, dt):
    """Eq. 3 taken literally: enumerate every subset of size k, keep one with the largest sum,
    take its minimum; then threshold the history with tau_R."""
    n = len(hist)
    best, best_sum = None, None
    for sub in itertools.combinations(range(n), k):
        s = sum(hist[j] for j in sub)
        if best is None or s > best_sum:
            best, best_sum = sub, s
    kth = min(hist[j] for j in best)
    tau_r = max(kth, t - dt)
    return [i for i in range(n) if hist[i] >= tau_r]


def test_recent_set_brute_force_all_small_histories():
    ninf = -math.inf
    checked = 0
    for n in (1, 2, 3, 4, 5):
        for k in (1, 2, 3):
            if k > n:
                continue
            for hist in itertools.product((ninf, 1, 2, 3, 4), repeat=n):
                for t in (4, 5):
                    for dt in (0, 1, 3):
                        assert eco.recent_set(list(hist), k, t, dt) == \
                            _literal_recent(list(hist), k, t, dt), (hist, k, t, dt)
                        checked += 1
    assert checked > 10000


def test_recent_set_examples():
    ninf = -math.inf
    # fewer than k decoded: the rank threshold is -inf, the step bound decides
    assert eco.recent_set([ninf, 5, ninf, 3], 3, 5, 2) == [1, 3]      # t-dt = 3
    assert eco.recent_set([ninf, 5, ninf, 3], 3, 5, 0) == [1]         # t-dt = 5
    # k most recent, but never older than the last full step
    assert eco.recent_set([1, 2, 3, 4, 5, 6], 2, 6, 5) == [4, 5]      # rank bound (5) wins
    assert eco.recent_set([1, 2, 3, 4, 5, 6], 4, 6, 1) == [4, 5]      # step bound (5) wins
    # ties with the k-th entry are all included
    assert eco.recent_set([7, 7, 7, 2], 2, 7, 7) == [0, 1, 2]


# ---- e4m3 weight storage (matrices as 8-bit codes with per-row scales) ------------------------
def test_e4m3_decode_matches_the_format_and_a_library():
    """The oracle's table against values the format fixes by definition (bias 7, 3 mantissa
    bits, subnormals, no infinities) and against torch's float8_e4m3fn."""
    import torch
    v = eco.e4m3_values()
    assert v[0x00] == 0.0 and v[0x38] == 1.0 and v[0x40] == 2.0 and v[0x3C] == 1.5
    assert v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9 and v[0x08] == 2.0 ** -6
    assert v[0x7E] == 448.0 and np.isnan(v[0x7F]) and np.isnan(v[0xFF])
    assert np.array_equal(v[0x80:0xFF], -v[0x00:0x7F])
    assert np.all(np.diff(v[:0x7F]) > 0)                       # monotonic in the code
    t = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.nan_to_num(t, nan=7e9), np.nan_to_num(v, nan=7e9))


def test_e4m3_encoder_rounds_to_nearest_even_and_saturates():
    """The input generator's encoder: brute-force nearest representable value (ties to the even
    code), exact round trip of every code, saturation, and torch's conversion."""
    import torch
    import ec_inputs
    v = eco.e4m3_values()
    codes = np.array([c for c in range(256) if not np.isnan(v[c])], dtype=np.uint8)
    back = ec_inputs.f32_to_e4m3_bits(v[codes].astype(np.float32))
    assert np.array_equal(back[codes != 0x80], codes[codes != 0x80])     # (-0 keeps its sign too)
    assert back[list(codes).index(0x80)] == 0x80
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(20000) * s for s in (0.004, 0.3, 20.0, 300.0)]
                       ).astype(np.float32)
    pos = v[:0x7F]
    mids = (pos[:-1] + pos[1:]) / 2                                       # ties listed exactly
    x = np.concatenate([x, mids.astype(np.float32), -mids.astype(np.float32),
                        np.float32([448.0, 449.0, 1e9, -1e9, np.inf, 464.0, 0.0])])
    got = ec_inputs.f32_to_e4m3_bits(x)
    for xi, ci in zip(x.astype(np.float64), got):
        a = min(abs(xi), 448.0)
        d = np.abs(pos - a)
        best = np.flatnonzero(d == d.min())
        want = best[0] if len(best) == 1 else [b for b in best if b % 2 == 0][0]
        assert (ci & 0x7F) == want and (ci >> 7) == int(np.signbit(xi)), (xi, ci, want)
    ref = torch.from_numpy(np.clip(x, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, ref)


def test_quantised_model_is_exactly_its_dequantised_model():
    """A model stored as e4m3 codes + row scales must behave, in the oracle, exactly like the
    float model holding scale * value (decoded here through torch, not through the oracle)."""
    import torch
    import ec_inputs
    cfg = ec_inputs.ModelCfg(n_layers=2, d_model=64, n_heads=2, n_kv_heads=1, head_dim=32,
                             d_ffn=128, vocab=80, mask_id=79, logit_scale=3.0, dtype="fp8w")
    w = ec_inputs.make_weights(cfg, 5, std=0.3, gain_jitter=0.2, threads=1)
    assert w["wq"][0].codes.dtype == np.uint8 and w["wq"][0].scale.shape == (64,)
    # per-row scale maps the row's largest magnitude onto 448, the largest e4m3 value
    assert np.all((w["w_up"][1].codes & 0x7F).max(axis=1) == 0x7E)

    def deq(m):
        t = torch.from_numpy(m.codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
        return t * m.scale.astype(np.float64)[:, None]
    wf = {k: ([deq(x) if hasattr(x, "codes") else eco.to_f64(x) for x in v] if isinstance(v, list)
              else (deq(v) if hasattr(v, "codes") else eco.to_f64(v))) for k, v in w.items()}
    dec = ec_inputs.DecodeCfg(gen_len=8, block=4, k_recent=2, tokens_per_step=1, tau=1.0)
    prompt = np.arange(5, dtype=np.int32)
    a = eco.eco_init(eco.OracleModel(cfg, w), dec, prompt)
    b = eco.eco_init(eco.OracleModel(cfg.replace(dtype="f32"), wf), dec, prompt)
    for mode in (eco.FULL, eco.PARTIAL, eco.PARTIAL):
        ra, rb = eco.eco_step(a, mode), eco.eco_step(b, mode)
        assert np.array_equal(ra["logits"], rb["logits"]) and ra["positions"] == rb["positions"]
    assert np.array_equal(a.Kc, b.Kc)
    # and quantisation moved every weight by at most half a grid step of its row
    x = ec_inputs.normal_tensor(5, "wq.0", (64, 64), 0.3, "f32")
    err = np.abs(deq(w["wq"][0]) - x)
    assert np.all(err <= 0.5 * 32.0 * w["wq"][0].scale[:, None] + 1e-12)   # step <= 32 below 448
