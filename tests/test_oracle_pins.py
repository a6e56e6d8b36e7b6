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
