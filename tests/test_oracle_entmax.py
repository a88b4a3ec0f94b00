"""Pins for the oracle's alpha-entmax and attention (CPU only).

Each test checks the oracle against something other than itself: brute force, a textbook
closed form, a value the paper prints, or an invariant the paper proves."""
import itertools
import os
import math
import numpy as np
import pytest
from scipy.optimize import brentq

from oracle import entmaxkv_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALPHAS = [1.25, 4.0 / 3.0, 1.5, 2.0]


def brute_force_entmax(s, alpha):
    """Sec. 2.2 Eq. 2-3 by enumeration: the support is the unique subset S such that the root tau_S
    of sum_{i in S} ((alpha-1)s_i - tau)^beta = 1 makes exactly the members of S exceed tau_S."""
    a = alpha - 1.0
    beta = 1.0 / a
    z = a * np.asarray(s, dtype=np.float64)
    n = len(z)
    found = []
    for r in range(1, n + 1):
        for S in itertools.combinations(range(n), r):
            zs = z[list(S)]
            f = lambda t: np.sum((zs - t) ** beta) - 1.0
            hi = zs.min()
            if f(hi) >= 0:         # even at the smallest member the mass is >= 1: no root below it
                continue
            tau = brentq(f, hi - 1.0 - 1e-6, hi, xtol=1e-15, rtol=1e-15, maxiter=500)
            if set(np.nonzero(z > tau)[0]) == set(S):
                found.append((S, tau))
    assert len(found) == 1, found
    S, tau = found[0]
    p = np.zeros(n)
    p[list(S)] = (z[list(S)] - tau) ** beta
    return p, tau


@pytest.mark.parametrize("alpha", ALPHAS)
@pytest.mark.parametrize("seed", range(6))
def test_bruteforce_small(alpha, seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1, 9))
    s = rng.normal(size=n) * rng.choice([0.3, 1.0, 4.0])
    p_ref, tau_ref = brute_force_entmax(s, alpha)
    p, tau, mask = orc.entmax_probs(s, alpha)
    np.testing.assert_allclose(p, p_ref, atol=1e-12)
    assert abs(tau - tau_ref) < 1e-12
    assert np.array_equal(mask, p_ref > 0)


def sparsemax_textbook(s):
    """Sparsemax closed form (Martins & Astudillo 2016): k(z)=max{k: 1+k z_(k) > sum_{j<=k} z_(j)},
    tau=(sum_{j<=k} z_(j) - 1)/k."""
    zs = np.sort(s)[::-1]
    cs = np.cumsum(zs)
    ks = np.arange(1, len(s) + 1)
    k = ks[1 + ks * zs > cs].max()
    tau = (cs[k - 1] - 1.0) / k
    return np.maximum(s - tau, 0.0), tau


@pytest.mark.parametrize("seed", range(5))
def test_alpha2_is_sparsemax(seed):
    rng = np.random.default_rng(seed)
    s = rng.normal(size=200) * 2.0
    p_ref, tau_ref = sparsemax_textbook(s)
    p, tau, _ = orc.entmax_probs(s, 2.0)
    np.testing.assert_allclose(p, p_ref, atol=1e-13)
    assert abs(tau - tau_ref) < 1e-13


def test_alpha_to_one_approaches_softmax():
    rng = np.random.default_rng(7)
    s = rng.normal(size=50)
    sm = np.exp(s - s.max()); sm /= sm.sum()
    errs = []
    for alpha in (1.2, 1.05, 1.01, 1.002):
        p, _, _ = orc.entmax_probs(s, alpha)
        errs.append(np.abs(p - sm).max())
    assert errs[0] > errs[1] > errs[2] > errs[3]
    assert errs[3] < 2e-3


@pytest.mark.parametrize("alpha", ALPHAS + [1.1, 1.7, 3.0])
def test_normalisation_and_threshold_equation(alpha):
    rng = np.random.default_rng(11)
    s = rng.normal(size=3000) * 3.0
    p, tau, mask = orc.entmax_probs(s, alpha)
    assert abs(p.sum() - 1.0) < 1e-12
    a = alpha - 1.0
    assert abs(np.sum(np.maximum(a * s - tau, 0.0) ** (1.0 / a)) - 1.0) < 1e-12
    assert np.array_equal(mask, p > 0)
    assert np.all(a * s[mask] > tau) and np.all(a * s[~mask] <= tau)


def test_two_token_closed_form_alpha15():
    # alpha=1.5, s=(x,0), z=s/2: both in the support iff z1-z2<1; then with d=z1-z2
    # tau = mean - sqrt((1-d^2/2)/2), p1 = (d/2 + sqrt((1-d^2/2)/2))^2 (solve the quadratic by hand).
    for x in (0.0, 0.4, 1.0, 1.9):
        d = x / 2.0
        p1 = (d / 2.0 + np.sqrt((1.0 - d * d / 2.0) / 2.0)) ** 2
        p, _, _ = orc.entmax_probs(np.array([x, 0.0]), 1.5)
        np.testing.assert_allclose(p, [p1, 1.0 - p1], atol=1e-14)
    p, _, mask = orc.entmax_probs(np.array([2.0, 0.0]), 1.5)   # z1-z2 = 1 exactly: second token has p=0
    np.testing.assert_allclose(p, [1.0, 0.0], atol=1e-15)
    assert list(mask) == [True, False]                         # strict inequality of Eq. 3


def test_degenerate_inputs():
    for alpha in ALPHAS:
        p, tau, mask = orc.entmax_probs(np.array([3.7]), alpha)
        assert p.tolist() == [1.0] and mask.tolist() == [True]
        assert abs(tau - ((alpha - 1) * 3.7 - 1.0)) < 1e-15
        p, _, _ = orc.entmax_probs(np.full(4, -2.5), alpha)
        np.testing.assert_allclose(p, 0.25, atol=1e-15)


@pytest.mark.parametrize("alpha", ALPHAS)
def test_shift_and_permutation(alpha):
    rng = np.random.default_rng(3)
    s = rng.normal(size=64)
    p, tau, _ = orc.entmax_probs(s, alpha)
    p2, tau2, _ = orc.entmax_probs(s + 5.0, alpha)
    np.testing.assert_allclose(p2, p, atol=1e-12)
    assert abs(tau2 - (tau + (alpha - 1.0) * 5.0)) < 1e-12
    perm = rng.permutation(64)
    p3, tau3, _ = orc.entmax_probs(s[perm], alpha)
    np.testing.assert_allclose(p3, p[perm], atol=1e-14)
    assert abs(tau3 - tau) < 1e-14


def test_attention_uses_q_dot_k_and_p_times_v():
    # one-hot query picks out a key column; values chosen so a transposed or mis-indexed operand fails
    d, n = 5, 7
    K = np.arange(n * d, dtype=np.float64).reshape(n, d) / 10.0
    V = np.eye(n, d) + 2.0
    q = np.zeros(d); q[3] = 2.0
    att = orc.entmax_attention(q, K, V, 1.5, 0.5)
    s = 0.5 * 2.0 * K[:, 3]
    np.testing.assert_allclose(att["s"], s, atol=1e-15)
    p_ref, _ = brute_force_entmax(s, 1.5)
    np.testing.assert_allclose(att["p"], p_ref, atol=1e-12)
    np.testing.assert_allclose(att["o"], sum(p_ref[j] * V[j] for j in range(n)), atol=1e-12)


def test_softmax_attention_output_is_p_times_v():
    # same construction for the softmax baseline: probabilities and log-sum-exp typed out term by term, and the
    # output as the explicit sum p_j v_j over a candidate subset (a transposed V, a sum over the wrong axis or
    # values taken from the wrong tokens all fail)
    d, n = 5, 7
    K = np.arange(n * d, dtype=np.float64).reshape(n, d) / 10.0
    V = np.eye(n, d) + 2.0 + np.arange(n)[:, None] * 0.25
    q = np.zeros(d); q[1] = -1.5
    tokens = np.array([6, 0, 3, 4])
    att = orc.softmax_attention(q, K, V, 0.5, tokens=tokens)
    s = [0.5 * -1.5 * K[j, 1] for j in tokens]
    z = sum(math.exp(x) for x in s)
    p_ref = [math.exp(x) / z for x in s]
    np.testing.assert_allclose(att["s"], s, atol=1e-15)
    np.testing.assert_allclose(att["p"], p_ref, atol=1e-15)
    assert abs(att["lse"] - math.log(z)) < 1e-14
    o_ref = np.zeros(d)
    for pj, j in zip(p_ref, tokens):
        o_ref += pj * V[j]
    np.testing.assert_allclose(att["o"], o_ref, atol=1e-14)
    # one candidate: its value row exactly
    one = orc.softmax_attention(q, K, V, 0.5, tokens=np.array([2]))
    np.testing.assert_array_equal(one["o"], V[2])


def test_relative_output_error_by_hand():
    # R = ||o - o~|| / ||o|| with the FULL-cache output in the denominator (App. E.1): o = (3, 4), o~ = (3, 0)
    o, ot = np.array([3.0, 4.0]), np.array([3.0, 0.0])
    assert orc.relative_output_error(o, ot) == pytest.approx(4.0 / 5.0, abs=1e-15)
    assert orc.relative_output_error(ot, o) == pytest.approx(4.0 / 3.0, abs=1e-15)     # not symmetric
    assert orc.relative_output_error(o, o) == 0.0
    assert orc.relative_output_error(np.array([0.0, 2.0, 0.0]), np.array([1.0, 2.0, 2.0])) == pytest.approx(math.sqrt(5.0) / 2.0)


def test_prop1_tightness_golden():
    """Prop. 1 tightness example (App. C): p=(1-delta, delta), v=+-B u, keep token 1 only."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "prop1_tightness.txt")) if l.strip() and l[0] != "#"]
    for delta, B, err in [(float(a), float(b), float(c)) for a, b, c in rows]:
        u = np.array([0.6, 0.8])
        V = np.array([B * u, -B * u])
        p = np.array([1.0 - delta, delta])
        o = p @ V
        o_t, dlt = orc.renormalised_truncation(p, V, [0])
        assert abs(dlt - delta) < 1e-15
        assert abs(np.linalg.norm(o - o_t) - err) < 1e-12
        np.testing.assert_allclose(o, (1 - 2 * delta) * B * u, atol=1e-12)
        np.testing.assert_allclose(o_t, B * u, atol=1e-12)


@pytest.mark.parametrize("alpha", [1.5, 2.0, 1.25])
def test_prop2_exact_when_support_kept_and_prop1_bound(alpha):
    rng = np.random.default_rng(21)
    n, d, P = 640, 16, 16
    q = rng.normal(size=d); K = rng.normal(size=(n, d)); V = rng.normal(size=(n, d))
    scale = 0.3
    full = orc.entmax_attention(q, K, V, alpha, scale)
    S = full["support"]
    assert 1 < len(S) < n // 4
    B = np.linalg.norm(V, axis=1).max()
    # (a) candidate pages = pages of the support plus some random ones: exact (Prop. 2)
    pages = np.union1d(np.unique(S // P), rng.choice(n // P, 5, replace=False))
    tok = orc.pages_to_tokens(pages, P, n)
    sp = orc.entmax_attention(q, K, V, alpha, scale, tok)
    assert abs(sp["tau"] - full["tau"]) < 1e-13
    np.testing.assert_allclose(sp["o"], full["o"], atol=1e-13)
    assert np.array_equal(sp["support"], S)
    assert orc.dropped_mass(full["p"], tok) == 0.0
    # (b) drop the page holding the heaviest token: tau drops, error bounded by 2 B delta (Prop. 1)
    heavy_page = int(np.argmax(full["p"])) // P
    pages_b = np.setdiff1d(pages, [heavy_page])
    tok_b = orc.pages_to_tokens(pages_b, P, n)
    sp_b = orc.entmax_attention(q, K, V, alpha, scale, tok_b)
    delta = orc.dropped_mass(full["p"], tok_b)
    assert delta > 0 and sp_b["tau"] < full["tau"]
    o_ren, delta2 = orc.renormalised_truncation(full["p"], V, tok_b)
    assert abs(delta - delta2) < 1e-15
    assert np.linalg.norm(full["o"] - o_ren) <= 2 * B * delta + 1e-12
    assert np.linalg.norm(full["o"] - sp_b["o"]) <= 2 * B * delta + 1e-12
    # delta from the full threshold alone: 1 - sum_{j in C} (z_j - tau_full)_+^beta
    a = alpha - 1.0
    z_c = a * scale * (K[tok_b] @ q)
    assert abs(delta - (1.0 - np.sum(np.maximum(z_c - full["tau"], 0) ** (1 / a)))) < 1e-12
    rho = orc.support_retention(S, tok_b)
    assert abs(rho - np.isin(S // P, pages_b).mean()) < 1e-15
    assert orc.relative_output_error(full["o"], full["o"]) == 0.0


def test_eq8_dropped_mass_decomposition():
    rng = np.random.default_rng(5)
    n, d = 400, 8
    q = rng.normal(size=d); K = rng.normal(size=(n, d)); V = rng.normal(size=(n, d))
    ent = orc.entmax_attention(q, K, V, 1.5, 1.0)
    sm = orc.softmax_attention(q, K, V, 1.0)
    keep = np.sort(rng.choice(n, 150, replace=False))
    drop = np.setdiff1d(np.arange(n), keep)
    S = ent["support"]
    d_sm = orc.dropped_mass(sm["p"], keep)
    d_ent = orc.dropped_mass(ent["p"], keep)
    in_S = np.isin(drop, S)
    miss = np.sum(sm["p"][drop[in_S]] - ent["p"][drop[in_S]])
    tail = np.sum(sm["p"][drop[~in_S]])
    assert abs((d_sm - d_ent) - (miss + tail)) < 1e-13
    assert abs(sm["p"].sum() - 1) < 1e-13
    # log-sum-exp is the softmax normaliser
    s = K @ q
    assert abs(sm["lse"] - np.log(np.exp(s).sum())) < 1e-12
