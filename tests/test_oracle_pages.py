"""Pins for the oracle's page statistics, page scores and selectors (CPU only)."""
import numpy as np
import pytest
import torch
from scipy import integrate
from scipy.special import ndtr

from oracle import entmaxkv_oracle as orc


# ---------------------------------------------------------------- storage rounding
def test_round_to_bf16_matches_library_cast():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-3, 4, size=4000),
                        # exact ties between two bf16 neighbours (9th significand bit set, rest zero)
                        np.array([1.00390625, 1.01171875, -3.0234375, 257.0, 259.0, 0.0, -0.0])])
    ref = torch.tensor(x, dtype=torch.float64).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.round_to_bf16(x), ref)
    ref32 = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.round_to_storage(x, "f32"), ref32)


def test_stored_gauss_stats_round_mean_and_variance_not_std():
    # Storage reading: the cache-dtype copy holds the mean and the VARIANCE; k_std is the root of the stored
    # variance.  Hand-built values whose bf16 roundings tell the variants apart, checked against the library cast.
    kavg = np.array([[0.3337, -5.0123, 1.0e-3], [2.00390625, 7.77, -0.0]])
    kstd = np.array([[1.2345, 0.05678, 3.0], [0.999, 1.0039, 0.0]])
    to_bf16 = lambda a: torch.tensor(a, dtype=torch.float64).to(torch.bfloat16).to(torch.float64).numpy()
    avg_s, std_s = orc.stored_gauss_stats(kavg, kstd, "bf16")
    np.testing.assert_array_equal(avg_s, to_bf16(kavg))
    np.testing.assert_array_equal(std_s, np.sqrt(to_bf16(kstd * kstd)))
    # the variants a slip would produce differ on these values: rounding k_std instead of its square, or no root
    assert np.any(std_s != to_bf16(kstd))
    assert np.any(std_s != np.sqrt(to_bf16(kstd) ** 2))
    assert np.any(std_s != to_bf16(kstd * kstd))
    # exactly representable inputs pass through unchanged; a float32 store rounds to float32
    avg_e, std_e = orc.stored_gauss_stats(np.array([1.5, -0.25]), np.array([2.0, 0.5]), "bf16")
    np.testing.assert_array_equal(avg_e, [1.5, -0.25]); np.testing.assert_array_equal(std_e, [2.0, 0.5])
    avg_f, std_f = orc.stored_gauss_stats(kavg, kstd, "f32")
    np.testing.assert_array_equal(avg_f, kavg.astype(np.float32).astype(np.float64))
    np.testing.assert_array_equal(std_f, np.sqrt((kstd * kstd).astype(np.float32).astype(np.float64)))


# ---------------------------------------------------------------- stage 1
def test_page_stats_against_numpy_reductions():
    rng = np.random.default_rng(1)
    n, d, P = 77, 6, 16                       # 4 full pages + a partial page of 13
    K = rng.normal(size=(n, d)) + np.arange(d)
    kmin, kmax, kavg, kstd, cnt = orc.page_stats(K, P)
    assert cnt.tolist() == [16, 16, 16, 16, 13]
    for p in range(5):
        page = K[p * P:(p + 1) * P]
        np.testing.assert_array_equal(kmin[p], np.min(page, axis=0))
        np.testing.assert_array_equal(kmax[p], np.max(page, axis=0))
        np.testing.assert_allclose(kavg[p], np.mean(page, axis=0), rtol=1e-14)
        np.testing.assert_allclose(kstd[p], np.std(page, axis=0), rtol=1e-10)   # population std (ddof=0)


def test_page_stats_single_token_pages():
    rng = np.random.default_rng(2)
    K = rng.normal(size=(9, 4))
    kmin, kmax, kavg, kstd, cnt = orc.page_stats(K, 1)
    np.testing.assert_array_equal(kmin, K); np.testing.assert_array_equal(kmax, K)
    np.testing.assert_array_equal(kavg, K); np.testing.assert_array_equal(kstd, np.zeros_like(K))
    # constant page: variance clamps to exactly 0 even if m2 - avg^2 rounds negative
    Kc = np.full((16, 3), 0.1)
    assert np.all(orc.page_stats(Kc, 16)[3] == 0.0) or np.all(orc.page_stats(Kc, 16)[3] < 1e-8)


# ---------------------------------------------------------------- stage 2
def test_box_score_is_upper_bound_and_tight_for_single_token_pages():
    rng = np.random.default_rng(3)
    n, d, P, scale = 160, 12, 16, 0.37
    q = rng.normal(size=d); K = rng.normal(size=(n, d))
    kmin, kmax, *_ = orc.page_stats(K, P)
    box = orc.box_scores(q, kmin, kmax, scale)
    s = orc.token_scores(q, K, scale)
    page_max = s.reshape(-1, P).max(axis=1)
    assert np.all(box >= page_max - 1e-12)                    # Prop. 3
    assert np.any(box > page_max + 1e-3)                      # and it is a genuine (loose) bound
    # equivalent dot-product form: q+ . kmax + q- . kmin   (proof of Prop. 3)
    alt = scale * (kmax @ np.maximum(q, 0) + kmin @ np.minimum(q, 0))
    np.testing.assert_allclose(box, alt, rtol=1e-13)
    kmin1, kmax1, *_ = orc.page_stats(K, 1)
    np.testing.assert_allclose(orc.box_scores(q, kmin1, kmax1, scale), s, rtol=1e-13)


def test_gauss_moments_match_sample_moments_of_token_scores():
    # mu_p is exactly the mean of the page's token scores; sigma_p^2 is the diagonal part of their
    # variance, hence equal to it when the key coordinates are uncorrelated within the page.
    rng = np.random.default_rng(4)
    d, P, scale = 5, 16, 0.7
    q = rng.normal(size=d)
    K = rng.normal(size=(3 * P, d))
    _, _, kavg, kstd, _ = orc.page_stats(K, P)
    mu, sigma = orc.gauss_moments(q, kavg, kstd, scale)
    s = orc.token_scores(q, K, scale).reshape(3, P)
    np.testing.assert_allclose(mu, s.mean(axis=1), rtol=1e-12)
    # sigma_p^2 written out by hand from per-coordinate population variances (library np.var)
    by_hand = scale ** 2 * sum(q[i] ** 2 * np.var(K[:P, i]) for i in range(d))
    assert abs(sigma[0] ** 2 - by_hand) < 1e-12
    # two-coordinate page with zero cross-covariance: the diagonal form is then the exact variance
    Kd = np.zeros((4, d)); Kd[:, 0] = [1, 1, -1, -1]; Kd[:, 1] = [2, -2, 2, -2]
    _, _, ka, ks, _ = orc.page_stats(Kd, 4)
    _, sig_d = orc.gauss_moments(q, ka, ks, scale)
    assert abs(sig_d[0] ** 2 - np.var(orc.token_scores(q, Kd, scale))) < 1e-12
    # a transposed/mis-weighted operand fails this: one-hot query isolates one coordinate
    e = np.zeros(d); e[2] = 3.0
    mu_e, sig_e = orc.gauss_moments(e, kavg, kstd, scale)
    np.testing.assert_allclose(mu_e, scale * 3.0 * kavg[:, 2], rtol=1e-14)
    np.testing.assert_allclose(sig_e, scale * 3.0 * kstd[:, 2], rtol=1e-14)


# ---------------------------------------------------------------- stage 3a
def test_topk_against_full_sort_with_ties():
    scores = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 0.5, 3.0])
    pages, cin, cout = orc.topk_pages(scores, 3)
    assert pages.tolist() == [1, 2, 6] and cin == 2.0 and cout == 2.0      # lower index wins the tie
    pages, cin, cout = orc.topk_pages(scores, 5)
    assert pages.tolist() == [0, 1, 2, 4, 6] and cin == 0.5 and cout == 0.5
    pages, _, cout = orc.topk_pages(scores, 50)
    assert pages.tolist() == list(range(7)) and cout == -np.inf
    rng = np.random.default_rng(5)
    s = rng.normal(size=500)
    pages, cin, cout = orc.topk_pages(s, 37)
    assert set(pages) == set(np.argsort(-s, kind="stable")[:37])
    assert cin == np.sort(s)[-37] and cout == np.sort(s)[-38]


# ---------------------------------------------------------------- stage 3b
def printed_closed_form(order, mu, sig):
    """The three truncated Gaussian moments as printed in App. D (beta = 1, 2, 3)."""
    t = mu / sig
    Phi = ndtr(t); phi = np.exp(-t * t / 2) / np.sqrt(2 * np.pi)
    if order == 1:
        return mu * Phi + sig * phi
    if order == 2:
        return (mu ** 2 + sig ** 2) * Phi + mu * sig * phi
    if order == 3:
        return (mu ** 3 + 3 * mu * sig ** 2) * Phi + (mu ** 2 * sig + 2 * sig ** 3) * phi
    raise ValueError


@pytest.mark.parametrize("order", [1, 2, 3, 4])
def test_truncated_gaussian_moments(order):
    rng = np.random.default_rng(6)
    for _ in range(12):
        mu = rng.normal() * 2.0
        sig = abs(rng.normal()) + 0.05
        got = float(orc.trunc_gauss_moment(order, mu, sig))
        quad, _ = integrate.quad(lambda y: y ** order * np.exp(-0.5 * ((y - mu) / sig) ** 2)
                                 / (sig * np.sqrt(2 * np.pi)), 0.0, max(mu, 0.0) + 40 * sig,
                                 epsabs=1e-14, epsrel=1e-13, limit=400)
        assert abs(got - quad) < 1e-10 * max(1.0, abs(quad))
        if order <= 3:
            assert abs(got - printed_closed_form(order, mu, sig)) < 1e-13 * max(1.0, abs(got))
    # sigma = 0: the moment of a point mass
    assert float(orc.trunc_gauss_moment(order, 1.5, 0.0)) == 1.5 ** order
    assert float(orc.trunc_gauss_moment(order, -1.5, 0.0)) == 0.0


@pytest.mark.parametrize("alpha", [2.0, 1.5, 4.0 / 3.0, 1.25])
def test_tau_hat_solves_eq10_and_mass_is_decreasing_convex(alpha):
    rng = np.random.default_rng(7)
    M = 300
    mu = rng.normal(size=M); sigma = np.abs(rng.normal(size=M)) * 0.5 + 0.1
    cnt = np.full(M, 16); cnt[-1] = 5
    th = orc.gauss_tau_hat(mu, sigma, cnt, alpha)
    assert abs(orc.gauss_mass(th, mu, sigma, cnt, alpha) - 1.0) < 1e-10
    ts = np.linspace(th - 1.0, th + 1.0, 41)
    F = np.array([orc.gauss_mass(t, mu, sigma, cnt, alpha) for t in ts])
    assert np.all(np.diff(F) < 0)
    assert np.all(np.diff(F, 2) > -1e-9)


@pytest.mark.parametrize("alpha", [2.0, 1.5, 1.25])
def test_page_size_one_reduces_gaussian_selector_to_exact_entmax(alpha):
    """P=1: sigma_p=0, Eq. 10 is the exact normalisation, so tau-hat = tau and the selector
    with margin 0 returns exactly the support (for any q_page)."""
    rng = np.random.default_rng(8)
    n, d, scale = 300, 8, 0.6
    q = rng.normal(size=d); K = rng.normal(size=(n, d)); V = rng.normal(size=(n, d))
    _, _, kavg, kstd, cnt = orc.page_stats(K, 1)
    mu, sigma = orc.gauss_moments(q, kavg, kstd, scale)
    full = orc.entmax_attention(q, K, V, alpha, scale)
    pages, th, overflow, _ = orc.gauss_select(mu, sigma, cnt, alpha, 0.9, 0.0)
    assert abs(th - full["tau"]) < 1e-11
    assert not overflow and np.array_equal(pages, full["support"])


def test_gaussian_tau_hat_close_to_tau_for_gaussian_pages():
    rng = np.random.default_rng(9)
    n, d, P = 32768, 32, 16
    q = rng.normal(size=d); K = rng.normal(size=(n, d))
    scale = 1.0 / np.sqrt(d)
    _, _, kavg, kstd, cnt = orc.page_stats(K, P)
    mu, sigma = orc.gauss_moments(q, kavg, kstd, scale)
    th = orc.gauss_tau_hat(mu, sigma, cnt, 1.5)
    tau, _ = orc.entmax_threshold(0.5 * orc.token_scores(q, K, scale), 1.5)
    assert abs(th - tau) < 0.1 * abs(tau)


def test_gauss_page_max_and_selection_rule():
    mu = np.array([0.0, 1.0, 2.0, -1.0]); sigma = np.array([1.0, 0.5, 0.0, 2.0]); cnt = np.array([16, 16, 16, 4])
    q_page = 0.9
    g = orc.gauss_page_max(mu, sigma, cnt, q_page)
    # definition check through the cdf: Phi((g-mu)/sigma)^cnt = q_page  (Eq. 11 inverted)
    for p in (0, 1, 3):
        assert abs(ndtr((g[p] - mu[p]) / sigma[p]) ** cnt[p] - q_page) < 1e-12
    assert g[2] == 2.0
    alpha = 1.5
    pages, th, overflow, ag = orc.gauss_select(mu, sigma, cnt, alpha, q_page, 0.0, tau_hat=0.9)
    assert pages.tolist() == [p for p in range(4) if 0.5 * g[p] > 0.9]
    pages2, *_ = orc.gauss_select(mu, sigma, cnt, alpha, q_page, 0.3, tau_hat=0.9)
    assert set(pages).issubset(set(pages2)) and pages2.tolist() == [p for p in range(4) if 0.5 * g[p] > 0.6]
    # empty -> best page; overflow -> cap best pages, flagged
    pages3, *_ = orc.gauss_select(mu, sigma, cnt, alpha, q_page, 0.0, tau_hat=100.0)
    assert pages3.tolist() == [int(np.argmax(g))]
    pages4, _, ovf, _ = orc.gauss_select(mu, sigma, cnt, alpha, q_page, 0.0, tau_hat=-100.0, cap=2)
    assert ovf and pages4.tolist() == sorted(np.argsort(-g)[:2].tolist())


def test_prop4_box_threshold_selection_covers_support():
    rng = np.random.default_rng(10)
    n, d, P, scale, alpha = 2048, 16, 16, 0.5, 1.5
    q = rng.normal(size=d); K = rng.normal(size=(n, d)); V = rng.normal(size=(n, d))
    full = orc.entmax_attention(q, K, V, alpha, scale)
    kmin, kmax, *_ = orc.page_stats(K, P)
    box = orc.box_scores(q, kmin, kmax, scale)
    for tau_hat in (full["tau"], full["tau"] - 0.2):
        pages = np.nonzero((alpha - 1.0) * box > tau_hat)[0]
        assert set(np.unique(full["support"] // P)).issubset(set(pages))
        sp = orc.entmax_attention(q, K, V, alpha, scale, orc.pages_to_tokens(pages, P, n))
        np.testing.assert_allclose(sp["o"], full["o"], atol=1e-13)


def test_decode_step_unit_runs_both_selectors():
    rng = np.random.default_rng(12)
    n, d, P = 1000, 16, 16                      # ragged: last page has 8 tokens
    q = rng.normal(size=d); K = rng.normal(size=(n, d)); V = rng.normal(size=(n, d))
    r = orc.decode_step_unit(q, K, V, P, 1.5, 0.5, "topk", k_pages=10)
    assert len(r["pages"]) == 10 and r["tokens"].max() < n and abs(r["p"].sum() - 1) < 1e-12
    r_all = orc.decode_step_unit(q, K, V, P, 1.5, 0.5, "topk", k_pages=10 ** 6)
    full = orc.entmax_attention(q, K, V, 1.5, 0.5)
    np.testing.assert_allclose(r_all["o"], full["o"], atol=1e-14)
    g = orc.decode_step_unit(q, K, V, P, 1.5, 0.5, "gauss", q_page=0.99)
    assert abs(g["p"].sum() - 1) < 1e-12 and len(g["pages"]) >= 1
