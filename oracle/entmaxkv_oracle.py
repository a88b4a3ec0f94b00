"""EntmaxKV decode path -- plain float64 CPU oracle.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import this module.  It shares nothing with the
HIP library: no kernels, headers, tables, helpers or constants.  Everything is
numpy float64, one (batch, query head) unit at a time, written straight from the
paper's definitions so that it can be checked against the paper by eye:

  stage 1  page statistics          Sec. 4.2 (page min/max; k_avg, m_2, k_std)
  stage 2  box page score           Sec. 4.2 Eq. 9, App. B.1
           8-bit page bounds        extension of Eq. 9 (bounds rounded outward to OCP E4M3)
           Gaussian page moments    Sec. 4.3 (mu_p, sigma_p^2)
  stage 3  top-k page selection     Sec. 4.3 "Top-k page selection"
           Gaussian tau-hat         Sec. 4.3 Eq. 10, App. D (truncated Gaussian moments)
           Gaussian page selection  Sec. 4.3 Eq. 11-12
           box-threshold selection  App. B.2 (support superset from page bounds)
  stage 4  entmax attention over a candidate token set (all tokens = full cache)
                                    Sec. 2.1 Eq. 1, Sec. 2.2 Eq. 2-3, Sec. 4.1
  metrics  delta, rho, R, softmax dropped mass   Sec. 3 Eq. 4, 7, 8; App. E.1

Exact pieces (statistics, box bound, top-k, entmax over a given set, delta/rho)
are the definition written out; the entmax threshold is found by sorting.  The
one heuristic piece (Gaussian tau-hat and page-max estimate) follows the paper's
steps, with the scalar root taken to float64 convergence by bisection.

Parity pins (tests/test_oracle_*.py): brute-force subset enumeration, sparsemax
closed form, softmax limit, normalisation, the tightness example of Prop. 1,
Prop. 2-4 invariants, P=1 reduction, printed truncated-moment closed forms vs
quadrature; box-threshold refinement: a worked example, the P=1 reduction and
"one refinement from any start reaches the full-cache result"; 8-bit bounds: the value
table against a library decoder, directed rounding by brute force over the table, a worked
example, and "8-bit score >= cache-dtype score >= largest token score"; the storage reading of the Gaussian
statistics (mean and VARIANCE rounded, k_std = root of the stored variance) against the library's bf16 cast on
hand-built values; the softmax baseline's output as the explicit sum p_j v_j; R on a hand-worked pair.  Unpinned: which pages a *good* Gaussian selector should pick
(selection quality; the paper states no hyper-parameters) -- "parity unpinned".
"""
import numpy as np
from scipy.special import ndtr, ndtri  # standard normal cdf and its inverse (library primitives)

_SQRT_2PI = np.sqrt(2.0 * np.pi)


# --------------------------------------------------------------------------------------
# storage rounding (what a cache-dtype copy of a float64 statistic holds)
# --------------------------------------------------------------------------------------
def round_to_bf16(x):
    """Round float64 to the nearest bfloat16 value (8 significand bits, ties to even).

    Returned as float64.  Normal range only (no bf16 subnormal handling)."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                      # x = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)   # np.rint rounds half to even


def stored_gauss_stats(kavg, kstd, kv_dtype):
    """(k_avg, k_std) as recovered from the statistics a cache-dtype store keeps.

    Storage reading (the paper does not fix a precision): the mean and the VARIANCE k_std^2 are kept,
    each rounded to the cache dtype; k_std is the square root of the stored variance."""
    kvar = round_to_storage(np.asarray(kstd, dtype=np.float64) ** 2, kv_dtype)
    return round_to_storage(kavg, kv_dtype), np.sqrt(kvar)


def round_to_storage(x, kv_dtype):
    """Value held by a statistic stored in the cache dtype ('f32' or 'bf16')."""
    if kv_dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)
    if kv_dtype == "bf16":
        return round_to_bf16(x)
    raise ValueError(kv_dtype)


# --------------------------------------------------------------------------------------
# stage 1: page statistics (Sec. 4.2)
# --------------------------------------------------------------------------------------
def page_stats(K, P):
    """Per-page key statistics of one (sequence, KV head).

    K: [n, d] keys of the n valid tokens in logical order.  Page p holds tokens
    [pP, min((p+1)P, n)); the last page may be partial and its statistics are over
    its cnt_p tokens only.  Population statistics (divide by cnt_p); a slightly
    negative m2 - avg^2 is clamped to 0 before the square root.
    Returns kmin, kmax, kavg, kstd: [M, d] and cnt: [M]."""
    K = np.asarray(K, dtype=np.float64)
    n, d = K.shape
    M = -(-n // P)
    kmin = np.empty((M, d)); kmax = np.empty((M, d))
    kavg = np.empty((M, d)); kstd = np.empty((M, d))
    cnt = np.empty(M, dtype=np.int64)
    for p in range(M):
        page = K[p * P:min((p + 1) * P, n)]
        cnt[p] = page.shape[0]
        kmin[p] = page.min(axis=0)
        kmax[p] = page.max(axis=0)
        kavg[p] = page.sum(axis=0) / cnt[p]
        m2 = (page * page).sum(axis=0) / cnt[p]
        kstd[p] = np.sqrt(np.maximum(m2 - kavg[p] * kavg[p], 0.0))
    return kmin, kmax, kavg, kstd, cnt


# --------------------------------------------------------------------------------------
# stage 2: page scoring
# --------------------------------------------------------------------------------------
def box_scores(q, kmin, kmax, scale):
    """Eq. 9 with 1/sqrt(d) generalised to `scale`: upper bound of scale*q.k over a page."""
    q = np.asarray(q, dtype=np.float64)
    return scale * np.maximum(q[None, :] * kmin, q[None, :] * kmax).sum(axis=1)


def gauss_moments(q, kavg, kstd, scale):
    """Sec. 4.3: mu_p = scale*q.k_avg ; sigma_p^2 = scale^2 * sum_i q_i^2 k_std,i^2.

    Returns (mu, sigma), sigma >= 0."""
    q = np.asarray(q, dtype=np.float64)
    mu = scale * (kavg @ q)
    var = scale * scale * ((kstd * kstd) @ (q * q))
    return mu, np.sqrt(var)


# --------------------------------------------------------------------------------------
# stage 1'/2': 8-bit page bounds (an extension: the paper keeps its metadata in the cache dtype)
# --------------------------------------------------------------------------------------
# Eq. 9 stays an upper bound of scale*q.k over the page as long as the stored k_min is not above the
# true minimum and the stored k_max not below the true maximum (App. B.1's argument uses nothing
# else).  The bounds can therefore be kept in any coarser number format if k_min is rounded DOWN and
# k_max UP to that format.  Format here: the 8-bit float E4M3 of the OCP 8-bit floating point
# specification (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; subnormals; no infinities;
# the all-ones exponent-and-mantissa code is NaN; largest finite value 448).
def e4m3_grid():
    """Every finite E4M3 value, ascending (253 distinct values, -448 .. 448), from the format's
    definition: code (e, m) is (m/8) * 2^-6 for e = 0, else (1 + m/8) * 2^(e-7); (15, 7) is NaN."""
    pos = []
    for e in range(16):
        for m in range(8):
            if e == 15 and m == 7:
                continue
            pos.append((m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    pos = np.array(pos, dtype=np.float64)
    return np.concatenate([-pos[:0:-1], pos])


def round_e4m3(x, direction):
    """Directed rounding to E4M3: 'down' = the largest finite format value <= x, 'up' = the smallest
    >= x.  NaN where no such value exists (x > 448 rounding up, x < -448 rounding down) or x is NaN."""
    grid = e4m3_grid()
    x = np.asarray(x, dtype=np.float64)
    out = np.full(x.shape, np.nan)
    ok = ~np.isnan(x)
    if direction == "down":
        i = np.searchsorted(grid, x[ok], side="right") - 1          # last grid value <= x
        vals = np.where(i >= 0, grid[np.maximum(i, 0)], np.nan)
    elif direction == "up":
        i = np.searchsorted(grid, x[ok], side="left")               # first grid value >= x
        vals = np.where(i < len(grid), grid[np.minimum(i, len(grid) - 1)], np.nan)
    else:
        raise ValueError(direction)
    out[ok] = vals
    return out


def box8_stats(kmin, kmax):
    """8-bit page bounds: (k_min rounded down, k_max rounded up), as float64 (NaN = not representable)."""
    return round_e4m3(kmin, "down"), round_e4m3(kmax, "up")


def box8_scores(q, lo8, hi8, scale):
    """Eq. 9 on the 8-bit bounds.  A page with a bound that the format cannot hold (NaN) gets +inf:
    it is always selected, which keeps the score an upper bound."""
    bad = np.isnan(lo8).any(axis=1) | np.isnan(hi8).any(axis=1)
    s = box_scores(q, np.nan_to_num(lo8), np.nan_to_num(hi8), scale)
    return np.where(bad, np.inf, s)


# --------------------------------------------------------------------------------------
# stage 3a: top-k pages (Sec. 4.3)
# --------------------------------------------------------------------------------------
def topk_pages(scores, k):
    """Indices of the k largest scores; equal scores: lower page index wins.

    Returns (ascending index array of min(k, M) pages, score of the last page
    taken, score of the best page left out or -inf)."""
    scores = np.asarray(scores, dtype=np.float64)
    M = scores.shape[0]
    k = min(int(k), M)
    order = np.lexsort((np.arange(M), -scores))     # score descending, then index ascending
    taken = order[:k]
    cut_in = scores[taken[-1]] if k > 0 else np.inf
    cut_out = scores[order[k]] if k < M else -np.inf
    return np.sort(taken), cut_in, cut_out


# --------------------------------------------------------------------------------------
# stage 3a': one page list per KV head, shared by the G query heads of its group
# --------------------------------------------------------------------------------------
def group_max_scores(box_heads):
    """Page score of a KV-head group: the maximum over its query heads' box scores.

    box_heads [G, M].  The paper selects "for each attention head" and does not treat
    grouped-query attention; sharing one list per KV head is this repository's
    variant.  The maximum keeps the bound of Sec. 4.2 Eq. 9 valid for every head of
    the group (it is >= each head's own bound), so the exact-recovery and
    box-threshold statements carry over head by head."""
    return np.max(np.asarray(box_heads, dtype=np.float64), axis=0)


# --------------------------------------------------------------------------------------
# stage 3c: box-threshold selection (App. B.2, the proposition on page bounds)
# --------------------------------------------------------------------------------------
def box_threshold_pages(box, alpha, tau_lo):
    """Pages p with (alpha-1) * box_p > tau_lo, ascending.

    App. B.2: if tau_lo does not exceed the exact entmax threshold, every page that
    holds a support token is in this set (the box score bounds every token score of
    the page from above)."""
    box = np.asarray(box, dtype=np.float64)
    return np.nonzero((alpha - 1.0) * box > tau_lo)[0]


def refine_selection(box, alpha, tau_lo, pages):
    """Union of a page list with box_threshold_pages(box, alpha, tau_lo).

    Returns (ascending union, ascending array of the pages that were added).  With
    tau_lo the threshold of the sparse solve over `pages` (never above the
    full-cache threshold, since dropping candidates only lowers the mass), an empty
    `added` certifies that the sparse result is exact, and otherwise the union
    holds the whole support, so one more sparse solve over it is exact (Prop. 2)."""
    pages = np.asarray(pages, dtype=np.int64)
    thr = box_threshold_pages(box, alpha, tau_lo)
    added = np.setdiff1d(thr, pages)
    return np.union1d(pages, thr), added


# --------------------------------------------------------------------------------------
# stage 3b: Gaussian-aware selector (Sec. 4.3 Eq. 10-12, App. D)
# --------------------------------------------------------------------------------------
def trunc_gauss_moment(order, mu_y, sig_y):
    """E[(Y)_+^order] for Y ~ N(mu_y, sig_y^2), integer order >= 0 (App. D).

    M_0 = Phi(t), M_1 = mu Phi(t) + sig phi(t), M_n = mu M_{n-1} + (n-1) sig^2 M_{n-2},
    t = mu/sig.  The recurrence follows from integrating y^n phi by parts; for n=1,2,3
    it reproduces the three closed forms printed in App. D.  sig = 0: (mu)_+^n."""
    mu_y = np.asarray(mu_y, dtype=np.float64)
    sig_y = np.asarray(sig_y, dtype=np.float64)
    mu_y, sig_y = np.broadcast_arrays(mu_y, sig_y)
    pos = sig_y > 0.0
    safe_sig = np.where(pos, sig_y, 1.0)
    t = mu_y / safe_sig
    cdf = ndtr(t)
    pdf = np.exp(-0.5 * t * t) / _SQRT_2PI
    m_prev = cdf                                   # M_0
    if order == 0:
        m = m_prev
    else:
        m = mu_y * cdf + safe_sig * pdf            # M_1
        for n in range(2, order + 1):
            m, m_prev = mu_y * m + (n - 1) * safe_sig * safe_sig * m_prev, m
    degenerate = np.maximum(mu_y, 0.0) ** order if order > 0 else (mu_y > 0).astype(np.float64)
    return np.where(pos, m, degenerate)


def gauss_mass(tau, mu, sigma, cnt, alpha):
    """Left side of Eq. 10: sum_p cnt_p E[g_alpha(S_p; tau)], S_p ~ N(mu_p, sigma_p^2)."""
    a = alpha - 1.0
    beta = int(round(1.0 / a))
    if abs(beta * a - 1.0) > 1e-12:
        raise ValueError("closed-form Gaussian moments need integer 1/(alpha-1)")
    return float(np.sum(cnt * trunc_gauss_moment(beta, a * mu - tau, a * sigma)))


def gauss_tau_hat(mu, sigma, cnt, alpha):
    """Root tau-hat of Eq. 10, to float64 convergence.

    The left side is continuous and strictly decreasing in tau wherever positive.
    At tau = a*mu_max - 1 it is >= 1 (Jensen: cnt*E[(Y)_+^beta] >= cnt*(E Y)_+^beta = cnt >= 1
    for the page of largest mean), so that is a valid left end; the right end is found
    by doubling; then plain bisection."""
    a = alpha - 1.0
    lo = a * float(np.max(mu)) - 1.0
    step = 1.0
    hi = lo + step
    while gauss_mass(hi, mu, sigma, cnt, alpha) >= 1.0:
        step *= 2.0
        hi = lo + step
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if mid <= lo or mid >= hi:
            break
        if gauss_mass(mid, mu, sigma, cnt, alpha) >= 1.0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def gauss_page_max(mu, sigma, cnt, q_page):
    """Eq. 11: q_page-confidence estimate of the largest score in each page."""
    zq = ndtri(np.power(q_page, 1.0 / np.asarray(cnt, dtype=np.float64)))
    return mu + sigma * zq


def gauss_select(mu, sigma, cnt, alpha, q_page, margin, tau_hat=None, cap=None):
    """Eq. 12: pages with (alpha-1)*s_Gauss > tau_hat - margin, ascending.

    Readings where the paper is silent: an empty result is replaced by the single page
    of largest s_Gauss (lowest index on ties); more than `cap` pages keeps the `cap`
    largest s_Gauss (lower index first on ties) and reports overflow.
    Returns (pages, tau_hat, overflow, a*s_Gauss)."""
    a = alpha - 1.0
    if tau_hat is None:
        tau_hat = gauss_tau_hat(mu, sigma, cnt, alpha)
    g = a * gauss_page_max(mu, sigma, cnt, q_page)
    pages = np.nonzero(g > tau_hat - margin)[0]
    overflow = False
    if pages.size == 0:
        pages = np.array([int(np.lexsort((np.arange(g.size), -g))[0])])
    if cap is not None and pages.size > cap:
        overflow = True
        order = np.lexsort((pages, -g[pages]))
        pages = np.sort(pages[order[:cap]])
    return pages, tau_hat, overflow, g


# --------------------------------------------------------------------------------------
# stage 4: alpha-entmax (Sec. 2.2 Eq. 2-3, App. A)
# --------------------------------------------------------------------------------------
def _mass_above(z_sorted, tau, beta):
    """sum_j (z_j - tau)_+^beta"""
    return float(np.sum(np.maximum(z_sorted - tau, 0.0) ** beta))


def entmax_threshold(z, alpha):
    """Exact threshold of alpha-entmax for z = (alpha-1)*s, by sorting.

    With z_(1) >= z_(2) >= ... the support is the k* largest entries where k* is the
    number of k such that sum_{j<=k} (z_(j) - z_(k))^beta < 1 (the k-th entry still has
    positive probability when the threshold sits at it; the left side is non-decreasing
    in k).  tau is the root of sum_{j<=k*} (z_(j) - tau)^beta = 1 below z_(k*):
    closed form for beta=1 and beta=2, bisection on the fixed support otherwise.
    Returns (tau, k*)."""
    z = np.asarray(z, dtype=np.float64)
    beta = 1.0 / (alpha - 1.0)
    zs = np.sort(z)[::-1]
    n = zs.size
    # largest k with mass(z_(k)) < 1 ; mass(z_(k)) is non-decreasing in k -> binary search
    lo, hi = 1, n                                   # k=1 always qualifies (mass 0)
    while lo < hi:
        mid = (lo + hi + 1) // 2
        if _mass_above(zs[:mid], zs[mid - 1], beta) < 1.0:
            lo = mid
        else:
            hi = mid - 1
    k = lo
    top = zs[:k]
    if abs(beta - 1.0) < 1e-15:
        tau = (top.sum() - 1.0) / k
    elif abs(beta - 2.0) < 1e-15:
        mean = top.sum() / k
        ss = np.sum((top - mean) ** 2)
        tau = mean - np.sqrt(max(1.0 - ss, 0.0) / k)
    else:
        # the root lies in [z_(k) - 1, z_(k)): at z_(k) - 1 the k-th term alone gives 1
        t_lo, t_hi = top[-1] - 1.0, top[-1]
        for _ in range(200):
            mid = 0.5 * (t_lo + t_hi)
            if mid <= t_lo or mid >= t_hi:
                break
            if np.sum((top - mid) ** beta) >= 1.0:
                t_lo = mid
            else:
                t_hi = mid
        tau = 0.5 * (t_lo + t_hi)
    return float(tau), int(k)


def entmax_probs(s, alpha):
    """alpha-entmax of a score vector s (Eq. 2): p, tau, support mask (strict >, Eq. 3)."""
    a = alpha - 1.0
    z = a * np.asarray(s, dtype=np.float64)
    tau, _ = entmax_threshold(z, alpha)
    p = np.maximum(z - tau, 0.0) ** (1.0 / a)
    return p, tau, z > tau


def token_scores(q, K, scale):
    """s_j = scale * q.k_j (Eq. 1 with 1/sqrt(d) -> scale)."""
    return scale * (np.asarray(K, dtype=np.float64) @ np.asarray(q, dtype=np.float64))


def entmax_attention(q, K, V, alpha, scale, tokens=None):
    """Entmax attention of one head over the candidate token set (Sec. 4.1).

    tokens: ascending indices into K/V rows; None = the full cache.  The threshold is
    re-solved on the candidates (the method of Sec. 4.1, not the renormalised
    truncation of Sec. 3).  Returns dict(o, tau, p (over the candidate list), support
    (token indices with p>0), s (candidate scores))."""
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    if tokens is None:
        tokens = np.arange(K.shape[0])
    tokens = np.asarray(tokens, dtype=np.int64)
    s = token_scores(q, K[tokens], scale)
    p, tau, mask = entmax_probs(s, alpha)
    o = p @ V[tokens]
    return {"o": o, "tau": tau, "p": p, "support": tokens[mask], "s": s, "tokens": tokens}


def pages_to_tokens(pages, P, n):
    """Token indices (ascending) covered by the given pages, cut at n."""
    pages = np.sort(np.asarray(pages, dtype=np.int64))
    tok = (pages[:, None] * P + np.arange(P)[None, :]).reshape(-1)
    return tok[tok < n]


def softmax_attention(q, K, V, scale, tokens=None):
    """Softmax attention over the candidate set (the sparse softmax baseline, App. E.1)."""
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    if tokens is None:
        tokens = np.arange(K.shape[0])
    s = token_scores(q, K[tokens], scale)
    m = s.max()
    e = np.exp(s - m)
    p = e / e.sum()
    return {"o": p @ V[tokens], "p": p, "lse": m + np.log(e.sum()), "s": s}


# --------------------------------------------------------------------------------------
# metrics (Sec. 3)
# --------------------------------------------------------------------------------------
def dropped_mass(p_full, keep_tokens):
    """Eq. 4: full-cache probability outside the kept set."""
    keep = np.zeros(p_full.shape[0], dtype=bool)
    keep[np.asarray(keep_tokens, dtype=np.int64)] = True
    return float(p_full[~keep].sum())


def support_retention(support_full, keep_tokens):
    """Eq. 7: |S n keep| / |S|"""
    return float(np.isin(support_full, keep_tokens).sum()) / float(len(support_full))


def relative_output_error(o_full, o_sparse):
    """R = ||o - o~||_2 / ||o||_2 (App. E.1)"""
    return float(np.linalg.norm(o_full - o_sparse) / np.linalg.norm(o_full))


def renormalised_truncation(p_full, V, keep_tokens):
    """Sec. 3.1: p~_i = p_i/(1-delta) on the kept set, 0 elsewhere; returns (o~, delta)."""
    keep = np.zeros(p_full.shape[0], dtype=bool)
    keep[np.asarray(keep_tokens, dtype=np.int64)] = True
    delta = float(p_full[~keep].sum())
    pt = np.where(keep, p_full / (1.0 - delta), 0.0)
    return pt @ np.asarray(V, dtype=np.float64), delta


# --------------------------------------------------------------------------------------
# one whole decode step for one (batch, query head) unit
# --------------------------------------------------------------------------------------
def decode_step_unit(q, K, V, P, alpha, scale, selector, kv_dtype="f32",
                     k_pages=None, q_page=0.99, margin=0.0, cap=None):
    """Stats -> score -> select -> sparse entmax attention for one head.

    q [d], K,V [n,d] (already the exact stored cache values, widened to float64).
    selector: 'topk' (box bound, k_pages) or 'gauss' (tau-hat, adaptive).  The page
    statistics used for scoring are the values a cache-dtype copy would hold
    (min/max are cache values already; mean and variance are rounded to kv_dtype)."""
    n = K.shape[0]
    kmin, kmax, kavg, kstd, cnt = page_stats(K, P)
    out = {}
    if selector == "topk":
        box = box_scores(q, kmin, kmax, scale)
        pages, cut_in, cut_out = topk_pages(box, k_pages)
        out.update(box=box, cut_in=cut_in, cut_out=cut_out)
    elif selector == "gauss":
        kavg_s, kstd_s = stored_gauss_stats(kavg, kstd, kv_dtype)
        mu, sigma = gauss_moments(q, kavg_s, kstd_s, scale)
        pages, tau_hat, overflow, g = gauss_select(mu, sigma, cnt, alpha, q_page, margin, cap=cap)
        out.update(mu=mu, sigma=sigma, tau_hat=tau_hat, overflow=overflow, g=g)
    else:
        raise ValueError(selector)
    tokens = pages_to_tokens(pages, P, n)
    att = entmax_attention(q, K, V, alpha, scale, tokens)
    out.update(pages=pages, tokens=tokens, **{k: att[k] for k in ("o", "tau", "support", "p")})
    return out
