"""Pins of the oracle's box-threshold selection and refinement (App. B.2) against what the paper and
the mathematics fix: a hand-worked example, the P=1 reduction, the superset property for every
conservative threshold, and exactness after one refinement from an arbitrary starting selection."""
import os
import numpy as np
import pytest

from oracle import entmaxkv_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "box_threshold_example.txt")


def _unit(seed, n=512, P=16, d=32, alpha=1.5, scale=0.6, planted=6):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal(d)
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    idx = rng.choice(n, planted, replace=False)
    K[idx] = 2.0 * q / np.linalg.norm(q) + 0.3 * rng.standard_normal((planted, d))
    kmin, kmax, *_ = orc.page_stats(K, P)
    box = orc.box_scores(q, kmin, kmax, scale)
    return q, K, V, box


def test_hand_worked_example():
    """tests/golden/box_threshold_example.txt: four pages, alpha = 1.5, written out by hand."""
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    vals = {r[0]: [float(x) for x in r[1:]] for r in rows}
    alpha, tau_lo = vals["alpha"][0], vals["tau_lo"][0]
    got = orc.box_threshold_pages(np.array(vals["box"]), alpha, tau_lo)
    assert got.tolist() == [int(x) for x in vals["pages"]]
    union, added = orc.refine_selection(np.array(vals["box"]), alpha, tau_lo, [int(x) for x in vals["start"]])
    assert union.tolist() == [int(x) for x in vals["union"]]
    assert added.tolist() == [int(x) for x in vals["added"]]


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
def test_page_size_one_reduces_to_the_support(alpha):
    """P = 1: the box score of a page is its token's score, so thresholding at the exact tau returns
    exactly the support, and at any lower value a superset of it."""
    rng = np.random.default_rng(3)
    q, K = rng.standard_normal(16), rng.standard_normal((200, 16))
    V = rng.standard_normal((200, 16))
    ref = orc.entmax_attention(q, K, V, alpha, 0.7)
    kmin, kmax, *_ = orc.page_stats(K, 1)
    box = orc.box_scores(q, kmin, kmax, 0.7)
    assert np.allclose(box, ref["s"], rtol=0, atol=1e-12)
    # the oracle's tau is the root to rounding; step just below every score it separates
    got = orc.box_threshold_pages(box, alpha, ref["tau"])
    assert got.tolist() == ref["support"].tolist()
    lower = orc.box_threshold_pages(box, alpha, ref["tau"] - 0.05)
    assert set(ref["support"].tolist()) <= set(lower.tolist())
    z = (alpha - 1.0) * ref["s"]
    assert orc.box_threshold_pages(box, alpha, ref["tau"] - 1.0).tolist() == np.nonzero(z > ref["tau"] - 1.0)[0].tolist()


@pytest.mark.parametrize("seed", range(6))
def test_conservative_threshold_never_misses_a_support_page(seed):
    q, K, V, box = _unit(seed)
    alpha, scale, P = 1.5, 0.6, 16
    ref = orc.entmax_attention(q, K, V, alpha, scale)
    supp_pages = set((ref["support"] // P).tolist())
    for slack in (0.0, 1e-3, 0.1, 0.5):
        pages = orc.box_threshold_pages(box, alpha, ref["tau"] - slack)
        assert supp_pages <= set(pages.tolist())
    # a threshold ABOVE tau may lose support pages: the guarantee needs tau_lo <= tau
    z = (alpha - 1.0) * ref["s"]
    assert len(orc.box_threshold_pages(box, alpha, (alpha - 1.0) * box.max())) == 0 and z.max() > ref["tau"]


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("alpha", [1.5, 2.0])
def test_one_refinement_from_any_start_is_exact(seed, alpha):
    """Any starting selection: the sparse threshold is a lower bound of the full one; refining with it
    gives a set over which the sparse solve reproduces the full-cache result; nothing added <=> the
    start already held every page above the bound (and then the start was already exact)."""
    P, scale = 16, 0.6
    q, K, V, box = _unit(100 + seed, alpha=alpha)
    n = K.shape[0]
    rng = np.random.default_rng(seed)
    full = orc.entmax_attention(q, K, V, alpha, scale)
    start = np.sort(rng.choice(n // P, 1 + seed % 5, replace=False))
    sp = orc.entmax_attention(q, K, V, alpha, scale, orc.pages_to_tokens(start, P, n))
    assert sp["tau"] <= full["tau"] + 1e-12
    union, added = orc.refine_selection(box, alpha, sp["tau"], start)
    assert set(start.tolist()) <= set(union.tolist())
    assert set(added.tolist()) == set(union.tolist()) - set(start.tolist())
    again = orc.entmax_attention(q, K, V, alpha, scale, orc.pages_to_tokens(union, P, n))
    assert abs(again["tau"] - full["tau"]) <= 1e-12
    assert np.allclose(again["o"], full["o"], rtol=0, atol=1e-12)
    assert again["support"].tolist() == full["support"].tolist()
    if len(added) == 0:
        assert np.allclose(sp["o"], full["o"], rtol=0, atol=1e-12)
    # a start that holds the support and every page above its own threshold is certified at once
    good = orc.box_threshold_pages(box, alpha, full["tau"])
    spg = orc.entmax_attention(q, K, V, alpha, scale, orc.pages_to_tokens(good, P, n))
    _, added_g = orc.refine_selection(box, alpha, spg["tau"], good)
    assert len(added_g) == 0 and abs(spg["tau"] - full["tau"]) <= 1e-12


# ---------------------------------------------------------------------------- group-shared selection
def _group(seed, G=4, n=384, P=16, d=32, scale=0.6):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    Q = rng.standard_normal((G, d))
    for g in range(G):
        idx = rng.choice(n, 4, replace=False)
        K[idx] = 2.0 * Q[g] / np.linalg.norm(Q[g]) + 0.3 * rng.standard_normal((4, d))
    kmin, kmax, *_ = orc.page_stats(K, P)
    box = np.stack([orc.box_scores(Q[g], kmin, kmax, scale) for g in range(G)])
    return Q, K, V, box


def test_group_max_is_a_bound_for_every_head_and_reduces_for_one_head():
    Q, K, V, box = _group(1)
    gs = orc.group_max_scores(box)
    assert gs.shape == (box.shape[1],)
    for g in range(Q.shape[0]):
        s = orc.token_scores(Q[g], K, 0.6)
        page_max = s.reshape(-1, 16).max(axis=1)
        assert np.all(gs >= box[g]) and np.all(gs >= page_max - 1e-12)
    # every page's group score is attained by one of the heads
    assert np.all(np.isin(gs, box))
    assert np.array_equal(orc.group_max_scores(box[:1]), box[0])


@pytest.mark.parametrize("seed", range(4))
def test_group_threshold_selection_recovers_every_head_of_the_group(seed):
    """Thresholding the group score at the smallest full-cache tau of the group keeps every head's
    support pages, so each head's sparse result over the shared list equals its full-cache result."""
    alpha, scale, P = 1.5, 0.6, 16
    Q, K, V, box = _group(10 + seed)
    n = K.shape[0]
    full = [orc.entmax_attention(Q[g], K, V, alpha, scale) for g in range(Q.shape[0])]
    tau_min = min(f["tau"] for f in full)
    shared = orc.box_threshold_pages(orc.group_max_scores(box), alpha, tau_min)
    tok = orc.pages_to_tokens(shared, P, n)
    for g, f in enumerate(full):
        assert set((f["support"] // P).tolist()) <= set(shared.tolist())
        sp = orc.entmax_attention(Q[g], K, V, alpha, scale, tok)
        assert abs(sp["tau"] - f["tau"]) <= 1e-12 and np.allclose(sp["o"], f["o"], rtol=0, atol=1e-12)
