"""Pins of the oracle's 8-bit page bounds (OCP E4M3, rounded outward) -- CPU only.

The value table is checked against a library decoder (torch's float8_e4m3fn), the directed rounding by
brute force over that table and against the library's round-to-nearest conversion, the score against a
hand-worked example and against the inequalities that make it usable: 8-bit score >= cache-dtype score
>= largest token score of the page."""
import os
import numpy as np
import pytest
import torch

from oracle import entmaxkv_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "box8_example.txt")


def library_table():
    """All 256 codes decoded by torch (an implementation independent of the oracle's formula)."""
    codes = torch.arange(256, dtype=torch.uint8)
    return codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)


def test_grid_is_the_e4m3_value_set():
    grid = orc.e4m3_grid()
    tab = library_table()
    assert np.isnan(tab[0x7F]) and np.isnan(tab[0xFF]) and np.isnan(tab).sum() == 2
    finite = np.unique(tab[~np.isnan(tab)])                  # +0 and -0 collapse
    np.testing.assert_array_equal(grid, finite)
    assert len(grid) == 253 and grid[-1] == 448.0 and grid[0] == -448.0
    pos = grid[grid > 0]
    assert pos[0] == 2.0 ** -9 and 1.0 in pos
    np.testing.assert_array_equal(np.diff(pos[(pos >= 1) & (pos <= 2)]), 0.125)
    np.testing.assert_array_equal(np.diff(pos[pos >= 256]), 32.0)
    np.testing.assert_array_equal(grid, -grid[::-1])


def test_directed_rounding_by_brute_force():
    tab = library_table()
    finite = tab[~np.isnan(tab)]
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4000) * 3, rng.normal(size=2000) * 1e-2, rng.uniform(-460, 460, 2000),
                        finite, finite + 1e-9, finite - 1e-9, [0.0, -0.0, 1e-12, -1e-12, 448.0, -448.0]])
    lo, hi = orc.round_e4m3(x, "down"), orc.round_e4m3(x, "up")
    for xi, l, h in zip(x, lo, hi):
        below, above = finite[finite <= xi], finite[finite >= xi]
        if len(below): assert l == below.max(), (xi, l)
        else: assert np.isnan(l) and xi < -448
        if len(above): assert h == above.min(), (xi, h)
        else: assert np.isnan(h) and xi > 448
    on = np.isin(x, finite)
    np.testing.assert_array_equal(lo[on], hi[on])
    np.testing.assert_array_equal(lo[on], x[on])


def test_nearest_conversion_of_the_library_is_one_of_the_two_neighbours():
    rng = np.random.default_rng(1)
    x = (rng.normal(size=5000) * 5).astype(np.float32)
    near = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    lo, hi = orc.round_e4m3(x.astype(np.float64), "down"), orc.round_e4m3(x.astype(np.float64), "up")
    assert np.all((near == lo) | (near == hi))
    # and it is the closer one
    assert np.all(np.abs(near - x) <= np.minimum(np.abs(lo - x), np.abs(hi - x)) + 1e-12)


def test_examples_and_range_ends():
    r = orc.round_e4m3
    assert r(0.3, "down") == 0.28125 and r(0.3, "up") == 0.3125
    assert r(-0.3, "down") == -0.3125 and r(-0.3, "up") == -0.28125
    assert r(17.0, "down") == 16.0 and r(17.0, "up") == 18.0
    assert r(1e-4, "down") == 0.0 and r(1e-4, "up") == 2.0 ** -9
    assert r(-1e-4, "down") == -(2.0 ** -9) and r(-1e-4, "up") == 0.0
    assert r(449.0, "down") == 448.0 and np.isnan(r(449.0, "up"))
    assert np.isnan(r(-449.0, "down")) and r(-449.0, "up") == -448.0
    assert np.isnan(r(np.nan, "down")) and np.isnan(r(np.nan, "up"))
    assert r(np.inf, "down") == 448.0 and r(-np.inf, "up") == -448.0


def test_worked_example():
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip(): continue
        key, *vals = line.split()
        rows[key] = np.array([float(v) for v in vals])
    lo8, hi8 = orc.box8_stats(rows["kmin"], rows["kmax"])
    np.testing.assert_array_equal(lo8, rows["lo8"])
    np.testing.assert_array_equal(hi8, rows["hi8"])
    assert orc.box8_scores(rows["q"], lo8[None], hi8[None], 1.0)[0] == rows["score8"][0]
    assert abs(orc.box_scores(rows["q"], rows["kmin"][None], rows["kmax"][None], 1.0)[0] - rows["score"][0]) < 1e-12


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_eight_bit_score_bounds_the_cache_dtype_score_and_every_token(seed):
    rng = np.random.default_rng(seed)
    n, d, P = 512, 128, 16
    K = rng.normal(size=(n, d)) + (rng.random(d) < 0.05) * 5.0
    K = orc.round_to_bf16(K)
    q = orc.round_to_bf16(rng.normal(size=d))
    kmin, kmax, *_ = orc.page_stats(K, P)
    lo8, hi8 = orc.box8_stats(kmin, kmax)
    assert np.all(lo8 <= kmin) and np.all(hi8 >= kmax)
    s8 = orc.box8_scores(q, lo8, hi8, 0.1)
    s16 = orc.box_scores(q, kmin, kmax, 0.1)
    tok = orc.token_scores(q, K, 0.1).reshape(-1, P).max(axis=1)
    assert np.all(s8 >= s16 - 1e-12) and np.all(s16 >= tok - 1e-12)
    assert np.any(s8 > s16)                                   # the rounding does cost something
    # format values in, same score out
    grid = orc.e4m3_grid()
    Kg = grid[rng.integers(60, len(grid) - 60, size=(n, d))]
    kmin, kmax, *_ = orc.page_stats(Kg, P)
    lo8, hi8 = orc.box8_stats(kmin, kmax)
    np.testing.assert_array_equal(orc.box8_scores(q, lo8, hi8, 0.1), orc.box_scores(q, kmin, kmax, 0.1))


def test_unrepresentable_bound_selects_the_page():
    rng = np.random.default_rng(3)
    K = rng.normal(size=(64, 8)); K[20, 3] = 500.0; K[40, 1] = -1000.0
    kmin, kmax, *_ = orc.page_stats(K, 16)
    lo8, hi8 = orc.box8_stats(kmin, kmax)
    s8 = orc.box8_scores(rng.normal(size=8), lo8, hi8, 1.0)
    assert np.isposinf(s8[1]) and np.isposinf(s8[2]) and np.all(np.isfinite(s8[[0, 3]]))
