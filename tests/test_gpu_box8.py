"""GPU parity of the 8-bit page bounds (k_min rounded down, k_max rounded up to OCP E4M3) against the
oracle: the stored codes (decoded with torch's float8_e4m3fn, a library decoder), the box score computed
from them, and the whole top-k step that selects on that score.

Acceptance: stored bounds equal the oracle's value for value (NaN where the oracle has NaN); scores within
1e-5 * max(1, |score|) and +inf exactly where the oracle has +inf; page sets identical except pages within
1e-5 * max(1, |cut|) of the cut; tau, supports and outputs as in tests/test_gpu_parity.py."""
import math
import numpy as np
import pytest
import torch

from oracle import entmaxkv_oracle as orc
from paper_2605_21649_amd import binding as ekv
from paper_2605_21649_amd import synth
from tests.helpers import (DeviceState, unit_kv, oracle_stats, sets_equal_up_to_cut, rel_err, to_f64,
                           check_decode_of_gpu_list)

pytestmark = pytest.mark.gpu

W2 = synth.C2.scaled(name="C2-8k", context=8192 + 16, ragged=3)
W3 = synth.C3.scaled(name="C3-small", batch=2, context=4096)
W5 = synth.C5.scaled(name="C5-small", batch=2, context=8192, alpha=1.25)
WP8 = synth.C2.scaled(name="C2-p8-g2", context=2048 + 8, ragged=3, page_size=8, n_q_heads=4, n_kv_heads=2)
WP64 = synth.C2.scaled(name="C2-p64-g8", context=4096 + 64, ragged=21, page_size=64, n_q_heads=16, n_kv_heads=2)
ALL = [W2, W3, W5, WP8, WP64]
IDS = [w.name for w in ALL]
_cache = {}


def get_inputs(w, extreme=False):
    key = (w.name, extreme)
    if key not in _cache:
        cfg_id = ["C1", "C2", "C3", "C4", "C5"].index(w.name[:2]) + 1
        inp = synth.make_inputs(w, 1000 * cfg_id + 50, device="cpu")
        if extreme:
            # values the 8-bit format cannot bound, values below its subnormal step, exact format values
            kp = inp["k_pool"]
            rng = np.random.default_rng(8)
            flat = kp.view(-1)
            pos = torch.from_numpy(rng.choice(flat.numel(), 400, replace=False))
            vals = torch.tensor([500.0, -500.0, 3.0e4, -3.0e4, 448.0, -448.0, 1e-4, -1e-4, 0.0, 2.0 ** -9, 0.28125,
                                 -0.3125, 1e-30, -1e-30, 464.0, -464.0], dtype=torch.float32)
            flat[pos] = vals[torch.from_numpy(rng.integers(0, len(vals), size=400))].to(kp.dtype)
        _cache[key] = inp
    return _cache[key]


def decode_box8(t):
    """uint8 [..., 16, 2, 8] codes -> (lo8, hi8) float64 [..., 128]."""
    v = t.cpu().view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    lo, hi = v[..., 0, :], v[..., 1, :]
    return lo.reshape(*lo.shape[:-2], 128), hi.reshape(*hi.shape[:-2], 128)


def encode_box8(lo8, hi8):
    """Oracle bounds (already format values or NaN) -> uint8 [M, 16, 2, 8]; the conversion is exact."""
    M = lo8.shape[0]
    both = np.stack([lo8.reshape(M, 16, 8), hi8.reshape(M, 16, 8)], axis=2).astype(np.float32)
    t = torch.from_numpy(both).to(torch.float8_e4m3fn)
    back = t.to(torch.float32).numpy()
    assert np.array_equal(back, both, equal_nan=True)
    return t.view(torch.uint8)


@pytest.mark.parametrize("extreme", [False, True], ids=["plain", "extreme-values"])
@pytest.mark.parametrize("w", ALL, ids=IDS)
def test_box8_statistics_build_and_append(w, extreme):
    inp = get_inputs(w, extreme)
    st = DeviceState(w, inp)
    st.enable_box8()
    ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
    torch.cuda.synchronize()
    lo_g, hi_g = decode_box8(st.box8_stats)
    n_nan = 0
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            kmin, kmax, _, _, cnt = oracle_stats(inp, w, b, h)
            lo8, hi8 = orc.box8_stats(kmin, kmax)
            M = len(cnt)
            assert np.array_equal(lo_g[b, h, :M], lo8, equal_nan=True)
            assert np.array_equal(hi_g[b, h, :M], hi8, equal_nan=True)
            n_nan += int(np.isnan(lo8).sum() + np.isnan(hi8).sum())
    assert (n_nan > 0) == extreme
    # append: the last token of every sequence removed and appended again gives the same bytes
    ref8, ref_box = st.box8_stats.clone(), st.box_stats.clone()
    n = st.inp["seq_lens"].clone()
    P = w.page_size
    rows = torch.stack([st.inp["block_table"][b, (int(n[b]) - 1) // P] for b in range(w.batch)]).long()
    slot = [(int(n[b]) - 1) % P for b in range(w.batch)]
    k_new = torch.stack([st.inp["k_pool"][rows[b], :, slot[b]] for b in range(w.batch)]).contiguous()
    v_new = torch.stack([st.inp["v_pool"][rows[b], :, slot[b]] for b in range(w.batch)]).contiguous()
    st.inp["seq_lens"] -= 1
    ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
    ekv.ekv_stats_append(st.cfg, st.cache(), st.stats(), k_new, v_new)
    st.inp["seq_lens"] += 1
    torch.cuda.synchronize()
    M = -(-int(n.max()) // P)
    for b in range(w.batch):
        Mb = -(-int(n[b]) // P)
        assert torch.equal(st.box8_stats[b, :, :Mb], ref8[b, :, :Mb])
        assert torch.equal(st.box_stats[b, :, :Mb].view(torch.uint8), ref_box[b, :, :Mb].view(torch.uint8))


@pytest.mark.parametrize("extreme", [False, True], ids=["plain", "extreme-values"])
@pytest.mark.parametrize("w", ALL, ids=IDS)
def test_box8_scores_on_shared_bounds(w, extreme):
    """Scores from the oracle's 8-bit bounds uploaded to the device: per head, and the group maximum."""
    inp = get_inputs(w, extreme)
    st = DeviceState(w, inp)
    st.enable_box8()
    dev = st.box.device
    bounds = {}
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            kmin, kmax, _, _, cnt = oracle_stats(inp, w, b, h)
            lo8, hi8 = orc.box8_stats(kmin, kmax)
            st.box8_stats[b, h, : len(cnt)] = encode_box8(lo8, hi8).to(dev)
            bounds[(b, h)] = (lo8, hi8, kmin, kmax)
    ekv.ekv_score_pages(st.cfg, st.inp["q"], st.stats(), st.inp["seq_lens"], ekv.EKV_SCORE_BOX8, st.box)
    gbox = torch.zeros(w.batch, w.n_kv_heads, st.Mmax, device=dev)
    ekv.ekv_score_pages(st.cfg, st.inp["q"], st.stats(), st.inp["seq_lens"],
                        ekv.EKV_SCORE_BOX8 | ekv.EKV_SCORE_GROUP_MAX, gbox)
    torch.cuda.synchronize()
    box, gb = st.box.cpu().numpy(), gbox.cpu().numpy()
    G = w.group
    n_inf = 0
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            lo8, hi8, kmin, kmax = bounds[(b, h)]
            M = lo8.shape[0]
            heads = []
            for g in range(G):
                hq = h * G + g
                q = to_f64(inp["q"][b, hq])
                ref = orc.box8_scores(q, lo8, hi8, w.score_scale)
                inf = np.isposinf(ref)
                assert np.array_equal(np.isposinf(box[b, hq, :M]), inf)
                err = np.abs(box[b, hq, :M][~inf] - ref[~inf]) / np.maximum(1.0, np.abs(ref[~inf]))
                assert np.all(err <= 1e-5), err.max()
                assert np.all(np.isneginf(box[b, hq, M:]))
                # still an upper bound of the cache-dtype score where the cache-dtype bounds are finite
                s16 = orc.box_scores(q, kmin, kmax, w.score_scale)
                assert np.all(ref >= s16 - 1e-9)
                heads.append(ref)
                n_inf += int(inf.sum())
            ref_g = orc.group_max_scores(np.stack(heads))
            inf = np.isposinf(ref_g)
            assert np.array_equal(np.isposinf(gb[b, h, :M]), inf)
            assert np.all(np.abs(gb[b, h, :M][~inf] - ref_g[~inf]) / np.maximum(1.0, np.abs(ref_g[~inf])) <= 1e-5)
    assert (n_inf > 0) == extreme


@pytest.mark.parametrize("w", [W2, W3, W5, WP64], ids=["C2-8k", "C3-small", "C5-small", "C2-p64-g8"])
def test_box8_topk_step(w):
    """append + 8-bit scoring in one launch (equal to the two calls bit for bit), top-k, sparse decode,
    against the oracle's step that selects on the 8-bit score."""
    inp = get_inputs(w)
    k = max(2, min(w.pages_per_seq // 4, 2048 // w.page_size))
    st = DeviceState(w, inp, cap=k)
    st.enable_box8()
    P = w.page_size
    n = st.inp["seq_lens"].clone()
    rows = torch.stack([st.inp["block_table"][b, (int(n[b]) - 1) // P] for b in range(w.batch)]).long()
    k_new = torch.stack([st.inp["k_pool"][rows[b], :, (int(n[b]) - 1) % P] for b in range(w.batch)]).contiguous()
    v_new = torch.stack([st.inp["v_pool"][rows[b], :, (int(n[b]) - 1) % P] for b in range(w.batch)]).contiguous()
    st.inp["seq_lens"] -= 1
    ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
    # two calls ...
    ekv.ekv_stats_append(st.cfg, st.cache(), st.stats(), k_new, v_new)
    st.inp["seq_lens"] += 1
    ekv.ekv_score_pages(st.cfg, st.inp["q"], st.stats(), st.inp["seq_lens"], ekv.EKV_SCORE_BOX8, st.box)
    torch.cuda.synchronize()
    box_two, stats_two = st.box.clone(), st.box8_stats.clone()
    # ... and the fused one, from the same starting state
    st.inp["seq_lens"] -= 1
    ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
    st.box.zero_()
    ekv.ekv_append_score_pages(st.cfg, st.cache(), st.stats(), k_new, v_new, st.inp["q"], ekv.EKV_SCORE_BOX8, st.box,
                               None, None)
    st.inp["seq_lens"] += 1
    torch.cuda.synchronize()
    assert torch.equal(st.box.view(torch.int32), box_two.view(torch.int32))
    assert torch.equal(st.box8_stats, stats_two)
    ekv.ekv_select_topk(st.cfg, st.box, st.inp["seq_lens"], k, st.page_idx, st.n_sel, st.workspace(ekv.EKV_OP_SELECT_TOPK))
    ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau, st.supp,
                          st.workspace(ekv.EKV_OP_DECODE_SPARSE))
    torch.cuda.synchronize()
    idx, ns = st.page_idx.cpu().numpy(), st.n_sel.cpu().numpy()
    units = [(b, h) for b in range(w.batch) for h in range(w.n_q_heads)]
    rng = np.random.default_rng(5)
    for i in sorted(rng.choice(len(units), min(6, len(units)), replace=False)):
        b, hq = units[i]
        q, K, V = unit_kv(inp, w, b, hq)
        kmin, kmax, *_ = orc.page_stats(K, P)
        lo8, hi8 = orc.box8_stats(kmin, kmax)
        s8 = orc.box8_scores(q, lo8, hi8, w.score_scale)
        pages, cut_in, cut_out = orc.topk_pages(s8, k)
        ok, bad = sets_equal_up_to_cut(idx[b, hq, : ns[b, hq]], pages, s8, [cut_in, cut_out], 1e-5 * max(1.0, abs(cut_in)))
        assert ok, (b, hq, bad)
        check_decode_of_gpu_list(w, q, K, V, idx[b, hq, : ns[b, hq]], st.out[b, hq].cpu().numpy(), st.tau[b, hq],
                                 st.supp[b, hq])
