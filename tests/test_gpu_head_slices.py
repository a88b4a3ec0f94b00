"""A config may address a subset of the KV heads of a cache (pool_kv_heads = the cache's head count, pool
pointers advanced to the first head).  Two halves of the heads run as independent problems on two streams
must give, bit for bit, what one call over all heads gives -- statistics, scores, selections, sparse,
grouped, dense and softmax decode -- and, being the same kernels, stand on the oracle parity of the whole."""
import numpy as np
import pytest
import torch

from paper_2605_21649_amd import binding as ekv
from paper_2605_21649_amd import synth
from tests.device_state import DeviceState, HeadSlice

pytestmark = pytest.mark.gpu


def run_all(p, cache_prev, cache_now, k_new, v_new, k, gcfg, gbufs):
    """Every entry point once on problem `p` (a DeviceState or a HeadSlice); returns nothing, fills p's arrays."""
    q, seq = (p.inp["q"], p.inp["seq_lens"]) if isinstance(p, DeviceState) else (p.q, p.seq_lens)
    ekv.ekv_stats_build(p.cfg, cache_now, p.stats())
    ekv.ekv_append_score_pages(p.cfg, cache_prev, p.stats(), k_new, v_new, q, ekv.EKV_SCORE_BOX, p.box, None, None)
    ekv.ekv_score_pages(p.cfg, q, p.stats(), seq, ekv.EKV_SCORE_GAUSS, None, p.mu, p.sigma)
    ekv.ekv_select_topk(p.cfg, p.box, seq, k, p.page_idx, p.n_sel, p.workspace(ekv.EKV_OP_SELECT_TOPK))
    ekv.ekv_decode_sparse(p.cfg, q, cache_now, p.page_idx, p.n_sel, p.out, p.tau, p.supp,
                          p.workspace(ekv.EKV_OP_DECODE_SPARSE))
    res = [p.out.clone(), p.tau.clone(), p.supp.clone(), p.page_idx.clone()]
    lse = torch.zeros_like(p.tau)
    ekv.ekv_decode_sparse_softmax(p.cfg, q, cache_now, p.page_idx, p.n_sel, p.out, lse,
                                  p.workspace(ekv.EKV_OP_DECODE_SPARSE_SOFTMAX))
    res += [p.out.clone(), lse]
    ekv.ekv_select_gauss(p.cfg, p.mu, p.sigma, seq, 0.9, 0.02, p.tau_hat, p.page_idx, p.n_sel, p.overflow,
                         p.workspace(ekv.EKV_OP_SELECT_GAUSS))
    ekv.ekv_decode_sparse(p.cfg, q, cache_now, p.page_idx, p.n_sel, p.out, p.tau, p.supp,
                          p.workspace(ekv.EKV_OP_DECODE_SPARSE))
    res += [p.out.clone(), p.tau.clone(), p.n_sel.clone(), p.tau_hat.clone()]
    ekv.ekv_decode_full(p.cfg, q, cache_now, p.out, p.tau, p.supp, p.workspace(ekv.EKV_OP_DECODE_FULL))
    res += [p.out.clone(), p.tau.clone(), p.supp.clone()]
    # one list per KV head
    gbox, g_idx, g_n, ws_sel = gbufs
    ekv.ekv_score_pages(p.cfg, q, p.stats(), seq, ekv.EKV_SCORE_BOX8 | ekv.EKV_SCORE_GROUP_MAX, gbox)
    ekv.ekv_select_topk(gcfg, gbox, seq, k, g_idx, g_n, ws_sel)
    ekv.ekv_decode_sparse_group(p.cfg, q, cache_now, g_idx, g_n, p.out, p.tau, p.supp,
                                p.workspace(ekv.EKV_OP_DECODE_SPARSE))
    res += [p.out.clone(), p.tau.clone(), g_idx.clone()]
    return res


@pytest.mark.parametrize("w", [synth.C2.scaled(name="C2-8k-b1", context=8192 + 16, ragged=3),
                               synth.C5.scaled(name="C5-p32-b1", batch=1, context=4096, ragged=9)],
                         ids=["C2-8k", "C5-p32"])
def test_two_head_halves_on_two_streams_equal_one_call(w):
    dev = torch.device("cuda")
    inp = synth.make_inputs(w, 2000 + 11, device="cpu")
    k = 24
    Hkv, G = w.n_kv_heads, w.group
    g = torch.Generator().manual_seed(5)
    k_new = torch.randn(1, Hkv, w.head_dim, generator=g).to(synth.torch_dtype(w.kv_dtype)).to(dev)
    v_new = torch.randn(1, Hkv, w.head_dim, generator=g).to(synth.torch_dtype(w.kv_dtype)).to(dev)

    def group_bufs(n_heads, st):
        gcfg = ekv.make_config(1, n_heads, n_heads, w.head_dim, w.page_size, w.kv_dtype, w.alpha, w.score_scale,
                               st.Mmax, k)
        bufs = (torch.zeros(1, n_heads, st.Mmax, device=dev), torch.zeros(1, n_heads, k, device=dev, dtype=torch.int32),
                torch.zeros(1, n_heads, device=dev, dtype=torch.int32),
                torch.empty(max(256, ekv.ekv_workspace_bytes(gcfg, ekv.EKV_OP_SELECT_TOPK)), device=dev, dtype=torch.uint8))
        return gcfg, bufs

    results = {}
    for mode in ("whole", "halves"):
        st = DeviceState(w, inp, cap=k, device=dev)
        st.enable_box8()
        seq_prev = (st.inp["seq_lens"] - 1).contiguous()
        if mode == "whole":
            cache_prev = ekv.cache_view(st.inp["k_pool"], st.inp["v_pool"], st.inp["block_table"], seq_prev)
            gcfg, bufs = group_bufs(Hkv, st)
            res = run_all(st, cache_prev, st.cache(), k_new, v_new, k, gcfg, bufs)
            torch.cuda.synchronize()
            results[mode] = (res, st)
        else:
            halves = [HeadSlice(st, 0, Hkv // 2), HeadSlice(st, Hkv // 2, Hkv)]
            streams = [torch.cuda.Stream(), torch.cuda.Stream()]
            parts = []
            torch.cuda.synchronize()
            for hs, s in zip(halves, streams):
                with torch.cuda.stream(s):
                    kn, vn = hs.new_token(k_new, v_new)
                    gcfg, bufs = group_bufs(hs.h1 - hs.h0, st)
                    parts.append(run_all(hs, hs.cache(seq_prev), hs.cache(), kn.contiguous(), vn.contiguous(), k,
                                         gcfg, bufs))
            torch.cuda.synchronize()
            results[mode] = ([torch.cat([a, b], dim=1) for a, b in zip(*parts)], st)
    whole, st_w = results["whole"]
    halves, st_h = results["halves"]
    for i, (a, b) in enumerate(zip(whole, halves)):
        assert a.shape == b.shape and torch.equal(a.view(torch.uint8), b.view(torch.uint8)), i
    for name in ("box_stats", "gauss_stats", "box8_stats", "box", "mu", "sigma"):
        assert torch.equal(getattr(st_w, name).view(torch.uint8), getattr(st_h, name).view(torch.uint8)), name
    assert torch.equal(st_w.inp["k_pool"], st_h.inp["k_pool"]) and torch.equal(st_w.inp["v_pool"], st_h.inp["v_pool"])
