"""The decode step under HIP graph capture.

The library only launches kernels on the caller's stream (no allocation, no memset, no synchronisation), so
a whole step -- append inside the scoring launch, length update, selection (top-k, Gaussian-aware, or one
list per KV head on the 8-bit bounds), sparse or dense decode -- can be recorded once and replayed.  One
graph is replayed for consecutive decode steps (the new token is copied into a fixed staging buffer before
each replay, the sequence lengths live on the device and are bumped inside the graph); after EVERY replay
the results are compared, bit for bit, with an eager run of the same steps on a second copy of the cache,
with eager work and synchronisations between the replays.  The eager path itself is checked against the
oracle in tests/test_gpu_parity.py."""
import numpy as np
import pytest
import torch

from paper_2605_21649_amd import binding as ekv
from paper_2605_21649_amd import synth
from tests.helpers import DeviceState

pytestmark = pytest.mark.gpu


class LoopState:
    def __init__(self, w, inp, k, start, dev):
        self.st = st = DeviceState(w, {key: v.clone() for key, v in inp.items()}, cap=k, device=dev)
        self.k = k
        st.inp["seq_lens"].copy_(start)
        self.k_new = torch.zeros(w.batch, w.n_kv_heads, w.head_dim, dtype=st.inp["k_pool"].dtype, device=dev)
        self.v_new = torch.zeros_like(self.k_new)
        self.ws_t = st.workspace(ekv.EKV_OP_SELECT_TOPK)
        self.ws_d = st.workspace(ekv.EKV_OP_DECODE_SPARSE)
        ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())

    def step(self, variant="topk"):
        """Launches only; reads the token to append from the staging buffers."""
        st, w = self.st, self.st.w
        if variant == "topk":
            ekv.ekv_append_score_pages(st.cfg, st.cache(), st.stats(), self.k_new, self.v_new, st.inp["q"],
                                       ekv.EKV_SCORE_BOX, st.box, None, None)
            st.inp["seq_lens"] += 1
            ekv.ekv_select_topk(st.cfg, st.box, st.inp["seq_lens"], self.k, st.page_idx, st.n_sel, self.ws_t)
            ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau, st.supp,
                                  self.ws_d)
        elif variant == "gauss":
            ekv.ekv_append_score_pages(st.cfg, st.cache(), st.stats(), self.k_new, self.v_new, st.inp["q"],
                                       ekv.EKV_SCORE_GAUSS, None, st.mu, st.sigma)
            st.inp["seq_lens"] += 1
            ekv.ekv_select_gauss(st.cfg, st.mu, st.sigma, st.inp["seq_lens"], 0.9, 0.02, st.tau_hat, st.page_idx,
                                 st.n_sel, st.overflow, st.workspace(ekv.EKV_OP_SELECT_GAUSS))
            ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau, st.supp,
                                  self.ws_d)
        elif variant == "group":
            if not hasattr(self, "gcfg"):
                dev = st.box.device
                self.gcfg = ekv.make_config(w.batch, w.n_kv_heads, w.n_kv_heads, w.head_dim, w.page_size, w.kv_dtype,
                                            w.alpha, w.score_scale, st.Mmax, self.k)
                self.gbox = torch.zeros(w.batch, w.n_kv_heads, st.Mmax, device=dev)
                self.g_idx = torch.zeros(w.batch, w.n_kv_heads, self.k, device=dev, dtype=torch.int32)
                self.g_n = torch.zeros(w.batch, w.n_kv_heads, device=dev, dtype=torch.int32)
                self.ws_g = torch.empty(max(256, ekv.ekv_workspace_bytes(self.gcfg, ekv.EKV_OP_SELECT_TOPK)), device=dev,
                                        dtype=torch.uint8)
            ekv.ekv_append_score_pages(st.cfg, st.cache(), st.stats(), self.k_new, self.v_new, st.inp["q"],
                                       ekv.EKV_SCORE_BOX8 | ekv.EKV_SCORE_GROUP_MAX, self.gbox, None, None)
            st.inp["seq_lens"] += 1
            ekv.ekv_select_topk(self.gcfg, self.gbox, st.inp["seq_lens"], self.k, self.g_idx, self.g_n, self.ws_g)
            ekv.ekv_decode_sparse_group(st.cfg, st.inp["q"], st.cache(), self.g_idx, self.g_n, st.out, st.tau,
                                        st.supp, self.ws_d)
            st.page_idx[:, : w.n_kv_heads].copy_(self.g_idx)           # into the compared results
        else:                                                           # dense decode after a plain append
            ekv.ekv_stats_append(st.cfg, st.cache(), st.stats(), self.k_new, self.v_new)
            st.inp["seq_lens"] += 1
            ekv.ekv_decode_full(st.cfg, st.inp["q"], st.cache(), st.out, st.tau, st.supp,
                                st.workspace(ekv.EKV_OP_DECODE_FULL))

    def results(self):
        st = self.st
        return [t.clone() for t in (st.inp["seq_lens"], st.n_sel, st.page_idx, st.out, st.tau, st.supp, st.box,
                                    st.mu, st.sigma, st.tau_hat)]


@pytest.mark.parametrize("variant", ["topk", "gauss", "group", "dense"])
def test_graph_replay_of_the_decode_step_equals_eager(variant):
    w = synth.C2.scaled(name="C2-graph", batch=2, context=4096, n_q_heads=8, n_kv_heads=2)
    dev = torch.device("cuda")
    inp = synth.make_inputs(w, 2000 + 7, device="cpu")
    P, T, k = w.page_size, 20, 24
    start = torch.tensor([4096 - T - 5, 4096 - T - 14], dtype=torch.int32)     # both cross a page boundary
    B, Hkv = w.batch, w.n_kv_heads
    k_log = torch.stack([torch.stack([synth.logical_kv(inp, w, b, h)[0] for h in range(Hkv)]) for b in range(B)])
    v_log = torch.stack([torch.stack([synth.logical_kv(inp, w, b, h)[1] for h in range(Hkv)]) for b in range(B)])
    eager, graphed = LoopState(w, inp, k, start, dev), LoopState(w, inp, k, start, dev)
    for ls in (eager, graphed):
        ls.st.enable_box8()
        ekv.ekv_stats_build(ls.st.cfg, ls.st.cache(), ls.st.stats())
        ls.st.workspace(ekv.EKV_OP_SELECT_GAUSS); ls.st.workspace(ekv.EKV_OP_DECODE_FULL)   # allocated before capture

    def stage_token(ls, step):
        pos = (start + step).long()
        ls.k_new.copy_(torch.stack([k_log[b, :, pos[b]] for b in range(B)]))
        ls.v_new.copy_(torch.stack([v_log[b, :, pos[b]] for b in range(B)]))

    # step 0 runs eagerly on both copies (warm-up before the capture)
    for ls in (eager, graphed):
        stage_token(ls, 0)
        ls.step(variant)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=side):
        graphed.step(variant)
    torch.cuda.synchronize()
    # the capture itself executes nothing
    assert torch.equal(graphed.st.inp["seq_lens"], eager.st.inp["seq_lens"])
    for step in range(1, T):
        stage_token(graphed, step)
        g.replay()
        stage_token(eager, step)                    # eager launches and a synchronisation between replays
        eager.step(variant)
        torch.cuda.synchronize()
        for a, b_ in zip(graphed.results(), eager.results()):
            assert torch.equal(a.view(torch.uint8), b_.view(torch.uint8)), step
    assert int(eager.st.inp["seq_lens"][0]) == int(start[0]) + T
    # the caches the two loops filled are identical, statistics included
    for key in ("k_pool", "v_pool"):
        assert torch.equal(graphed.st.inp[key], eager.st.inp[key])
    assert torch.equal(graphed.st.box_stats.view(torch.uint8), eager.st.box_stats.view(torch.uint8))
    assert torch.equal(graphed.st.gauss_stats.view(torch.uint8), eager.st.gauss_stats.view(torch.uint8))
    if variant == "topk":
        assert np.all(graphed.st.n_sel.cpu().numpy() == k)
