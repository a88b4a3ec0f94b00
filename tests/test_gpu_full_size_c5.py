"""GPU parity at the full size of the alpha and baseline sweep workload (C5: 8 sequences of 262 144 tokens,
32 query / 8 KV heads, 8192 pages of 32 tokens, bf16): top-k at the matched budget of 4096 tokens per head
under alpha = 1.25, 1.5 and 2, the dense decode of the same alpha, and softmax over the same page lists with
its dropped mass (Sec. 3.3, Eq. 8).

The float64 oracle runs SAMPLED (sequence, query head) units, each over its whole KV head; its inputs are
copied from the generated cache before any library call.  Acceptance rules are those of
tests/test_gpu_parity.py; alpha = 2 is also checked against the sparsemax closed form (Sec. 2.2)."""
import math
import numpy as np
import pytest
import torch

from oracle import entmaxkv_oracle as orc
from paper_2605_21649_amd import binding as ekv
from paper_2605_21649_amd import synth
from tests.helpers import (DeviceState, sets_equal_up_to_cut, rel_err, to_f64, check_decode_unit,
                           check_decode_of_gpu_list)

pytestmark = pytest.mark.gpu

W = synth.C5
SEED = 5000
K_PAGES = 4096 // W.page_size
UNITS = [(0, 2), (3, 13), (7, 30)]


@pytest.fixture(scope="module")
def c5():
    dev = torch.device("cuda")
    inp = synth.make_inputs(W, SEED, device=dev)
    cpu = {}
    for (b, hq) in UNITS:
        k, v = synth.logical_kv(inp, W, b, hq // W.group)
        cpu[(b, hq)] = (to_f64(inp["q"][b, hq]), to_f64(k), to_f64(v))
    return dict(inp=inp, cpu=cpu)


def run_alpha(inp, alpha):
    """Statistics, box scores, top-k, sparse decode (with the kept mass under the dense threshold) and the dense
    decode (with its log-sum-exp) under one alpha."""
    st = DeviceState(W.scaled(alpha=alpha), inp, cap=K_PAGES, device=inp["q"].device)
    ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
    ekv.ekv_score_pages(st.cfg, inp["q"], st.stats(), inp["seq_lens"], ekv.EKV_SCORE_BOX, st.box)
    ekv.ekv_select_topk(st.cfg, st.box, inp["seq_lens"], K_PAGES, st.page_idx, st.n_sel,
                        st.workspace(ekv.EKV_OP_SELECT_TOPK))
    full = dict(out=torch.zeros_like(st.out), tau=torch.zeros_like(st.tau), supp=torch.zeros_like(st.supp),
                lse=torch.zeros_like(st.tau))
    ekv.ekv_decode_full(st.cfg, inp["q"], st.cache(), full["out"], full["tau"], full["supp"],
                        st.workspace(ekv.EKV_OP_DECODE_FULL), extras=ekv.decode_extras(lse=full["lse"]))
    kept, kept_n = torch.zeros_like(st.tau), torch.zeros_like(st.supp)
    ekv.ekv_decode_sparse(st.cfg, inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau, st.supp,
                          st.workspace(ekv.EKV_OP_DECODE_SPARSE),
                          extras=ekv.decode_extras(tau_ref=full["tau"], kept_mass_ref=kept, kept_supp_ref=kept_n))
    torch.cuda.synchronize()
    return st, full, kept, kept_n


def sparsemax_tau(z):
    """Threshold of sparsemax by its sort closed form (Sec. 2.2): k = max{k: 1 + k z_(k) > sum_{j<=k} z_(j)}."""
    zs = np.sort(z)[::-1]
    cs = np.cumsum(zs)
    ks = np.arange(1, len(zs) + 1)
    kk = ks[1.0 + ks * zs > cs].max()
    return (cs[kk - 1] - 1.0) / kk


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0])
def test_full_size_topk_and_dense_under_each_alpha(c5, alpha):
    inp = c5["inp"]
    st, full, kept, kept_n = run_alpha(inp, alpha)
    a, P, n = alpha - 1.0, W.page_size, W.context
    idx, ns = st.page_idx.cpu().numpy(), st.n_sel.cpu().numpy()
    assert np.all(ns == K_PAGES)
    for (b, hq) in UNITS:
        q, K, V = c5["cpu"][(b, hq)]
        ref = orc.decode_step_unit(q, K, V, P, alpha, W.score_scale, "topk", W.kv_dtype, k_pages=K_PAGES)
        got_box = st.box[b, hq].cpu().numpy()
        assert np.max(np.abs(got_box - ref["box"]) / np.maximum(1.0, np.abs(ref["box"]))) <= 1e-5
        band = 1e-5 * max(1.0, abs(ref["cut_in"]))
        ok, bad = sets_equal_up_to_cut(idx[b, hq], ref["pages"], ref["box"], [ref["cut_in"], ref["cut_out"]], band)
        assert ok, (hq, bad)
        wa = W.scaled(alpha=alpha)
        dense = orc.entmax_attention(q, K, V, alpha, W.score_scale)
        # tau, output, and the support count exact up to tokens whose z lies within float32 resolution of tau
        check_decode_unit(wa, full["out"][b, hq].cpu().numpy(), float(full["tau"][b, hq]), int(full["supp"][b, hq]),
                          None, dense)
        lse_ref = float(np.log(np.sum(np.exp(dense["s"] - dense["s"].max()))) + dense["s"].max())
        assert abs(float(full["lse"][b, hq]) - lse_ref) <= 1e-4 * max(1.0, abs(lse_ref))
        if alpha == 2.0:
            assert abs(float(full["tau"][b, hq]) - sparsemax_tau(a * dense["s"])) <= 4e-6
        # the sparse decode of the list the GPU chose (equal to the oracle's or not: pages inside the tie band)
        own = check_decode_of_gpu_list(wa, q, K, V, idx[b, hq], st.out[b, hq].cpu().numpy(), st.tau[b, hq],
                                       st.supp[b, hq])
        # dropped mass and support recall of that selection under the dense threshold (Eq. 4, Eq. 7); a dense
        # support token on the float32 boundary of tau may or may not be counted
        delta = orc.dropped_mass(dense["p"], own["tokens"])
        assert abs((1.0 - float(kept[b, hq])) - delta) <= 1e-4
        rho = orc.support_retention(dense["support"], own["tokens"])
        zb = a * dense["s"]
        n_bound = int(np.sum(np.abs(zb - dense["tau"]) <= 2e-6 * max(1.0, abs(dense["tau"]))))
        assert abs(int(kept_n[b, hq]) - rho * len(dense["support"])) <= n_bound + 0.5
        assert float(st.tau[b, hq]) <= float(full["tau"][b, hq]) + 1e-6    # a sparse solve never overshoots


def test_full_size_softmax_over_the_topk_lists(c5):
    """Softmax restricted to the lists the top-k selector returns, and its dropped mass against entmax's on
    the same lists (Eq. 8's two sides)."""
    inp = c5["inp"]
    st, full, kept, _ = run_alpha(inp, 1.5)
    lse = torch.zeros_like(st.tau)
    out = torch.zeros_like(st.out)
    ekv.ekv_decode_sparse_softmax(st.cfg, inp["q"], st.cache(), st.page_idx, st.n_sel, out, lse,
                                  st.workspace(ekv.EKV_OP_DECODE_SPARSE_SOFTMAX))
    torch.cuda.synchronize()
    idx = st.page_idx.cpu().numpy()
    for (b, hq) in UNITS:
        q, K, V = c5["cpu"][(b, hq)]
        tok = orc.pages_to_tokens(idx[b, hq], W.page_size, K.shape[0])         # the list the GPU decoded
        ref = orc.softmax_attention(q, K, V, W.score_scale, tok)
        assert rel_err(out[b, hq].cpu().numpy(), ref["o"]) <= 2e-3
        assert abs(float(lse[b, hq]) - ref["lse"]) <= 2e-5 * max(1.0, abs(ref["lse"]))
        soft = orc.softmax_attention(q, K, V, W.score_scale)
        d_sm = orc.dropped_mass(soft["p"], tok)
        got_sm = 1.0 - math.exp(float(lse[b, hq]) - float(full["lse"][b, hq]))
        assert abs(got_sm - d_sm) <= 1e-4
        dense = orc.entmax_attention(q, K, V, 1.5, W.score_scale)
        d_ent = orc.dropped_mass(dense["p"], tok)
        assert abs((1.0 - float(kept[b, hq])) - d_ent) <= 1e-4
