"""ekv_decode_sparse_static -- the entry point that allocates nothing (scratch in a static device array of the
library) -- against ekv_decode_sparse with a caller workspace: same kernels, so every output must be identical bit
for bit.  Two calls in a row on one GPU, the second on a smaller problem, each checked; the array keeps whatever
the previous call left, and the results must not depend on it."""
import pytest
import torch

from paper_2605_21649_amd import binding as ekv
from paper_2605_21649_amd import synth
from tests.helpers import DeviceState

pytestmark = pytest.mark.gpu


def run_both(w, seed, k):
    dev = torch.device("cuda")
    inp = synth.make_inputs(w, seed, device="cpu")
    st = DeviceState(w, inp, cap=k + 5, device=dev)
    q, seq = st.inp["q"], st.inp["seq_lens"]
    ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
    ekv.ekv_score_pages(st.cfg, q, st.stats(), seq, ekv.EKV_SCORE_BOX, st.box)
    ekv.ekv_select_topk(st.cfg, st.box, seq, k, st.page_idx, st.n_sel, st.workspace(ekv.EKV_OP_SELECT_TOPK))
    B, Hq = w.batch, w.n_q_heads
    res = []
    for static in (False, True):
        out = torch.full((B, Hq, w.head_dim), float("nan"), device=dev)
        tau = torch.full((B, Hq), float("nan"), device=dev)
        supp = torch.full((B, Hq), -1, device=dev, dtype=torch.int32)
        toks = torch.full((B, Hq, 256), -1, device=dev, dtype=torch.int32)
        evals = torch.full((B, Hq), -1, device=dev, dtype=torch.int32)
        ex = ekv.decode_extras(support_tokens=toks, solve_evals=evals)
        if static:
            assert ekv.ekv_workspace_bytes(st.cfg, ekv.EKV_OP_DECODE_SPARSE) <= ekv.EKV_STATIC_SCRATCH_BYTES
            ekv.ekv_decode_sparse_static(st.cfg, q, st.cache(), st.page_idx, st.n_sel, out, tau, supp, extras=ex)
        else:
            ekv.ekv_decode_sparse(st.cfg, q, st.cache(), st.page_idx, st.n_sel, out, tau, supp,
                                  st.workspace(ekv.EKV_OP_DECODE_SPARSE), extras=ex)
        torch.cuda.synchronize()
        res.append((out, tau, supp, toks, evals))
    for a, b in zip(*res):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    out, tau, supp = res[1][:3]
    assert torch.isfinite(out).all() and torch.isfinite(tau).all() and (supp > 0).all()


def test_static_scratch_decode_equals_workspace_decode_twice():
    # first a batch of two ragged 16K-token sequences (32 query heads, 40 pages each), then a smaller problem
    run_both(synth.C2.scaled(name="C2-b2-16k", batch=2, context=16384 + 16, ragged=5), 3101, 40)
    run_both(synth.C1.scaled(name="C1-2k", context=2048, ragged=3), 3102, 12)
    # and the larger one again, after the small one has overwritten the start of the array
    run_both(synth.C5.scaled(name="C5-p32-b1", batch=1, context=8192, ragged=9), 3103, 24)
