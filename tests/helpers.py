"""Shared test plumbing: device buffers for a workload, and the oracle run per (b, h) unit.

The oracle never sees anything produced by the HIP path; where a stage test needs "the same stored
statistics / scores on both sides", the oracle's values are uploaded to the GPU, never the reverse."""
import math
import numpy as np
import torch

from oracle import entmaxkv_oracle as orc
from paper_2605_21649_amd import binding as ekv
from paper_2605_21649_amd import synth
from tests.device_state import DeviceState  # noqa: F401  (re-exported for the tests)


def to_f64(t):
    """Exact widening of a cache-dtype torch tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float32).numpy().astype(np.float64)


def unit_kv(inp_cpu, w, b, hq):
    """float64 q [d], K, V [n_b, d] of unit (b, hq) in logical token order."""
    hkv = hq // w.group
    k, v = synth.logical_kv(inp_cpu, w, b, hkv)
    return to_f64(inp_cpu["q"][b, hq]), to_f64(k), to_f64(v)


def oracle_stats(inp_cpu, w, b, hkv):
    k, _ = synth.logical_kv(inp_cpu, w, b, hkv)
    return orc.page_stats(to_f64(k), w.page_size)


def storage_ulp(x, kv_dtype):
    """Spacing of the storage dtype at |x| (float64 array)."""
    bits = 8 if kv_dtype == "bf16" else 24
    _, e = np.frexp(np.maximum(np.abs(x), 1e-30))
    return np.ldexp(1.0, e - bits)


def sets_equal_up_to_cut(got, ref, scores, cuts, band):
    """Page sets identical except pages whose score lies within `band` of a cut value
    (`cuts`: one value, or the scores of the last page taken and of the best page left out)."""
    cuts = [c for c in np.atleast_1d(cuts) if np.isfinite(c)]
    got, ref = set(int(x) for x in got), set(int(x) for x in ref)
    diff = got.symmetric_difference(ref)
    bad = [p for p in diff if all(abs(scores[p] - c) > band for c in cuts)]
    return len(bad) == 0, bad


def rel_err(a, b):
    return float(np.linalg.norm(np.asarray(a, dtype=np.float64) - b) / max(np.linalg.norm(b), 1e-300))


# Output tolerance by cache dtype (relative L2): float32 accumulation of exact products on float32 caches; a bf16
# cache rounds q, K and V before either side sees them, the bound covers what float32 accumulation adds on top.
OUT_TOL = {"f32": 1e-5, "bf16": 2e-3}


def check_decode_unit(w, got_out, got_tau, got_supp, got_tokens, ref, boundary_expected=False):
    """One (b, h) unit of a decode against the oracle's entmax_attention result `ref` over the same candidate set:
    tau to 4e-6, output to OUT_TOL, support identical except tokens on the float32 resolution boundary of tau.
    `boundary_expected`: the input was built to crowd thousands of scores around tau (flat attention), so even a
    float32 cache may have a token inside the boundary band; the rule itself is unchanged."""
    tol = OUT_TOL[w.kv_dtype]
    assert abs(got_tau - ref["tau"]) <= 4e-6 * max(1.0, abs(ref["tau"])), (got_tau, ref["tau"])
    # tokens whose z sits within float32 resolution of tau may fall on either side; everything else
    # must match exactly.  On the float32-cache workloads the seeded inputs have no such token.
    z = (w.alpha - 1.0) * ref["s"]
    boundary = set(ref["tokens"][np.abs(z - ref["tau"]) <= 2e-6 * max(1.0, abs(ref["tau"]))].tolist())
    if w.kv_dtype == "f32" and not boundary_expected:
        assert not boundary, "seeded float32 input has a token on the support boundary"
    assert abs(got_supp - len(ref["support"])) <= len(boundary)
    if got_tokens is not None:
        diff = set(got_tokens[:got_supp].tolist()).symmetric_difference(ref["support"].tolist())
        assert diff.issubset(boundary), sorted(diff)
        assert np.all(np.diff(got_tokens[:got_supp]) > 0)
    assert rel_err(got_out, ref["o"]) <= tol, rel_err(got_out, ref["o"])


def check_decode_of_gpu_list(w, q, K, V, gpu_pages, got_out, got_tau, got_supp, got_tokens=None):
    """The decode of a page list the GPU selected, against the oracle's decode of THAT list -- whether or not the
    list equals the oracle's own selection (pages inside the tie band of the cut may differ; the decode is unique
    for any given list).  Returns the oracle result."""
    tok = orc.pages_to_tokens(np.asarray(gpu_pages), w.page_size, K.shape[0])
    ref = orc.entmax_attention(q, K, V, w.alpha, w.score_scale, tok)
    check_decode_unit(w, np.asarray(got_out), float(got_tau), int(got_supp), got_tokens, ref)
    return ref
