"""Shared test plumbing: device buffers for a workload, and the oracle run per (b, h) unit.

The oracle never sees anything produced by the HIP path; where a stage test needs "the same stored
statistics / scores on both sides", the oracle's values are uploaded to the GPU, never the reverse."""
import math
import numpy as np
import torch

from oracle import entmaxkv_oracle as orc
from paper_2605_21649_amd import binding as ekv
from paper_2605_21649_amd import synth
from paper_2605_21649_amd.device_state import DeviceState  # noqa: F401  (re-exported for the tests)


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
