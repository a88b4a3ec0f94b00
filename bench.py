#!/usr/bin/env python3
"""Decode-step benchmark of the EntmaxKV hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--budget 0.02] [--variant topk]

One step = one decode step of the top-k variant over a synthetic paged cache already resident in HBM:
  a2 append the new token + refresh its page statistics and a3 box page scoring (one launch:
  ekv_append_score_pages) -> a5 top-k selection -> a7 sparse alpha-entmax decode (exact tau).
The same run also times, outside the headline number, the Gaussian-selector step (a4 + a6 + a7), the
group-shared top-k step, the dense full-cache entmax decode (a8), the softmax-over-selection baseline (a9),
the box-threshold refinement, the bulk statistics build (a1), and the same steps on the 128K-token batch
workload (C3).  To keep reads coming from HBM rather than the 256 MB last-level cache, the step rotates
over several identical copies of the cache and its statistics.

Prints ONE JSON line: metric/value = mean latency of the K timed steps in
microseconds; `roofline` for the longest single kernel of the step; `cpu_baseline` = the float64 oracle
timed on this machine's host cores on a bounded sample of (batch, head) units.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch from the committed counter runs (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, each scaled by
# the same counter's reading for a plain copy of known size): NOT measured in this run, copied from
# profiles/bench_topk_step_C4.md, and valid for the C4 workload at the default budget only.
#   page scoring with the append inside (the launch the step runs): 256.32 MiB read + 8.02 MiB written;
#   without the append: 256.12 + 8.00;  score pass of the sparse decode: PMC_TRAFFIC_DECODE_SCORES_C4
PMC_TRAFFIC_SOURCE = "profiles/bench_topk_step_C4.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy)"
PMC_TRAFFIC_SCORE_PAGES_C4 = {True: int((256.32 + 8.02) * 1024 * 1024), False: int((256.12 + 8.00) * 1024 * 1024)}
PMC_TRAFFIC_DECODE_SCORES_C4 = int((166.69 + 2.88) * 1024 * 1024)

# the append runs inside the scoring launch (ekv_append_score_pages) unless --two-launch-append is given
STAGE_NAMES = {"topk": ["append_own_launch", "append+score_box", "select_topk", "decode_sparse"],
               "gauss": ["append_own_launch", "append+score_gauss", "select_gauss", "decode_sparse"],
               "group": ["append_own_launch", "append+score_group_max", "select_topk", "decode_sparse_group"],
               "dense": ["-", "-", "-", "decode_full"],
               "topk8": ["append_own_launch", "append+score_box8", "select_topk", "decode_sparse"],
               "group8": ["append_own_launch", "append+score_box8_group_max", "select_topk", "decode_sparse_group"]}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--budget", type=float, default=0.02, help="top-k budget as a fraction of the pages")
    ap.add_argument("--variant", default="topk", choices=["topk", "gauss", "group", "dense", "topk8", "group8"],
                    help="step timed as the headline: top-k (default, the metric's variant), Gaussian selector, "
                         "group-shared top-k, or the dense full-cache decode alone (for profiling the other rows)")
    ap.add_argument("--copies", type=int, default=4, help="rotating copies of the cache (defeats the LLC)")
    ap.add_argument("--q-page", type=float, default=0.99)
    ap.add_argument("--cap-frac", type=float, default=0.04,
                    help="capacity of the page lists as a fraction of the pages (room for the adaptive selector)")
    ap.add_argument("--two-launch-append", action="store_true",
                    help="append with its own launch (ekv_stats_append) instead of inside the scoring launch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="time only the headline step")
    ap.add_argument("--cpu-units", type=int, default=64, help="most (b,h) units the oracle is timed on (C4 has 32)")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (calibrates rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


class Runner:
    """Device state of one workload (several rotating copies) and its step functions.  Every step function
    takes a copy and, optionally, five HIP events to record between its stages."""

    def __init__(self, w, budget, n_copies, q_page, dev, cap_frac=0.04, fused_append=True):
        import torch
        from paper_2605_21649_amd import binding as ekv, synth
        from tests.device_state import DeviceState
        self.torch, self.ekv, self.w, self.dev, self.q_page = torch, ekv, w, dev, q_page
        self.fused_append = fused_append
        B, Hkv, d, P, n = w.batch, w.n_kv_heads, w.head_dim, w.page_size, w.context
        M = w.pages_per_seq
        self.k_pages = max(1, int(math.ceil(budget * M)))
        self.cap = max(self.k_pages, int(math.ceil(cap_frac * M)))     # room for the adaptive selector
        self.inp = synth.make_inputs(w, 4000, device=dev)     # seeded, generated on the GPU
        self.copies = []
        for c in range(n_copies):
            ic = self.inp if c == 0 else {k: (v.clone() if k in ("k_pool", "v_pool") else v)
                                          for k, v in self.inp.items()}
            st = DeviceState(w, ic, cap=self.cap, device=dev)
            ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
            st.ws_sparse = st.workspace(ekv.EKV_OP_DECODE_SPARSE)
            st.ws_gauss = st.workspace(ekv.EKV_OP_SELECT_GAUSS)
            st.ws_topk = st.workspace(ekv.EKV_OP_SELECT_TOPK)
            # the token appended by the step: the last token of the sequence, re-appended at n-1 every step
            st.seq_prev = (ic["seq_lens"] - 1).contiguous()
            st.cache_prev = ekv.cache_view(ic["k_pool"], ic["v_pool"], ic["block_table"], st.seq_prev)
            rows = ic["block_table"][:, (n - 1) // P].long()
            st.k_new = ic["k_pool"][rows, :, (n - 1) % P].contiguous()
            st.v_new = ic["v_pool"][rows, :, (n - 1) % P].contiguous()
            self.copies.append(st)
        # one page list per KV head shared by its G query heads (same budget of pages per list)
        self.gcfg = ekv.make_config(B, Hkv, Hkv, d, P, w.kv_dtype, w.alpha, w.score_scale, M, self.cap)
        self.gbox = torch.zeros(B, Hkv, M, device=dev)
        self.g_idx = torch.zeros(B, Hkv, self.cap, device=dev, dtype=torch.int32)
        self.g_n = torch.zeros(B, Hkv, device=dev, dtype=torch.int32)
        self.ws_gsel = torch.empty(max(256, ekv.ekv_workspace_bytes(self.gcfg, ekv.EKV_OP_SELECT_TOPK)), device=dev,
                                   dtype=torch.uint8)
        self.ws_full = None
        torch.cuda.synchronize()

    def ev(self):
        return self.torch.cuda.Event(enable_timing=True)

    def full_ws(self):
        """Scratch of the dense decode, one buffer shared by the copies."""
        if self.ws_full is None:
            self.ws_full = self.copies[0].workspace(self.ekv.EKV_OP_DECODE_FULL)
        return self.ws_full

    # ---- steps ---------------------------------------------------------------------------------
    def append_and_score(self, st, evs, mode, box=None, mu=None, sigma=None):
        """a2 + a3/a4: the new token is appended at n-1 (st.cache_prev holds the lengths before it) and the
        pages are scored over n tokens -- in one launch, or as the two separate calls."""
        ekv = self.ekv
        if evs: evs[0].record()
        if self.fused_append:
            if evs: evs[1].record()
            ekv.ekv_append_score_pages(st.cfg, st.cache_prev, st.stats(), st.k_new, st.v_new, st.inp["q"], mode,
                                       box, mu, sigma)
        else:
            ekv.ekv_stats_append(st.cfg, st.cache_prev, st.stats(), st.k_new, st.v_new)
            if evs: evs[1].record()
            ekv.ekv_score_pages(st.cfg, st.inp["q"], st.stats(), st.inp["seq_lens"], mode, box, mu, sigma)
        if evs: evs[2].record()

    def step_topk(self, st, evs=None):
        ekv = self.ekv
        self.append_and_score(st, evs, ekv.EKV_SCORE_BOX, box=st.box)
        ekv.ekv_select_topk(st.cfg, st.box, st.inp["seq_lens"], self.k_pages, st.page_idx, st.n_sel, st.ws_topk)
        if evs: evs[3].record()
        ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau, st.supp,
                              st.ws_sparse)
        if evs: evs[4].record()

    def step_gauss(self, st, evs=None):
        ekv = self.ekv
        self.append_and_score(st, evs, ekv.EKV_SCORE_GAUSS, mu=st.mu, sigma=st.sigma)
        ekv.ekv_select_gauss(st.cfg, st.mu, st.sigma, st.inp["seq_lens"], self.q_page, 0.0, st.tau_hat, st.page_idx,
                             st.n_sel, st.overflow, st.ws_gauss)
        if evs: evs[3].record()
        ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau, st.supp,
                              st.ws_sparse)
        if evs: evs[4].record()

    def step_gauss_seeded(self, st, evs=None):
        """The Gaussian step with tau-hat handed to the decode as the solver's starting point."""
        ekv = self.ekv
        if not hasattr(st, "ex_seed"):
            st.evals = self.torch.zeros_like(st.supp)
            st.ex_seed = ekv.decode_extras(tau_seed=st.tau_hat, solve_evals=st.evals)
        self.append_and_score(st, evs, ekv.EKV_SCORE_GAUSS, mu=st.mu, sigma=st.sigma)
        ekv.ekv_select_gauss(st.cfg, st.mu, st.sigma, st.inp["seq_lens"], self.q_page, 0.0, st.tau_hat, st.page_idx,
                             st.n_sel, st.overflow, st.ws_gauss)
        if evs: evs[3].record()
        ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau, st.supp,
                              st.ws_sparse, extras=st.ex_seed)
        if evs: evs[4].record()

    def step_topk8(self, st, evs=None):
        """Top-k step selecting on the 8-bit page bounds (half the metadata bytes)."""
        ekv = self.ekv
        self.append_and_score(st, evs, ekv.EKV_SCORE_BOX8, box=st.box)
        ekv.ekv_select_topk(st.cfg, st.box, st.inp["seq_lens"], self.k_pages, st.page_idx, st.n_sel, st.ws_topk)
        if evs: evs[3].record()
        ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau, st.supp,
                              st.ws_sparse)
        if evs: evs[4].record()

    def step_group8(self, st, evs=None):
        ekv = self.ekv
        self.append_and_score(st, evs, ekv.EKV_SCORE_BOX8 | ekv.EKV_SCORE_GROUP_MAX, box=self.gbox)
        ekv.ekv_select_topk(self.gcfg, self.gbox, st.inp["seq_lens"], self.k_pages, self.g_idx, self.g_n, self.ws_gsel)
        if evs: evs[3].record()
        ekv.ekv_decode_sparse_group(st.cfg, st.inp["q"], st.cache(), self.g_idx, self.g_n, st.out, st.tau, st.supp,
                                    st.ws_sparse)
        if evs: evs[4].record()

    def step_group(self, st, evs=None):
        ekv = self.ekv
        self.append_and_score(st, evs, ekv.EKV_SCORE_BOX | ekv.EKV_SCORE_GROUP_MAX, box=self.gbox)
        ekv.ekv_select_topk(self.gcfg, self.gbox, st.inp["seq_lens"], self.k_pages, self.g_idx, self.g_n, self.ws_gsel)
        if evs: evs[3].record()
        ekv.ekv_decode_sparse_group(st.cfg, st.inp["q"], st.cache(), self.g_idx, self.g_n, st.out, st.tau, st.supp,
                                    st.ws_sparse)
        if evs: evs[4].record()

    def step_dense(self, st, evs=None):
        if self.ws_full is None:                              # one scratch shared by the copies
            self.ws_full = self.copies[0].workspace(self.ekv.EKV_OP_DECODE_FULL)
        if evs:
            for e in evs[:4]: e.record()
        self.ekv.ekv_decode_full(st.cfg, st.inp["q"], st.cache(), st.out, st.tau, st.supp, self.ws_full)
        if evs: evs[4].record()

    def step(self, variant):
        return {"topk": self.step_topk, "gauss": self.step_gauss, "group": self.step_group,
                "dense": self.step_dense, "topk8": self.step_topk8, "group8": self.step_group8}[variant]

    # ---- timing --------------------------------------------------------------------------------
    def run_timed(self, step_fn, steps, warmup, stages=True):
        """W untimed steps, then exactly K steps between two synchronisations (wall clock, nothing but the
        step's own launches in the timed region).  A second pass of K steps records HIP events between the
        stages on the launch stream for the per-stage breakdown; the markers sit between dependent kernels
        and cost a little, so that pass is not the headline number."""
        import numpy as np
        torch, copies = self.torch, self.copies
        for i in range(warmup):
            step_fn(copies[i % len(copies)])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step_fn(copies[i % len(copies)])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        if not stages:
            return wall / steps * 1e6, None, None
        all_evs = [[self.ev() for _ in range(5)] for _ in range(steps)]
        for i in range(steps):
            step_fn(copies[i % len(copies)], all_evs[i])
        torch.cuda.synchronize()
        stage = np.array([[es[j].elapsed_time(es[j + 1]) * 1e3 for j in range(4)] for es in all_evs])   # us
        whole = np.array([es[0].elapsed_time(es[4]) * 1e3 for es in all_evs])
        return wall / steps * 1e6, stage, whole

    def back_to_back(self, fn, reps=60, warm=6):
        """Average launch duration of one entry point: N launches queued back to back on the launch stream
        between two HIP events (no marker between dependent kernels), rotating over the cache copies."""
        copies = self.copies
        for i in range(warm):
            fn(copies[i % len(copies)])
        a, b = self.ev(), self.ev()
        a.record()
        for i in range(reps):
            fn(copies[i % len(copies)])
        b.record()
        self.torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

    def time_call(self, fn, reps=20, warm=3):
        """Median duration of single calls, each bracketed by its own events and a synchronisation."""
        import numpy as np
        copies = self.copies
        for i in range(warm):
            fn(copies[i % len(copies)])
        self.torch.cuda.synchronize()
        ts = []
        for i in range(reps):
            a, b = self.ev(), self.ev()
            a.record(); fn(copies[i % len(copies)]); b.record()
            self.torch.cuda.synchronize()
            ts.append(a.elapsed_time(b) * 1e3)
        return float(np.median(ts))

    def release(self):
        self.copies = []
        self.inp = None
        self.ws_full = None
        self.torch.cuda.empty_cache()


# ---- CPU baseline: the float64 oracle's whole top-k step, one thread and all cores ----------------------------
def _bf16_bits_to_f64(bits):
    import numpy as np
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _cpu_worker(task):
    """One process of the all-core leg: loads the K and V of its KV heads (raw cache values written by the parent),
    waits until every process is ready, then times the oracle on its units.  No GPU, no torch."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import entmaxkv_oracle as orc
    threadpool_limits(1)
    units, wdict, k_pages, tmpdir, ready, go, done = task
    cache, t_units = {}, 0.0
    for (b, hq) in units:
        key = (b, hq // wdict["group"])
        if key not in cache:
            raw = np.load(os.path.join(tmpdir, "kv_%d_%d.npy" % key))
            conv = _bf16_bits_to_f64 if wdict["kv_dtype"] == "bf16" else (lambda x: x.astype(np.float64))
            cache[key] = (conv(raw[0]), conv(raw[1]))
    qs = np.load(os.path.join(tmpdir, "q.npy"))
    ready.release()
    go.wait()
    t0 = time.perf_counter()
    for (b, hq) in units:
        K64, V64 = cache[(b, hq // wdict["group"])]
        orc.decode_step_unit(qs[b, hq], K64, V64, wdict["P"], wdict["alpha"], wdict["scale"], "topk", wdict["kv_dtype"],
                             k_pages=k_pages)
    t_units = time.perf_counter() - t0
    done.put(t_units)


def cpu_baseline(inp, w, k_pages, max_units):
    """The oracle (numpy float64, never tuned for this) over (batch, head) units of the benchmark's own inputs:
    one thread over every unit, then all host cores (one process per core, units split evenly), no extrapolation
    unless the workload has more units than `max_units`."""
    import multiprocessing as mp
    import shutil
    import tempfile
    import numpy as np
    import torch
    from oracle import entmaxkv_oracle as orc
    from paper_2605_21649_amd import synth
    from tests.helpers import to_f64
    from threadpoolctl import threadpool_limits
    B, Hq, P = w.batch, w.n_q_heads, w.page_size
    all_units = [(b, h) for b in range(B) for h in range(Hq)]
    units = all_units[: max(1, min(max_units, len(all_units)))]
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    # raw cache values of the KV heads involved, for the worker processes (bf16 bit patterns: 2 bytes per element)
    shm = "/dev/shm" if os.path.isdir("/dev/shm") and shutil.disk_usage("/dev/shm").free > (8 << 30) else None
    tmpdir = tempfile.mkdtemp(prefix="ekv_cpu_", dir=shm)
    try:
        for key in sorted({(b, hq // w.group) for (b, hq) in units}):
            k_t, v_t = synth.logical_kv(inp, w, key[0], key[1])
            kv = torch.stack([k_t, v_t]).cpu()
            raw = kv.view(torch.int16).numpy().view(np.uint16) if w.kv_dtype == "bf16" else kv.numpy()
            np.save(os.path.join(tmpdir, "kv_%d_%d.npy" % key), raw)
            del k_t, v_t, kv, raw
        np.save(os.path.join(tmpdir, "q.npy"), to_f64(inp["q"]))
        # ---- one thread, every unit
        t_one, kv_key, K64, V64 = 0.0, None, None, None
        with threadpool_limits(1):
            for (b, hq) in units:
                if kv_key != (b, hq // w.group):                   # heads of one group share the K/V conversion
                    K64 = V64 = None
                    k_t, v_t = synth.logical_kv(inp, w, b, hq // w.group)
                    K64, V64 = to_f64(k_t), to_f64(v_t)
                    kv_key = (b, hq // w.group)
                    del k_t, v_t
                q64 = to_f64(inp["q"][b, hq])
                t0 = time.perf_counter()
                orc.decode_step_unit(q64, K64, V64, P, w.alpha, w.score_scale, "topk", w.kv_dtype, k_pages=k_pages)
                t_one += time.perf_counter() - t0
        K64 = V64 = None
        # ---- all cores: one process per core (fresh interpreters that never touch the GPU), units split evenly
        n_proc = max(1, min(cores, len(units)))
        chunks = [units[i * len(units) // n_proc:(i + 1) * len(units) // n_proc] for i in range(n_proc)]
        ctx = mp.get_context("spawn")
        ready, go, done = ctx.Semaphore(0), ctx.Event(), ctx.Queue()
        wdict = dict(group=w.group, kv_dtype=w.kv_dtype, P=P, alpha=w.alpha, scale=w.score_scale)
        procs = [ctx.Process(target=_cpu_worker, args=((c, wdict, k_pages, tmpdir, ready, go, done),)) for c in chunks]
        for pr in procs:
            pr.start()
        for _ in procs:
            ready.acquire()
        t0 = time.perf_counter()
        go.set()
        busy = [done.get() for _ in procs]
        t_all = time.perf_counter() - t0
        for pr in procs:
            pr.join()
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    scale_up = len(all_units) / len(units)
    note = "" if len(units) == len(all_units) else f"; {len(units)} of {len(all_units)} units timed, values scaled by {scale_up:.2f}"
    return {
        "value": round(t_all * scale_up * 1e6, 1), "unit": "us", "cores": n_proc, "kind": "oracle",
        "one_thread": {"value": round(t_one * scale_up * 1e6, 1), "unit": "us", "cores": 1},
        "host_cores_available": cores,
        "sample": f"float64 numpy oracle, whole top-k step (stats + box score + top-k + sparse entmax) of "
                  f"{len(units)} (batch, head) units of the benchmark's own inputs: {t_one:.1f} s on one thread, "
                  f"{t_all:.1f} s wall with {n_proc} single-threaded processes (slowest process busy {max(busy):.1f} s)" + note,
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(every (sequence, KV head) unit is independent, so more GPUs would take disjoint units).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_21649_amd import binding as ekv, synth
    from tests.device_state import DeviceState

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    ekv.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.WORKLOADS[args.workload]
    B, Hq, Hkv, d, P, n = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.page_size, w.context
    M = w.pages_per_seq
    e = 2 if w.kv_dtype == "bf16" else 4
    R = Runner(w, args.budget, args.copies, args.q_page, dev, args.cap_frac, fused_append=not args.two_launch_append)
    k_pages, copies = R.k_pages, R.copies
    stage_names = STAGE_NAMES[args.variant]
    if args.variant in ("topk8", "group8"):      # the 8-bit bounds exist only where a step reads them
        for st in copies:
            st.enable_box8()
            ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
        torch.cuda.synchronize()

    if args.pmc_copy:
        # a plain copy of known size: 1 GiB read + 1 GiB written by one elementwise kernel
        src = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------------------------------------------------------- headline: top-k step
    us_wall, stage, whole = R.run_timed(R.step(args.variant), args.steps, args.warmup)
    if args.variant != "topk":       # the byte accounting below is the top-k step's: leave its lists in place
        R.step_topk(copies[0]); torch.cuda.synchronize()
    stage_mean = stage.mean(axis=0)
    st0 = copies[0]
    supp_mean = float(st0.supp.float().mean())
    n_sel_mean = float(st0.n_sel.float().mean())

    # algorithmic bytes of the step: box metadata + selected K pages +
    # support V rows + score scratch (written then read once)
    sel_tokens = n_sel_mean * P
    bytes_meta = B * Hkv * M * 2 * d * e
    bytes_scores = B * Hq * M * 4 * 2
    bytes_k = B * Hq * sel_tokens * d * e
    bytes_v = B * Hq * supp_mean * d * e
    bytes_z = B * Hq * sel_tokens * 4 * 2
    step_bytes = bytes_meta + bytes_scores + bytes_k + bytes_v + bytes_z
    dense_bytes = B * Hkv * n * 2 * d * e

    # per-entry-point launch durations, measured live
    t_append = R.back_to_back(lambda st: ekv.ekv_stats_append(st.cfg, st.cache_prev, st.stats(), st.k_new, st.v_new))
    t_score = R.back_to_back(lambda st: ekv.ekv_score_pages(st.cfg, st.inp["q"], st.stats(), st.inp["seq_lens"],
                                                            ekv.EKV_SCORE_BOX, st.box))
    t_fused = R.back_to_back(lambda st: ekv.ekv_append_score_pages(st.cfg, st.cache_prev, st.stats(), st.k_new, st.v_new,
                                                                   st.inp["q"], ekv.EKV_SCORE_BOX, st.box))
    t_topk = R.back_to_back(lambda st: ekv.ekv_select_topk(st.cfg, st.box, st.inp["seq_lens"], k_pages, st.page_idx,
                                                           st.n_sel, st.ws_topk))
    t_dec = R.back_to_back(lambda st: ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel,
                                                            st.out, st.tau, st.supp, st.ws_sparse))
    ex_pass1 = ekv.decode_extras(score_pass_only=True)
    t_dec_scores = R.back_to_back(lambda st: ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel,
                                                                   st.out, st.tau, st.supp, st.ws_sparse, extras=ex_pass1))
    kernel_alg_bytes = {
        "stats_append": None,
        "score_pages(box)": bytes_meta + B * Hq * M * 4,                 # metadata read + scores written
        "append_score_pages(box)": bytes_meta + B * Hq * M * 4,
        "select_topk": B * Hq * M * 4,                                   # scores read (once, algorithmically)
        "decode_sparse": bytes_k + bytes_v + bytes_z,
    }
    kernel_us = {"stats_append": t_append, "score_pages(box)": t_score, "append_score_pages(box)": t_fused,
                 "select_topk": t_topk, "decode_sparse": t_dec}
    kernels = {}
    for nm, us in kernel_us.items():
        nb = kernel_alg_bytes[nm]
        kernels[nm] = {"launch_us": round(us, 2), "algorithmic_bytes": None if nb is None else int(nb),
                       "GBps": None if nb is None else round(nb / (us * 1e-6) / 1e9, 1)}
    kernels["select_topk"]["kernels"] = 3       # histogram, find, compaction (latency-bound, not a stream)
    kernels["decode_sparse"]["kernels"] = 2     # score pass (HBM-bound gather) + single-workgroup solve

    # The roofline entry is for the longest single kernel of the step: the page-scoring stream
    # (score_pages_mfma_kernel; the instantiation with the append inside when the step uses the fused call).
    # select_topk and decode_sparse are several shorter kernels each; the committed kernel trace under
    # profiles/ lists them one by one.
    roof_key = "append_score_pages(box)" if R.fused_append else "score_pages(box)"
    roof_us = t_fused if R.fused_append else t_score
    roof_bytes = kernel_alg_bytes[roof_key]
    achieved = roof_bytes / (roof_us * 1e-6) / 1e9
    # HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE counter runs (profiles/bench_topk_step_C4.md);
    # they hold for the workload those runs used
    pmc_traffic = {"C4": PMC_TRAFFIC_SCORE_PAGES_C4[bool(R.fused_append)]}
    roofline = {
        "bound": "hbm",
        "kernel": "score_pages_mfma_kernel<%d, 0, %s> (%s)" % (w.group, "true" if R.fused_append else "false",
                                                              "ekv_append_score_pages" if R.fused_append
                                                              else "ekv_score_pages"),
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": pmc_traffic.get(args.workload),
        "algorithmic_bytes_per_launch": int(roof_bytes), "avg_launch_us": round(roof_us, 2),
        "timing": "HIP events around 60 back-to-back launches on the launch stream, %d rotating copies" % args.copies,
    }
    roofline["traffic_source"] = PMC_TRAFFIC_SOURCE if roofline["traffic"] is not None else None
    # The sparse entmax decode itself (a7): its HBM-bound kernel is the score pass (gather of the selected K pages,
    # scores and group maxima written), timed alone through the score_pass_only measurement flag; `call` is the
    # whole entry point (score pass + solve, which also reads the V rows of the support).
    a7_bytes = bytes_k + bytes_z / 2 + B * Hq * sel_tokens / 64 * 4        # K pages read, z and group maxima written
    a7_ach = a7_bytes / (t_dec_scores * 1e-6) / 1e9
    call_ach = kernel_alg_bytes["decode_sparse"] / (t_dec * 1e-6) / 1e9
    roofline_a7 = {
        "bound": "hbm", "kernel": "decode_scores_mfma_kernel<1, 0, %d> (score pass of ekv_decode_sparse)" % P,
        "achieved": round(a7_ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(a7_ach / HBM_PEAK_GBS, 4),
        "traffic": PMC_TRAFFIC_DECODE_SCORES_C4 if (args.workload == "C4" and abs(args.budget - 0.02) < 1e-9) else None,
        "algorithmic_bytes_per_launch": int(a7_bytes), "avg_launch_us": round(t_dec_scores, 2),
        "call": {"entry_point": "ekv_decode_sparse (score pass + solve)", "avg_us": round(t_dec, 2),
                 "algorithmic_bytes": int(kernel_alg_bytes["decode_sparse"]), "GBps": round(call_ach, 1),
                 "frac": round(call_ach / HBM_PEAK_GBS, 4)},
        "timing": "HIP events around 60 back-to-back launches on the launch stream, %d rotating copies" % args.copies,
    }
    roofline_a7["traffic_source"] = PMC_TRAFFIC_SOURCE if roofline_a7["traffic"] is not None else None
    kernels["decode_sparse(score pass only)"] = {"launch_us": round(t_dec_scores, 2), "algorithmic_bytes": int(a7_bytes),
                                                 "GBps": round(a7_ach, 1), "kernels": 1}
    dom_name = stage_names[int(np.argmax(stage_mean))]

    result = {
        "metric": "decode-step latency", "value": round(us_wall, 2), "unit": "us", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us_wall / 1e3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic", "kv_dtype": w.kv_dtype,
        "config": {"workload": f"{w.name}: B{B} {Hq}q/{Hkv}kv d{d} ctx{n} page{P} {w.kv_dtype}, alpha={w.alpha}, "
                               f"top-k {k_pages} pages ({args.budget:.0%}) per query head",
                   "variant": "entmaxkv-" + args.variant, "copies_rotated": args.copies,
                   "append": "own launch" if args.two_launch_append else "inside the scoring launch"},
        "step_event_us": {"mean": round(float(whole.mean()), 2), "median": round(float(np.median(whole)), 2),
                          "p10": round(float(np.percentile(whole, 10)), 2),
                          "p90": round(float(np.percentile(whole, 90)), 2)},
        "stage_us": {nm: round(float(v), 2) for nm, v in zip(stage_names, stage_mean)},
        "dominant_stage": dom_name,
        "step_algorithmic_bytes": int(step_bytes),
        "effective_kv_GBps": round(step_bytes / (us_wall * 1e-6) / 1e9, 1),
        "effective_kv_frac_of_hbm_peak": round(step_bytes / (us_wall * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
        "dense_equivalent_GBps": round(dense_bytes / (us_wall * 1e-6) / 1e9, 1),
        "selected_pages_mean": n_sel_mean, "support_mean": supp_mean,
        "roofline": roofline,
        "roofline_a7": roofline_a7,
        "kernels": kernels,
    }

    # ---------------------------------------------------------------- the other rows, same run
    if not args.no_extras:
        extras = {}
        # The ceiling a read-only kernel reaches on this GPU (ekv_probe_read: pages of the K pools of the rotating
        # copies, 16-byte loads, nothing else), next to the published peak: the whole pool as a linear stream and
        # in permuted page order, and exactly the pages the sparse decode gathers (same list order, 4 KiB blocks of
        # (page, KV head)) -- bare, and with the score pass's second lookup and 256 B of output per wavefront.
        page_bytes = P * d * e
        if page_bytes in (4096, 8192):
            n_blocks = st0.inp["k_pool"].shape[0] * Hkv               # (page, KV head) blocks of one pool
            sink = torch.zeros(64, dtype=torch.int32, device=dev)
            gperm = torch.Generator(device=dev).manual_seed(123)
            ids_lin = torch.arange(n_blocks, dtype=torch.int32, device=dev)
            ids_perm = torch.randperm(n_blocks, generator=gperm, device=dev).to(torch.int32)
            # blocks of the step's own selection: physical page of every selected logical page, this head's KV head
            hkv_of = (torch.arange(Hq, device=dev) // w.group).view(1, Hq, 1)
            sel = st0.page_idx[:, :, :k_pages].long()
            phys = torch.gather(st0.inp["block_table"].long().unsqueeze(1).expand(B, Hq, M), 2, sel)
            ids_sel = (phys * Hkv + hkv_of).reshape(-1).to(torch.int32).contiguous()
            out_probe = torch.empty((ids_sel.numel() + 3) // 4 * 64, dtype=torch.float32, device=dev)

            def probe_rate(ids, lookup=None, out=None, reps=20):
                nn = ids.numel()
                us = R.back_to_back(lambda st: ekv.ekv_probe_read(st.inp["k_pool"], ids, nn, page_bytes, sink,
                                                                  lookup=lookup, out=out), reps=reps, warm=3)
                return {"us": round(us, 2), "bytes": int(nn * page_bytes), "GBps": round(nn * page_bytes / (us * 1e-6) / 1e9, 1)}
            extras["read_ceiling"] = {
                "kernel": "ekv_probe_read (probe_read_kernel): read-only, four pages per wavefront",
                "whole_pool_linear": probe_rate(ids_lin, reps=8),
                "whole_pool_permuted_pages": probe_rate(ids_perm, reps=8),
                "selected_pages_of_the_step": probe_rate(ids_sel),
                "selected_pages_with_lookup_and_output": probe_rate(ids_sel, lookup=ids_lin, out=out_probe),
                "note": "the last row has the memory behaviour of the decode's score pass (two dependent lookups, "
                        "256 B written per 64 tokens) without its arithmetic",
            }
            del ids_lin, ids_perm, ids_sel, out_probe, phys, sel
        # Fusing two dependent stages into one launch needs a hand-off between workgroups inside the kernel; what
        # that costs here against a plain launch of the same shape (512 workgroups x 4 KiB: the top-k histogram
        # kernel's shape), by mechanism (ekv_probe_handoff)
        hd = torch.zeros(512 * 1024, dtype=torch.float32, device=dev)
        hc = torch.zeros(1, dtype=torch.int32, device=dev); ho = torch.zeros(1, dtype=torch.float32, device=dev)
        extras["handoff_inside_a_launch_us"] = {
            name: round(R.back_to_back(lambda st: ekv.ekv_probe_handoff(hd, hc, ho, 512, mode), reps=30, warm=3), 2)
            for mode, name in ((0, "no_handoff"), (1, "device_fence_last_arriver"), (2, "write_through_atomics_last_arriver"))}
        # the sparse decode against the CAPACITY of its page lists (max_sel_pages): the same lists of k pages in
        # buffers of 1x, 2x and 8x that capacity -- the launch is sized by the device-side lengths, not by the capacity
        by_cap = {}
        for mult in (1, 2, 8):
            cap_m = min(M, k_pages * mult)
            cfg_m = ekv.make_config(B, Hq, Hkv, d, P, w.kv_dtype, w.alpha, w.score_scale, M, cap_m)
            idx_m = torch.zeros(B, Hq, cap_m, dtype=torch.int32, device=dev)
            idx_m[:, :, :k_pages] = st0.page_idx[:, :, :k_pages]
            ws_m = torch.empty(max(256, ekv.ekv_workspace_bytes(cfg_m, ekv.EKV_OP_DECODE_SPARSE)), dtype=torch.uint8, device=dev)
            by_cap[f"{mult}x"] = round(R.back_to_back(
                lambda st: ekv.ekv_decode_sparse(cfg_m, st.inp["q"], st.cache(), idx_m, st0.n_sel, st0.out, st0.tau,
                                                 st0.supp, ws_m), reps=40), 2)
            del idx_m, ws_m
        extras["decode_sparse_us_by_list_capacity"] = by_cap
        side = max(10, args.steps // 4)
        if R.fused_append:                                     # the same step with the append as its own launch
            R.fused_append = False
            us_2l, _, _ = R.run_timed(R.step_topk, side, 5, stages=False)
            R.fused_append = True
            extras["topk_step_two_launch_append_us"] = round(us_2l, 2)
        us_g, stage_g, _ = R.run_timed(R.step_gauss, side, 5)
        extras["gauss_step_us"] = round(us_g, 2)
        extras["gauss_stage_us"] = {nm: round(float(v), 2) for nm, v in zip(STAGE_NAMES["gauss"], stage_g.mean(axis=0))}
        extras["gauss_selected_pages_mean"] = float(copies[0].n_sel.float().mean())
        # warm start: tau-hat as the solver's first iterate (Sec. 4.3); evaluations of the mass per solve
        st0_ = copies[0]
        ev_plain = torch.zeros_like(st0_.supp)
        ekv.ekv_decode_sparse(st0_.cfg, st0_.inp["q"], st0_.cache(), st0_.page_idx, st0_.n_sel, st0_.out, st0_.tau,
                              st0_.supp, st0_.ws_sparse, extras=ekv.decode_extras(solve_evals=ev_plain))
        us_gs, _, _ = R.run_timed(R.step_gauss_seeded, side, 5, stages=False)
        extras["gauss_step_tau_hat_seeded_us"] = round(us_gs, 2)
        extras["gauss_solve_evals_mean"] = {"unseeded": round(float(ev_plain.float().mean()), 2),
                                            "tau_hat_seeded": round(float(st0_.evals.float().mean()), 2)}
        extras["gauss_overflow"] = int(copies[0].overflow.sum())
        ws_full = copies[0].workspace(ekv.EKV_OP_DECODE_FULL)       # one scratch shared by the copies
        out_f, tau_f, supp_f = torch.zeros_like(st0.out), torch.zeros_like(st0.tau), torch.zeros_like(st0.supp)
        dense_us = R.time_call(lambda st: ekv.ekv_decode_full(st.cfg, st.inp["q"], st.cache(), out_f, tau_f, supp_f,
                                                              ws_full), reps=10)
        extras["dense_full_us"] = round(dense_us, 2)
        extras["dense_full_GBps"] = round((dense_bytes / 2 + B * Hq * n * 8) / (dense_us * 1e-6) / 1e9, 1)
        extras["speedup_vs_dense"] = round(dense_us / us_wall, 2)
        extras["speedup_gauss_vs_dense"] = round(dense_us / us_g, 2)
        # dropped mass / support recall of the top-k selection against the dense threshold (GPU side outputs)
        kept_mass = torch.zeros_like(st0.tau); kept_supp = torch.zeros_like(st0.supp)
        # ... first of the Gaussian-aware selection (adaptive number of pages per head)
        R.step_gauss(st0)
        ekv.ekv_decode_sparse(st0.cfg, st0.inp["q"], st0.cache(), st0.page_idx, st0.n_sel, st0.out, st0.tau,
                              st0.supp, st0.ws_sparse,
                              extras=ekv.decode_extras(tau_ref=tau_f, kept_mass_ref=kept_mass, kept_supp_ref=kept_supp))
        torch.cuda.synchronize()
        extras["gauss_quality"] = {
            "pages_per_head_mean": float(st0.n_sel.float().mean()), "pages_per_head_max": int(st0.n_sel.max()),
            "delta_mean": round(float((1.0 - kept_mass).mean()), 6),
            "rho_mean": round(float((kept_supp.float() / supp_f.float()).mean()), 4),
            "R_mean": round(float(((st0.out - out_f).norm(dim=-1) / out_f.norm(dim=-1)).mean()), 6)}
        for frac in (0.01, 0.02, 0.04):
            kp = max(1, int(math.ceil(frac * M)))
            ekv.ekv_select_topk(st0.cfg, st0.box, st0.inp["seq_lens"], kp, st0.page_idx, st0.n_sel, st0.ws_topk)
            ekv.ekv_decode_sparse(st0.cfg, st0.inp["q"], st0.cache(), st0.page_idx, st0.n_sel, st0.out, st0.tau,
                                  st0.supp, st0.ws_sparse,
                                  extras=ekv.decode_extras(tau_ref=tau_f, kept_mass_ref=kept_mass, kept_supp_ref=kept_supp))
            torch.cuda.synchronize()
            Rerr = ((st0.out - out_f).norm(dim=-1) / out_f.norm(dim=-1)).mean()
            R.k_pages = kp                                         # whole step at this budget
            us_b, _, _ = R.run_timed(R.step_topk, side, 5, stages=False)
            R.k_pages = k_pages
            sel_b = B * Hq * kp * P
            # the score pass of the sparse decode alone at this budget (every copy holds this budget's lists now): its
            # fixed costs (the dependent lookups in front of a wavefront's first K load, the last wavefronts of the
            # launch) weigh less the more there is to read
            t_sp = R.back_to_back(lambda st: ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel,
                                                                   st.out, st.tau, st.supp, st.ws_sparse, extras=ex_pass1))
            sp_bytes = sel_b * d * e + sel_b * 4 + sel_b / 64 * 4
            extras[f"topk_{frac:.0%}"] = {
                "pages_per_head": kp, "step_us": round(us_b, 2),
                "decode_score_pass_us": round(t_sp, 2),
                "decode_score_pass_GBps": round(sp_bytes / (t_sp * 1e-6) / 1e9, 1),
                "decode_score_pass_frac_of_hbm_peak": round(sp_bytes / (t_sp * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                "effective_kv_GBps": round((bytes_meta + bytes_scores + sel_b * (d * e + 8)) / (us_b * 1e-6) / 1e9, 1),
                "delta_mean": round(float((1 - kept_mass).mean()), 6),
                "rho_mean": round(float((kept_supp.float() / supp_f.float()).mean()), 4),
                "R_mean": round(float(Rerr), 6)}
        # throughput with two independent steps in flight (two sequences or layers: rotating copies here) on two
        # streams: the latency-bound selection and solve of one run under the HBM-bound streams of the other
        sA, sB = torch.cuda.Stream(), torch.cuda.Stream()
        def two_in_flight(nsteps):
            for i in range(nsteps // 2):
                with torch.cuda.stream(sA): R.step_topk(copies[(2 * i) % len(copies)])
                with torch.cuda.stream(sB): R.step_topk(copies[(2 * i + 1) % len(copies)])
        torch.cuda.synchronize()
        two_in_flight(20); torch.cuda.synchronize()
        t0 = time.perf_counter()
        two_in_flight(2 * side); torch.cuda.synchronize()
        extras["topk_two_independent_steps_in_flight_us_per_step"] = round((time.perf_counter() - t0) / (2 * side) * 1e6, 2)
        us_gr, stage_gr, _ = R.run_timed(R.step_group, side, 5)
        extras["group_shared_step_us"] = round(us_gr, 2)
        extras["group_shared_stage_us"] = {nm: round(float(v), 2) for nm, v in
                                           zip(STAGE_NAMES["group"], stage_gr.mean(axis=0))}
        extras["speedup_group_shared_vs_dense"] = round(dense_us / us_gr, 2)
        # 64 consecutive decode steps: the sequence grows by one token per step (the length is bumped on the
        # device between steps, page boundaries are crossed every P steps), nothing is synchronised in between
        T = 64
        seq = st0.inp["seq_lens"]                              # shared by the copies
        seq_full = seq.clone()
        pos = [n - T + t for t in range(T)]
        rows_t = [st0.inp["block_table"][:, p_ // P].long() for p_ in pos]
        k_news = [st0.inp["k_pool"][rows_t[t], :, pos[t] % P].contiguous() for t in range(T)]
        v_news = [st0.inp["v_pool"][rows_t[t], :, pos[t] % P].contiguous() for t in range(T)]

        def run_loop():
            seq.fill_(n - T)
            for t in range(T):
                st = copies[t % len(copies)]
                if R.fused_append:
                    ekv.ekv_append_score_pages(st.cfg, st.cache(), st.stats(), k_news[t], v_news[t], st.inp["q"],
                                               ekv.EKV_SCORE_BOX, st.box)
                    seq.add_(1)
                else:
                    ekv.ekv_stats_append(st.cfg, st.cache(), st.stats(), k_news[t], v_news[t])
                    seq.add_(1)
                    ekv.ekv_score_pages(st.cfg, st.inp["q"], st.stats(), seq, ekv.EKV_SCORE_BOX, st.box)
                ekv.ekv_select_topk(st.cfg, st.box, seq, k_pages, st.page_idx, st.n_sel, st.ws_topk)
                ekv.ekv_decode_sparse(st.cfg, st.inp["q"], st.cache(), st.page_idx, st.n_sel, st.out, st.tau,
                                      st.supp, st.ws_sparse)
        run_loop()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_loop()
        torch.cuda.synchronize()
        extras["decode_loop_us_per_step"] = round((time.perf_counter() - t0) / T * 1e6, 2)
        extras["decode_loop_steps"] = T
        # the same loop recorded once as a HIP graph (the library only launches kernels) and replayed
        graph = torch.cuda.CUDAGraph()
        cap_stream = torch.cuda.Stream()
        cap_stream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=cap_stream):
            run_loop()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        extras["decode_loop_graph_replay_us_per_step"] = round((time.perf_counter() - t0) / (3 * T) * 1e6, 2)
        del graph
        seq.copy_(seq_full)
        for st in copies:                                      # last pages back to their full statistics
            ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
        torch.cuda.synchronize()
        # exactness certificate / refinement: pages whose box bound exceeds the sparse tau (App. B.2)
        ekv.ekv_select_topk(st0.cfg, st0.box, st0.inp["seq_lens"], k_pages, st0.page_idx, st0.n_sel, st0.ws_topk)
        ekv.ekv_decode_sparse(st0.cfg, st0.inp["q"], st0.cache(), st0.page_idx, st0.n_sel, st0.out, st0.tau,
                              st0.supp, st0.ws_sparse)
        ref_idx, ref_n = torch.zeros_like(st0.page_idx), torch.zeros_like(st0.n_sel)
        n_added, ovf = torch.zeros_like(st0.n_sel), torch.zeros_like(st0.n_sel)
        ws_box = st0.workspace(ekv.EKV_OP_SELECT_BOX_THRESHOLD)
        extras["box_threshold_refine_us"] = round(R.time_call(
            lambda st: ekv.ekv_select_box_threshold(st0.cfg, st0.box, st0.inp["seq_lens"], st0.tau, st0.page_idx,
                                                    st0.n_sel, ref_idx, ref_n, n_added, ovf, ws_box), reps=10), 2)
        extras["box_threshold_pages_added_mean"] = float(n_added.float().mean())
        extras["box_threshold_overflow_heads"] = int(ovf.sum())
        lse_sel = torch.zeros_like(st0.tau)
        ws_sm = copies[0].workspace(ekv.EKV_OP_DECODE_SPARSE_SOFTMAX)
        ekv.ekv_select_topk(st0.cfg, st0.box, st0.inp["seq_lens"], k_pages, st0.page_idx, st0.n_sel, st0.ws_topk)
        extras["softmax_sparse_us"] = round(R.time_call(
            lambda st: ekv.ekv_decode_sparse_softmax(st0.cfg, st0.inp["q"], st.cache(), st0.page_idx, st0.n_sel,
                                                     st0.out, lse_sel, ws_sm), reps=10), 2)
        extras["stats_build_us"] = round(R.time_call(lambda st: ekv.ekv_stats_build(st.cfg, st.cache(), st.stats()),
                                                     reps=8), 2)
        extras["stats_build_GBps"] = round((dense_bytes / 2 + 2 * bytes_meta) / (extras["stats_build_us"] * 1e-6) / 1e9, 1)
        # Gaussian-aware selector on plain random inputs (q, K, V ~ N(0,1), batch 8, page 16, 4K-64K tokens: the
        # setting of the paper's selector-quality table, App. E): coverage, dropped mass, recall, output error
        tab = {}
        for n_t in (4096, 8192, 16384, 32768, 65536):
            wt = synth.Workload("randn", 8, 8, 8, 128, n_t, 16, "bf16")
            it = synth.make_inputs(wt, 9000 + n_t, device=dev)
            stt = DeviceState(wt, it, cap=wt.pages_per_seq, device=dev)
            ekv.ekv_stats_build(stt.cfg, stt.cache(), stt.stats())
            ekv.ekv_score_pages(stt.cfg, it["q"], stt.stats(), it["seq_lens"], ekv.EKV_SCORE_GAUSS, None, stt.mu, stt.sigma)
            ekv.ekv_select_gauss(stt.cfg, stt.mu, stt.sigma, it["seq_lens"], args.q_page, 0.0, stt.tau_hat, stt.page_idx,
                                 stt.n_sel, stt.overflow, stt.workspace(ekv.EKV_OP_SELECT_GAUSS))
            o_f, t_f, s_f = torch.zeros_like(stt.out), torch.zeros_like(stt.tau), torch.zeros_like(stt.supp)
            ekv.ekv_decode_full(stt.cfg, it["q"], stt.cache(), o_f, t_f, s_f, stt.workspace(ekv.EKV_OP_DECODE_FULL))
            km_t, ks_t = torch.zeros_like(stt.tau), torch.zeros_like(stt.supp)
            ekv.ekv_decode_sparse(stt.cfg, it["q"], stt.cache(), stt.page_idx, stt.n_sel, stt.out, stt.tau, stt.supp,
                                  stt.workspace(ekv.EKV_OP_DECODE_SPARSE),
                                  extras=ekv.decode_extras(tau_ref=t_f, kept_mass_ref=km_t, kept_supp_ref=ks_t))
            torch.cuda.synchronize()
            if n_t == 16384:
                # the top-k selector on the same inputs at several coverages (the approximation-quality figure's setting)
                tk = {}
                ekv.ekv_score_pages(stt.cfg, it["q"], stt.stats(), it["seq_lens"], ekv.EKV_SCORE_BOX, stt.box)
                idx_t, ns_t = torch.zeros_like(stt.page_idx), torch.zeros_like(stt.n_sel)
                out_t, tau_t, supp_t = torch.zeros_like(stt.out), torch.zeros_like(stt.tau), torch.zeros_like(stt.supp)
                km2, ks2 = torch.zeros_like(stt.tau), torch.zeros_like(stt.supp)
                for cov_t in (0.0625, 0.125, 0.25, 0.5):
                    kp_t = int(cov_t * wt.pages_per_seq)
                    ekv.ekv_select_topk(stt.cfg, stt.box, it["seq_lens"], kp_t, idx_t, ns_t, stt.workspace(ekv.EKV_OP_SELECT_TOPK))
                    ekv.ekv_decode_sparse(stt.cfg, it["q"], stt.cache(), idx_t, ns_t, out_t, tau_t, supp_t,
                                          stt.workspace(ekv.EKV_OP_DECODE_SPARSE),
                                          extras=ekv.decode_extras(tau_ref=t_f, kept_mass_ref=km2, kept_supp_ref=ks2))
                    torch.cuda.synchronize()
                    tk[str(cov_t)] = {"delta_mean": round(float((1.0 - km2).mean()), 5),
                                      "rho_mean": round(float((ks2.float() / s_f.float()).mean()), 4),
                                      "R_mean": round(float(((out_t - o_f).norm(dim=-1) / o_f.norm(dim=-1)).mean()), 5)}
                extras["randn_topk_by_coverage_16k"] = tk
            tab[str(n_t)] = {"coverage": round(float(stt.n_sel.float().mean()) / wt.pages_per_seq, 4),
                             "delta_mean": round(float((1.0 - km_t).mean()), 5),
                             "rho_mean": round(float((ks_t.float() / s_f.float()).mean()), 4),
                             "R_mean": round(float(((stt.out - o_f).norm(dim=-1) / o_f.norm(dim=-1)).mean()), 5),
                             "tau_hat_minus_tau_mean": round(float((stt.tau_hat - t_f).mean()), 4)}
            del stt, it
        extras["randn_gauss_selector_by_context"] = {"q_page": args.q_page, "margin": 0.0, "rows": tab}
        # the Gaussian-aware selector alone on page moments that are NOT homogeneous (what attention sinks or a few
        # relevant pages produce): a few pages far above the bulk are caught by the start of the root iteration
        # (hottest page of every wavefront) and structure along the sequence by the per-slice mixture the start is
        # taken from, so the fixed launches still converge; of two populations interleaved at random a rare head needs
        # one more evaluation, done by its gathering workgroup alone
        gsel = {}
        gm = torch.Generator().manual_seed(17)
        base_mu = torch.randn(B, Hq, M, generator=gm)
        one_sg = torch.ones(B, Hq, M)
        hot64 = base_mu.clone(); hot64[:, :, torch.randperm(M, generator=gm)[:64]] += 8.0
        hot4 = base_mu.clone(); hot4[:, :, torch.randperm(M, generator=gm)[:4]] += 6.0
        bimodal = torch.cat([torch.randn(B, Hq, M // 2, generator=gm), 3 + 0.5 * torch.randn(B, Hq, M - M // 2, generator=gm)], dim=-1)
        shuffled = bimodal[:, :, torch.randperm(M, generator=gm)].contiguous()
        trend = base_mu + torch.linspace(0, 4, M)
        for name, mu_t in (("homogeneous", base_mu), ("4_pages_plus_6_sigma", hot4), ("64_pages_plus_8_sigma", hot64),
                           ("bimodal", bimodal), ("bimodal_interleaved", shuffled),
                           ("trend_plus_4_sigma_along_the_sequence", trend)):
            mu_d, sg_d = mu_t.to(dev).contiguous(), one_sg.to(dev)
            gsel[name] = round(R.time_call(lambda st: ekv.ekv_select_gauss(st0.cfg, mu_d, sg_d, st0.inp["seq_lens"], args.q_page,
                                                                           0.0, st0.tau_hat, st0.page_idx, st0.n_sel,
                                                                           st0.overflow, st0.ws_gauss), reps=10), 2)
        extras["select_gauss_us_by_page_moment_shape"] = gsel
        # the top-k selector alone on score rows that are not stationary along the sequence (synthetic rows at the
        # headline's shape): the key range of the slice histograms is sampled from runs spread over the sequence, and
        # a slice crowded with top pages is scanned alone
        tsel = {}
        ramp = torch.linspace(0, 1, M, device=dev)
        base_s = torch.randn(B, Hq, M, generator=gm).to(dev) * 3 + 17
        shapes_t = {"stationary": base_s, "trend_plus_6_sigma_along_the_sequence": base_s + 18 * ramp,
                    "last_5_percent_plus_10_sigma": base_s + 30 * (ramp > 0.95),
                    "first_1024_pages_plus_10_sigma": base_s + 30 * (ramp < 1024 / M),
                    "16_distinct_values": torch.round(base_s).clamp(10, 25)}
        near = base_s.clone()                                    # 5000 pages within 1e-3 of each other, where the cut falls
        near[:, :, torch.randperm(M, generator=gm)[:5000].to(dev)] = (25.0 + 1e-3 * torch.rand(5000, generator=gm)).to(dev)
        shapes_t["5000_pages_within_1e-3_at_the_cut"] = near
        for name, box_t in shapes_t.items():
            box_t = box_t.contiguous()
            tsel[name] = round(R.back_to_back(lambda st: ekv.ekv_select_topk(st0.cfg, box_t, st0.inp["seq_lens"], k_pages,
                                                                             st0.page_idx, st0.n_sel, st0.ws_topk), reps=20), 2)
        extras["select_topk_us_by_score_shape"] = tsel
        # 8-bit page bounds (an extension; the rows above keep the paper's cache-dtype metadata): allocated and
        # built only now, so that nothing above pays for them
        for st in copies:
            st.enable_box8()
            ekv.ekv_stats_build(st.cfg, st.cache(), st.stats())
        torch.cuda.synchronize()
        us_8, stage_8, _ = R.run_timed(R.step_topk8, side, 5)
        us_g8, _, _ = R.run_timed(R.step_group8, side, 5, stages=False)
        score8_us = R.time_call(lambda st: ekv.ekv_score_pages(st.cfg, st.inp["q"], st.stats(), st.inp["seq_lens"],
                                                               ekv.EKV_SCORE_BOX8, st.box), reps=20)
        bytes8 = B * Hkv * M * 256 + B * Hq * M * 4
        ekv.ekv_score_pages(st0.cfg, st0.inp["q"], st0.stats(), st0.inp["seq_lens"], ekv.EKV_SCORE_BOX8, st0.box)
        ekv.ekv_select_topk(st0.cfg, st0.box, st0.inp["seq_lens"], k_pages, st0.page_idx, st0.n_sel, st0.ws_topk)
        ekv.ekv_decode_sparse(st0.cfg, st0.inp["q"], st0.cache(), st0.page_idx, st0.n_sel, st0.out, st0.tau,
                              st0.supp, st0.ws_sparse,
                              extras=ekv.decode_extras(tau_ref=tau_f, kept_mass_ref=kept_mass, kept_supp_ref=kept_supp))
        torch.cuda.synchronize()
        extras["box8"] = {
            "topk_step_us": round(us_8, 2),
            "topk_stage_us": {nm: round(float(v), 2) for nm, v in zip(STAGE_NAMES["topk"], stage_8.mean(axis=0))},
            "group_shared_step_us": round(us_g8, 2),
            "score_pages_us": round(score8_us, 2), "score_pages_algorithmic_bytes": bytes8,
            "score_pages_GBps": round(bytes8 / (score8_us * 1e-6) / 1e9, 1),
            "speedup_vs_dense": round(dense_us / us_8, 2),
            "delta_mean": round(float((1.0 - kept_mass).mean()), 6),
            "rho_mean": round(float((kept_supp.float() / supp_f.float()).mean()), 4),
            "R_mean": round(float(((st0.out - out_f).norm(dim=-1) / out_f.norm(dim=-1)).mean()), 6)}
        result["other_rows"] = extras

    # ---------------------------------------------------------------- CPU baseline: the oracle, as it stands
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(R.inp, w, k_pages, args.cpu_units)

    # ---------------------------------------------------------------- the 128K-token batch workload, same steps
    if not args.no_extras and args.workload == "C4":
        R.release()
        del R, copies, st0
        w3 = synth.WORKLOADS["C3"]
        R3 = Runner(w3, args.budget, args.copies, args.q_page, dev, args.cap_frac, fused_append=not args.two_launch_append)
        side = max(10, args.steps // 4)
        row = {"workload": f"{w3.name}: B{w3.batch} {w3.n_q_heads}q/{w3.n_kv_heads}kv ctx{w3.context} page{w3.page_size} "
                           f"{w3.kv_dtype}, top-k {R3.k_pages} pages ({args.budget:.0%})"}
        us3, stage3, _ = R3.run_timed(R3.step_topk, side, 5)
        row["topk_step_us"] = round(us3, 2)
        row["topk_stage_us"] = {nm: round(float(v), 2) for nm, v in zip(STAGE_NAMES["topk"], stage3.mean(axis=0))}
        us3r, _, _ = R3.run_timed(R3.step_group, side, 5, stages=False)
        row["group_shared_step_us"] = round(us3r, 2)
        us3d, _, _ = R3.run_timed(R3.step_dense, max(5, side // 2), 3, stages=False)
        row["dense_full_us"] = round(us3d, 2)
        d3 = w3.batch * w3.n_kv_heads * w3.context * 2 * w3.head_dim * 2
        row["dense_full_GBps"] = round((d3 / 2 + w3.batch * w3.n_q_heads * w3.context * 8) / (us3d * 1e-6) / 1e9, 1)
        row["speedup_topk_vs_dense"] = round(us3d / us3, 2)

        def quality(Rq, step_fn):
            """delta, rho, R of the selection of `step_fn` against the dense decode (GPU side outputs), copy 0."""
            s_ = Rq.copies[0]
            o_f, t_f, n_f = torch.zeros_like(s_.out), torch.zeros_like(s_.tau), torch.zeros_like(s_.supp)
            ekv.ekv_decode_full(s_.cfg, s_.inp["q"], s_.cache(), o_f, t_f, n_f, Rq.full_ws())
            step_fn(s_)
            km_, ks_ = torch.zeros_like(s_.tau), torch.zeros_like(s_.supp)
            ekv.ekv_decode_sparse(s_.cfg, s_.inp["q"], s_.cache(), s_.page_idx, s_.n_sel, s_.out, s_.tau, s_.supp,
                                  s_.ws_sparse, extras=ekv.decode_extras(tau_ref=t_f, kept_mass_ref=km_, kept_supp_ref=ks_))
            torch.cuda.synchronize()
            return {"pages_per_head_mean": float(s_.n_sel.float().mean()), "pages_per_head_max": int(s_.n_sel.max()),
                    "coverage": round(float(s_.n_sel.float().mean()) / Rq.w.pages_per_seq, 4),
                    "support_full_mean": float(n_f.float().mean()),
                    "delta_mean": round(float((1.0 - km_).mean()), 6),
                    "rho_mean": round(float((ks_.float() / n_f.float()).mean()), 4),
                    "R_mean": round(float(((s_.out - o_f).norm(dim=-1) / o_f.norm(dim=-1)).mean()), 6)}
        # this workload's planted support is clustered (8 spans of 8 tokens per head): selection quality, top-k 2 %
        row["topk_quality"] = quality(R3, R3.step_topk)
        R3.release()
        del R3
        # at 128K the adaptive selector keeps 5-16 % of the pages of this data: its lists get that room
        # (the list capacity also sizes the decode's launch grid, so the top-k rows above keep the small one)
        R3g = Runner(w3, args.budget, args.copies, args.q_page, dev, cap_frac=0.25,
                     fused_append=not args.two_launch_append)
        us3g, stage3g, _ = R3g.run_timed(R3g.step_gauss, side, 5)
        row["gauss_step_us"] = round(us3g, 2)
        row["gauss_stage_us"] = {nm: round(float(v), 2) for nm, v in zip(STAGE_NAMES["gauss"], stage3g.mean(axis=0))}
        row["gauss_selected_pages_mean"] = float(R3g.copies[0].n_sel.float().mean())
        row["gauss_overflow_heads"] = int(R3g.copies[0].overflow.sum())
        row["speedup_gauss_vs_dense"] = round(us3d / us3g, 2)
        row["gauss_quality"] = quality(R3g, R3g.step_gauss)
        result["other_rows"]["C3-128k"] = row
        R3g.release()
        del R3g
        # latency against context length (one sequence of the headline's shape), the form of the paper's decode-only
        # efficiency figure: dense entmax decode, top-k (2 %) and Gaussian-aware steps, softmax over the top-k lists
        sweep = {}
        for ctx in (32768, 131072, 524288):
            wn = synth.WORKLOADS["C4"].scaled(name=f"C4-shape-{ctx}", context=ctx)
            Rn = Runner(wn, args.budget, args.copies, args.q_page, dev, cap_frac=max(args.cap_frac, 0.75 if ctx <= 32768 else 0.25 if ctx <= 131072 else 0.08),
                        fused_append=not args.two_launch_append)
            u_t, _, _ = Rn.run_timed(Rn.step_topk, side, 5, stages=False)
            u_g, _, _ = Rn.run_timed(Rn.step_gauss, side, 5, stages=False)
            ovf_g = int(Rn.copies[0].overflow.sum())
            u_d, _, _ = Rn.run_timed(Rn.step_dense, max(5, side // 2), 3, stages=False)
            stn = Rn.copies[0]
            Rn.step_topk(stn)
            ws_smn = stn.workspace(ekv.EKV_OP_DECODE_SPARSE_SOFTMAX)
            lse_n = torch.zeros_like(stn.tau)
            u_s = Rn.time_call(lambda st_: ekv.ekv_decode_sparse_softmax(stn.cfg, stn.inp["q"], st_.cache(), stn.page_idx,
                                                                         stn.n_sel, stn.out, lse_n, ws_smn), reps=10)
            sweep[str(ctx)] = {"dense_full_us": round(u_d, 2), "topk_step_us": round(u_t, 2), "gauss_step_us": round(u_g, 2),
                               "gauss_overflow_heads": ovf_g, "softmax_over_topk_lists_us": round(u_s, 2),
                               "speedup_topk_vs_dense": round(u_d / u_t, 2)}
            Rn.release()
            del Rn, stn
        sweep["1048576"] = {"dense_full_us": result["other_rows"]["dense_full_us"], "topk_step_us": result["value"],
                            "gauss_step_us": result["other_rows"]["gauss_step_us"],
                            "softmax_over_topk_lists_us": result["other_rows"]["softmax_sparse_us"],
                            "speedup_topk_vs_dense": result["other_rows"]["speedup_vs_dense"]}
        result["other_rows"]["latency_by_context_B1"] = sweep
        # decode latency against the size of the support: one sequence of 262 144 tokens of the headline's shape with
        # the score scale lowered so that attention gets flatter (sparse: top-k 2 % = 5248 candidate tokens per head)
        by_support = {}
        for mult in (1.0, 0.25, 0.12, 0.06, 0.04):
            wf = synth.WORKLOADS["C4"].scaled(name=f"C4-shape-262144-scale-x{mult}", context=262144,
                                              scale=mult / math.sqrt(synth.WORKLOADS["C4"].head_dim))
            Rf = Runner(wf, args.budget, args.copies, args.q_page, dev, cap_frac=args.cap_frac,
                        fused_append=not args.two_launch_append)
            stf = Rf.copies[0]
            Rf.step_topk(stf)
            u_sp = Rf.time_call(lambda st_: ekv.ekv_decode_sparse(st_.cfg, st_.inp["q"], st_.cache(), stf.page_idx, stf.n_sel,
                                                                  st_.out, st_.tau, st_.supp, st_.ws_sparse), reps=10)
            supp_sp = float(stf.supp.float().mean())
            u_dn, _, _ = Rf.run_timed(Rf.step_dense, max(5, side // 2), 3, stages=False)
            by_support[f"scale_x{mult}"] = {"sparse_support_mean": supp_sp, "decode_sparse_us": round(u_sp, 2),
                                            "dense_support_mean": float(stf.supp.float().mean()),
                                            "dense_full_us": round(u_dn, 2)}
            Rf.release()
            del Rf, stf
        result["other_rows"]["decode_us_by_support_size_256k"] = by_support
        # the alpha and baseline sweep workload (batch 8, 256K tokens per sequence, pages of 32): top-k at a matched
        # budget of 4096 tokens per head under alpha = 1.25 / 1.5 / 2 against the dense decode of the same alpha, and
        # softmax over the same lists (its dropped mass next to entmax's)
        w5 = synth.WORKLOADS["C5"]
        k5 = 4096 // w5.page_size
        row5 = {"workload": f"{w5.name}: B{w5.batch} {w5.n_q_heads}q/{w5.n_kv_heads}kv ctx{w5.context} page{w5.page_size} "
                            f"{w5.kv_dtype}, top-k {k5} pages (4096 tokens) per query head", "by_alpha": {}}
        for al in (1.25, 1.5, 2.0):
            R5 = Runner(w5.scaled(alpha=al), k5 / w5.pages_per_seq, 2, args.q_page, dev, cap_frac=k5 / w5.pages_per_seq,
                        fused_append=not args.two_launch_append)
            assert R5.k_pages == k5
            u5, stage5, _ = R5.run_timed(R5.step_topk, side, 5)
            u5d, _, _ = R5.run_timed(R5.step_dense, max(5, side // 2), 3, stages=False)
            s5 = R5.copies[0]
            o5, t5, n5, lse5 = (torch.zeros_like(s5.out), torch.zeros_like(s5.tau), torch.zeros_like(s5.supp),
                                torch.zeros_like(s5.tau))
            ekv.ekv_decode_full(s5.cfg, s5.inp["q"], s5.cache(), o5, t5, n5, R5.ws_full, extras=ekv.decode_extras(lse=lse5))
            km5, ks5 = torch.zeros_like(s5.tau), torch.zeros_like(s5.supp)
            R5.step_topk(s5)
            ekv.ekv_decode_sparse(s5.cfg, s5.inp["q"], s5.cache(), s5.page_idx, s5.n_sel, s5.out, s5.tau, s5.supp,
                                  s5.ws_sparse, extras=ekv.decode_extras(tau_ref=t5, kept_mass_ref=km5, kept_supp_ref=ks5))
            torch.cuda.synchronize()
            row5["by_alpha"][str(al)] = {
                "topk_step_us": round(u5, 2),
                "topk_stage_us": {nm: round(float(v), 2) for nm, v in zip(STAGE_NAMES["topk"], stage5.mean(axis=0))},
                "dense_full_us": round(u5d, 2), "speedup_topk_vs_dense": round(u5d / u5, 2),
                "support_full_mean": float(n5.float().mean()),
                "delta_mean": round(float((1.0 - km5).mean()), 6),
                "rho_mean": round(float((ks5.float() / n5.float()).mean()), 4),
                "R_mean": round(float(((s5.out - o5).norm(dim=-1) / o5.norm(dim=-1)).mean()), 6)}
            if al == 2.0:                                          # softmax does not depend on alpha: once
                lse_s5, o_s5 = torch.zeros_like(s5.tau), torch.zeros_like(s5.out)
                ws_s5 = s5.workspace(ekv.EKV_OP_DECODE_SPARSE_SOFTMAX)
                row5["softmax_over_topk_lists_us"] = round(R5.time_call(
                    lambda st_: ekv.ekv_decode_sparse_softmax(s5.cfg, s5.inp["q"], st_.cache(), s5.page_idx, s5.n_sel,
                                                              o_s5, lse_s5, ws_s5), reps=10), 2)
                row5["softmax_delta_mean"] = round(float((1.0 - torch.exp(lse_s5 - lse5)).mean()), 6)
            R5.release()
            del R5, s5
        result["other_rows"]["C5-256k"] = row5
        # many short sequences (64 x 8K tokens: 2048 (sequence, head) rows of 11 selected pages): the rows take the
        # one-wavefront-per-row selection and solve kernels
        wm = synth.Workload("B64-8k", 64, 32, 8, 128, 8192, 16, "bf16", n_planted=16, n_outlier_channels=4)
        Rm = Runner(wm, args.budget, 2, args.q_page, dev, args.cap_frac, fused_append=not args.two_launch_append)
        um, stage_m, _ = Rm.run_timed(Rm.step_topk, side, 5)
        umd, _, _ = Rm.run_timed(Rm.step_dense, max(5, side // 2), 3, stages=False)
        result["other_rows"]["B64-8k"] = {
            "workload": f"{wm.batch} sequences x {wm.context} tokens, 32q/8kv, top-k {Rm.k_pages} pages",
            "topk_step_us": round(um, 2),
            "topk_stage_us": {nm: round(float(v), 2) for nm, v in zip(STAGE_NAMES["topk"], stage_m.mean(axis=0))},
            "dense_full_us": round(umd, 2), "speedup_topk_vs_dense": round(umd / um, 2)}
        Rm.release()
        del Rm

    print(json.dumps(result))


if __name__ == "__main__":
    main()
