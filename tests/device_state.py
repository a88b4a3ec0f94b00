"""Device buffers of one workload: everything the entry points read and write, plus the ekv_config.

Plumbing for the tests and the benchmark (torch allocates, the library computes); no part of the method."""
import torch

from paper_2605_21649_amd import binding as ekv
from paper_2605_21649_amd import synth


class DeviceState:
    """All device buffers of one workload plus its ekv_config."""

    def __init__(self, w, inp, cap=None, device="cuda"):
        self.w = w
        dev = torch.device(device)
        self.inp = {k: v.to(dev) for k, v in inp.items()}
        B, Hq, Hkv, d, P = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.page_size
        self.Mmax = w.pages_per_seq
        self.cap = cap if cap is not None else self.Mmax
        self.cfg = ekv.make_config(B, Hq, Hkv, d, P, w.kv_dtype, w.alpha, w.score_scale, self.Mmax, self.cap)
        dt = synth.torch_dtype(w.kv_dtype)
        self.box_stats = torch.zeros(B, Hkv, self.Mmax, 2, d, device=dev, dtype=dt)
        self.gauss_stats = torch.zeros(B, Hkv, self.Mmax, 2, d, device=dev, dtype=dt)
        f32 = dict(device=dev, dtype=torch.float32)
        i32 = dict(device=dev, dtype=torch.int32)
        self.box = torch.zeros(B, Hq, self.Mmax, **f32)
        self.mu = torch.zeros(B, Hq, self.Mmax, **f32)
        self.sigma = torch.zeros(B, Hq, self.Mmax, **f32)
        self.page_idx = torch.zeros(B, Hq, self.cap, **i32)
        self.n_sel = torch.zeros(B, Hq, **i32)
        self.overflow = torch.zeros(B, Hq, **i32)
        self.tau_hat = torch.zeros(B, Hq, **f32)
        self.out = torch.zeros(B, Hq, d, **f32)
        self.tau = torch.zeros(B, Hq, **f32)
        self.supp = torch.zeros(B, Hq, **i32)
        self.ws = {}

    def cache(self):
        i = self.inp
        return ekv.cache_view(i["k_pool"], i["v_pool"], i["block_table"], i["seq_lens"])

    def stats(self):
        return ekv.stats_view(self.box_stats, self.gauss_stats, getattr(self, "box8_stats", None))

    def enable_box8(self):
        """Allocate the optional 8-bit bounds; from then on build/append keep them up to date."""
        w = self.w
        self.box8_stats = torch.zeros(w.batch, w.n_kv_heads, self.Mmax, 16, 2, 8, device=self.box.device,
                                      dtype=torch.uint8)
        return self.box8_stats

    def workspace(self, op):
        if op not in self.ws:
            n = ekv.ekv_workspace_bytes(self.cfg, op)
            self.ws[op] = torch.empty(max(n, 256), device=self.box.device, dtype=torch.uint8)
        return self.ws[op]


class HeadSlice:
    """The KV heads [h0, h1) of a batch-1 DeviceState (and their query heads) as a problem of its own: a config
    with the pools' head stride, pool pointers advanced to h0, and contiguous slices of every per-head array.
    Independent slices can run on separate streams."""

    def __init__(self, st, h0, h1):
        w = st.w
        assert w.batch == 1, "per-head arrays of a head range are contiguous only for batch 1"
        G = w.group
        self.st, self.h0, self.h1 = st, h0, h1
        q0, q1 = h0 * G, h1 * G
        self.cfg = ekv.make_config(1, q1 - q0, h1 - h0, w.head_dim, w.page_size, w.kv_dtype, w.alpha, w.score_scale,
                                   st.Mmax, st.cap, pool_kv_heads=w.n_kv_heads)
        i = st.inp
        self.q = i["q"][:, q0:q1]
        self.seq_lens = i["seq_lens"]
        self.box_stats, self.gauss_stats = st.box_stats[:, h0:h1], st.gauss_stats[:, h0:h1]
        self.box8_stats = st.box8_stats[:, h0:h1] if hasattr(st, "box8_stats") else None
        for name in ("box", "mu", "sigma", "page_idx", "n_sel", "overflow", "tau_hat", "out", "tau", "supp"):
            setattr(self, name, getattr(st, name)[:, q0:q1])
        self.ws = {}

    def cache(self, seq_lens=None):
        i = self.st.inp
        return ekv.cache_view_heads(i["k_pool"], i["v_pool"], i["block_table"],
                                    self.seq_lens if seq_lens is None else seq_lens, self.h0)

    def stats(self):
        return ekv.stats_view(self.box_stats, self.gauss_stats, self.box8_stats)

    def new_token(self, k_new, v_new):
        """[1][Hkv][d] tokens of all heads -> this slice's."""
        return k_new[:, self.h0:self.h1], v_new[:, self.h0:self.h1]

    def workspace(self, op):
        if op not in self.ws:
            n = ekv.ekv_workspace_bytes(self.cfg, op)
            self.ws[op] = torch.empty(max(n, 256), device=self.box.device, dtype=torch.uint8)
        return self.ws[op]
