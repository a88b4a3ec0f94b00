"""Seeded synthetic paged KV caches shaped like the paper's decode benchmarks.

Input generation only: nothing here computes any part of the method (no page
statistics, scores, selections or attention).  Both the HIP path and the CPU oracle
are fed from these tensors.

The paper's efficiency and approximation benchmarks draw q, K, V from a standard
normal (App. E.1).  The workload table of this repository adds, on top of that:
per-channel key offsets (a few channels with a large mean, as in real LLM keys) and
"planted" tokens whose keys are aligned with the query so that the entmax support
is non-trivial.  Tensors are produced with a torch.Generator on the requested device;
a (seed, device type) pair always gives the same tensors.
"""
from dataclasses import dataclass, field, replace
import math
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int                 # tokens per sequence (before `ragged` is subtracted)
    page_size: int
    kv_dtype: str                # 'f32' or 'bf16'
    alpha: float = 1.5
    scale: float = 0.0           # 0 -> 1/sqrt(head_dim)
    n_planted: int = 0           # planted q-aligned tokens per query head
    planted_spans: int = 0       # 0: scattered; >0: that many contiguous spans per head
    n_outlier_channels: int = 0  # channels whose keys get +outlier_mean
    outlier_mean: float = 5.0
    planted_gain: float = 3.0
    planted_noise: float = 0.3
    ragged: int = 0              # seq_len = context - ragged (last page partial)
    permute_pages: bool = True   # block table = seeded random permutation of physical pages

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    @property
    def pages_per_seq(self):
        return -(-self.context // self.page_size)

    @property
    def score_scale(self):
        return self.scale if self.scale > 0 else 1.0 / math.sqrt(self.head_dim)

    def scaled(self, **kw):
        return replace(self, **kw)


# The five workloads of the repository's benchmark table (shapes and data recipes).
C1 = Workload("C1-tiny-fp32", 1, 8, 8, 128, 4096, 16, "f32", scale=4.0 / math.sqrt(128.0),
              n_planted=32, permute_pages=True)
C2 = Workload("C2-llama8b-32k", 1, 32, 8, 128, 32768, 16, "bf16", n_planted=64, n_outlier_channels=4)
C3 = Workload("C3-batch4-128k", 4, 32, 8, 128, 131072, 16, "bf16", n_planted=64, planted_spans=8,
              n_outlier_channels=4)
C4 = Workload("C4-1M", 1, 32, 8, 128, 1048576, 16, "bf16", n_planted=64, n_outlier_channels=4)
C5 = Workload("C5-batch8-256k-p32", 8, 32, 8, 128, 262144, 32, "bf16", n_planted=64, n_outlier_channels=4)
WORKLOADS = {w.name.split("-")[0]: w for w in (C1, C2, C3, C4, C5)}


def torch_dtype(kv_dtype):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[kv_dtype]


def make_inputs(w: Workload, seed: int, device="cpu"):
    """Build q, the paged K/V pools, the block table and sequence lengths.

    Returns a dict of torch tensors on `device`:
      q            [B, H_q, d]                 cache dtype
      k_pool,v_pool[n_phys, H_kv, P, d]        cache dtype (n_phys = B * pages_per_seq)
      block_table  [B, pages_per_seq] int32    logical page -> physical page
      seq_lens     [B] int32
      planted      [B, H_q, n_planted] int64   logical token positions of planted keys
    Values are rounded to the cache dtype before anybody sees them.  Slots of the last
    page past seq_len hold ordinary random values (they must be masked by consumers)."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    B, Hq, Hkv, d, n, P = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.context, w.page_size
    G = w.group
    M = w.pages_per_seq
    n_pad = M * P
    dt = torch_dtype(w.kv_dtype)

    q = torch.randn(B, Hq, d, generator=g, device=dev, dtype=torch.float32)
    # logical layout [B, Hkv, n_pad, d], generated per (b) to bound peak memory
    n_phys = B * M
    k_pool = torch.empty(n_phys, Hkv, P, d, device=dev, dtype=dt)
    v_pool = torch.empty(n_phys, Hkv, P, d, device=dev, dtype=dt)
    if w.permute_pages:
        perm = torch.randperm(n_phys, generator=g, device=dev)
    else:
        perm = torch.arange(n_phys, device=dev)
    block_table = perm.view(B, M).to(torch.int32)
    seq_len = n - w.ragged
    planted = torch.zeros(B, Hq, max(w.n_planted, 1), dtype=torch.int64, device=dev)

    offs = torch.zeros(d, device=dev, dtype=torch.float32)
    if w.n_outlier_channels:
        ch = torch.randperm(d, generator=g, device=dev)[: w.n_outlier_channels]
        offs[ch] = w.outlier_mean

    for b in range(B):
        for h in range(Hkv):
            k = torch.randn(n_pad, d, generator=g, device=dev, dtype=torch.float32) + offs
            v = torch.randn(n_pad, d, generator=g, device=dev, dtype=torch.float32)
            if w.n_planted:
                # disjoint positions for the G query heads that share this KV head
                if w.planted_spans:
                    span = w.n_planted // w.planted_spans
                    n_slots = seq_len // span
                    slots = torch.randperm(n_slots, generator=g, device=dev)[: G * w.planted_spans]
                    pos = (slots[:, None] * span + torch.arange(span, device=dev)[None, :]).view(G, -1)
                else:
                    pos = torch.randperm(seq_len, generator=g, device=dev)[: G * w.n_planted].view(G, -1)
                for gi in range(G):
                    hq = h * G + gi
                    qv = q[b, hq]
                    noise = torch.randn(w.n_planted, d, generator=g, device=dev, dtype=torch.float32)
                    k[pos[gi]] = w.planted_gain * qv / qv.norm() + w.planted_noise * noise + offs
                    planted[b, hq, : w.n_planted] = pos[gi]
            rows = block_table[b].long()
            k_pool[rows, h] = k.view(M, P, d).to(dt)
            v_pool[rows, h] = v.view(M, P, d).to(dt)
            del k, v
    return {
        "q": q.to(dt),
        "k_pool": k_pool,
        "v_pool": v_pool,
        "block_table": block_table.contiguous(),
        "seq_lens": torch.full((B,), seq_len, dtype=torch.int32, device=dev),
        "planted": planted,
    }


def logical_kv(inp, w: Workload, b: int, h_kv: int):
    """Valid keys and values of sequence b, KV head h_kv in logical token order: [n_b, d] each
    (cache dtype, on the tensors' device).  A gather through the block table; no arithmetic."""
    rows = inp["block_table"][b].long()
    n_b = int(inp["seq_lens"][b])
    d = w.head_dim
    k = inp["k_pool"][rows, h_kv].reshape(-1, d)[:n_b]
    v = inp["v_pool"][rows, h_kv].reshape(-1, d)[:n_b]
    return k, v
