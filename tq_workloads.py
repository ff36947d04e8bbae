"""Seeded synthetic inputs shared by the HIP path's tests/bench and by the CPU oracle.

This module only *draws numbers*: it contains none of the method's arithmetic (no
quantisation, no attention).  Both sides receive the same fp16 bits.

The workloads stand in for the paper's Llama-3.1-70B and Gemma-4 attention shapes
(kernel benchmark, Table 2; kernel configuration, Table 7 / Appendix A): the paper's
own kernel benchmark is shape-only, and neither weights nor activations exist here.

  tiny      B1, 8 query heads, 1 KV head (GQA 8), d=128, S=1024,  alpha=1/sqrt(128); q,K,V ~ N(0,1)
  llama8k   B1, 64/8 heads, d=128, S=8192,   alpha=1/sqrt(128); N(0,1), 4 fixed K channels per
            KV head scaled x8 (outlier channels; indices = first 4 of a seeded permutation)
  llama128k as llama8k with S=131072 (the headline shape)
  gemma32k  B1, 32/16 heads, d=256, S=32768, alpha=1.0; q,K ~ N(0,0.1^2), V ~ N(0,1)
  global512_32k  B1, 32 query heads on 1 KV head (GQA 32), d=512, S=32768, alpha=1.0; values as gemma32k
            (the global-attention column of the kernel configuration table, Appendix A)
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    attn_scale: float
    seed: int
    qk_std: float = 1.0
    v_std: float = 1.0
    outlier_channels: int = 0      # number of K channels per KV head scaled up
    outlier_gain: float = 8.0

    @property
    def gqa(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def packed_bytes(self) -> int:
        """Bytes of int4 codes + fp16 scales + fp16 zero-points, K and V, for seq_len tokens."""
        d = self.head_dim
        per_tok = 2 * (d // 2 + 2 * 2 * (d // 32))
        return self.batch * self.n_kv_heads * self.seq_len * per_tok


WORKLOADS = {
    "tiny": Workload("tiny", 1, 8, 1, 128, 1024, 1.0 / math.sqrt(128), 1001),
    "llama8k": Workload("llama8k", 1, 64, 8, 128, 8192, 1.0 / math.sqrt(128), 1002,
                        outlier_channels=4),
    "llama128k": Workload("llama128k", 1, 64, 8, 128, 131072, 1.0 / math.sqrt(128), 1003,
                          outlier_channels=4),
    "gqa16_128k": Workload("gqa16_128k", 1, 128, 8, 128, 131072, 1.0 / math.sqrt(128), 1007,
                           outlier_channels=4),
    "gemma32k": Workload("gemma32k", 1, 32, 16, 256, 32768, 1.0, 1004, qk_std=0.1),
    "global512_32k": Workload("global512_32k", 1, 32, 1, 512, 32768, 1.0, 1006, qk_std=0.1),
}


def layer_workload(layer: int, batch_index: int, seq_len: int = 131072) -> Workload:
    """One (layer, batch element) of the 80-layer x batch-4 sweep: the llama128k shape with
    its own seed 1005 + 1000*layer + batch_index."""
    return replace(WORKLOADS["llama128k"], name=f"llama128k_L{layer}_b{batch_index}",
                   seq_len=seq_len, seed=1005 + 1000 * layer + batch_index)


def custom(name="custom", batch=1, n_q_heads=8, n_kv_heads=1, head_dim=128, seq_len=256,
           attn_scale=None, seed=7, **kw) -> Workload:
    if attn_scale is None:
        attn_scale = 1.0 / math.sqrt(head_dim)
    return Workload(name, batch, n_q_heads, n_kv_heads, head_dim, seq_len, attn_scale, seed, **kw)


def _randn(shape, gen, device, std):
    x = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    return x


def make_inputs(w: Workload, device="cpu"):
    """Returns (q, k, v) as fp16 tensors: q [B,H_q,d], k and v [B,H_kv,S,d].

    The draw order is fixed (q, k, v, then the outlier permutation per KV head) so that a
    seed names one set of bits per device type.  CPU and GPU generators differ; a caller
    that wants both sides to see the same bits draws once and copies.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    q = _randn((w.batch, w.n_q_heads, w.head_dim), gen, dev, w.qk_std)
    k = _randn((w.batch, w.n_kv_heads, w.seq_len, w.head_dim), gen, dev, w.qk_std)
    if w.outlier_channels:
        pg = torch.Generator(device="cpu")
        pg.manual_seed(w.seed + 17)
        for h in range(w.n_kv_heads):
            idx = torch.randperm(w.head_dim, generator=pg)[: w.outlier_channels].to(dev)
            k[:, h, :, idx] *= w.outlier_gain
    k = k.to(torch.float16)
    v = _randn((w.batch, w.n_kv_heads, w.seq_len, w.head_dim), gen, dev, w.v_std).to(torch.float16)
    return q.to(torch.float16), k, v


def make_queries(w: Workload, n_queries: int, device="cpu"):
    """Queries for the sequence's last n_queries tokens, fp16 [B, n_queries, H_q, d]: the last one is the
    workload's own query (the first draw of make_inputs), the earlier ones are drawn alike from seeds of
    their own."""
    dev = torch.device(device)
    rows = []
    for t in range(n_queries):
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed if t == n_queries - 1 else w.seed * 7919 + 500 + t)
        rows.append(_randn((w.batch, w.n_q_heads, w.head_dim), gen, dev, w.qk_std).to(torch.float16))
    return torch.stack(rows, dim=1).contiguous()


def make_new_token(w: Workload, step: int = 0, device="cpu"):
    """One appended token per sequence: (k_new, v_new) fp16 [B,H_kv,1,d], seeded from the
    workload seed and the step number."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed * 7919 + step + 1)
    shape = (w.batch, w.n_kv_heads, 1, w.head_dim)
    k = _randn(shape, gen, dev, w.qk_std).to(torch.float16)
    v = _randn(shape, gen, dev, w.v_std).to(torch.float16)
    return k, v
