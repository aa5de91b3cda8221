"""Seeded synthetic Q/K/V for the eviction step.

These tensors stand in for the per-layer patch queries and cache+block keys /
values that an LLM forward would produce during block-wise prefill (paper
Sec. 2.2-2.3, Sec. 3.1 Stage 2, App. A.3).  Only shapes, budgets and episode
counts follow the paper; the values are random with the structure each workload
names.  This module is shared by the tests of the CPU oracle and of the HIP
path and therefore contains none of the method's arithmetic: no logits, no
softmax, no selection, no gather.

Layout (row-major, innermost d contiguous):
  Q [n_batch, Hq,  p, d]   patch queries, batch item = episode (optionally
                           layer-major folded: item = layer * E + episode)
  K [n_batch, Hkv, C, d]   context keys; rows [0, n_cached) kept cache,
  V [n_batch, Hkv, C, d]   rows [n_cached, n_cached + n_block) the new block
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    L: int          # layers
    Hq: int         # query heads
    Hkv: int        # KV heads (the paper's H)
    d: int          # head dim
    dtype: str      # "f32" | "bf16"
    M: int          # per-head cache budget
    B: int          # block size M_block
    E: int          # episodes
    p: int          # patched-prompt length
    recipe: str     # value distribution, see _fill()
    seed: int

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def N(self) -> int:
        return self.M + self.B

    @property
    def R(self) -> int:
        return self.G * self.p

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in [
        Workload("tiny", 1, 8, 2, 64, "f32", 256, 128, 1, 32, "normal", 0xE91C0001),
        Workload("llama32_3b", 28, 24, 8, 128, "bf16", 2048, 2048, 4, 64,
                 "outlier_channels", 0xE91C0002),
        Workload("llama31_8b", 32, 32, 8, 128, "bf16", 4096, 4096, 4, 128,
                 "normal", 0xE91C0003),
        Workload("qwen25_7b", 28, 28, 4, 128, "bf16", 8192, 2048, 8, 64,
                 "topic_clusters", 0xE91C0004),
        Workload("stress", 32, 32, 8, 128, "bf16", 16384, 8192, 16, 256,
                 "student_t", 0xE91C0005),
    ]
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed & 0x7FFFFFFFFFFFFFFF)
    return g


def _mix(*parts: int) -> int:
    """Deterministic 63-bit mix of integer stream identifiers (splitmix64 steps)."""
    x = 0x9E3779B97F4A7C15
    for p in parts:
        x = (x ^ (p & 0xFFFFFFFFFFFFFFFF)) & 0xFFFFFFFFFFFFFFFF
        x = (x + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
        x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        x = x ^ (x >> 31)
    return x & 0x7FFFFFFFFFFFFFFF


def make_layer(w: Workload, layer: int = 0, step: int = 0, device="cpu",
               n_ctx: Optional[int] = None, capacity: Optional[int] = None):
    """Q, K, V of one layer for all E episodes (fp32 values, then cast to w.dtype).

    n_ctx   : number of valid context rows (default M + B)
    capacity: C >= n_ctx, rows of the K/V buffers (default n_ctx); rows beyond
              n_ctx are filled with random values too, so that a kernel reading
              them by mistake changes the result.
    """
    N = w.N if n_ctx is None else n_ctx
    C = N if capacity is None else capacity
    assert C >= N
    dev = torch.device(device)
    g = _gen(_mix(w.seed, layer, step), dev)
    E, Hq, Hkv, p, d = w.E, w.Hq, w.Hkv, w.p, w.d
    f32 = torch.float32

    def randn(*shape):
        return torch.randn(*shape, generator=g, device=dev, dtype=f32)

    q = randn(E, Hq, p, d)
    k = randn(E, Hkv, C, d)
    v = randn(E, Hkv, C, d)

    if w.recipe == "normal":
        pass
    elif w.recipe == "outlier_channels":
        # 4 channels per KV head (same for all tokens and episodes) carry 8x magnitude.
        for h in range(Hkv):
            ch = torch.randperm(d, generator=g, device=dev)[:4]
            k[:, h, :, ch] *= 8.0
            v[:, h, :, ch] *= 8.0
    elif w.recipe == "topic_clusters":
        # keys = topic mean + noise over contiguous runs; episode e's queries lean to topic e
        n_topics = 8
        mu = 0.5 * randn(n_topics, d)
        run_len = torch.randint(64, 513, (C // 64 + 2,), generator=g, device=dev)
        run_topic = torch.randint(0, n_topics, (C // 64 + 2,), generator=g, device=dev)
        topic_of_row = torch.repeat_interleave(run_topic, run_len)[:C]
        k += mu[topic_of_row].view(1, 1, C, d)
        q += mu[torch.arange(E, device=dev) % n_topics].view(E, 1, 1, d)
    elif w.recipe == "student_t":
        # K element ~ Student-t(nu=3) = z / sqrt(chi2_3 / 3)
        chi2 = randn(E, Hkv, C, d).square_()
        chi2 += randn(E, Hkv, C, d).square_()
        chi2 += randn(E, Hkv, C, d).square_()
        k /= (chi2 / 3.0).sqrt_()
        del chi2
    else:
        raise ValueError(w.recipe)
    dt = w.torch_dtype
    return q.to(dt).contiguous(), k.to(dt).contiguous(), v.to(dt).contiguous()


def make_folded(w: Workload, layers, step: int = 0, device="cpu"):
    """Layers folded into the batch axis, layer-major: item = layer_pos * E + episode."""
    qs, ks, vs = [], [], []
    for layer in layers:
        q, k, v = make_layer(w, layer, step, device)
        qs.append(q), ks.append(k), vs.append(v)
    return torch.cat(qs), torch.cat(ks), torch.cat(vs)


def to_f64_numpy(t: torch.Tensor):
    """Exact widening of an fp32/bf16 tensor to a float64 numpy array (host)."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def raw_bits_numpy(t: torch.Tensor):
    """Bit pattern of a tensor as an unsigned integer numpy array (host)."""
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy().view("uint32")
    raise TypeError(t.dtype)
