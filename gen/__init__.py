"""Seeded synthetic inputs for the RefreshKV decode-attention path.

This module only draws random tensors and lays them out; it holds none of the
method's arithmetic (no softmax, no selection, no similarity).  The CPU oracle
and the HIP path are both fed from here, so that they see the same bits.

The paper evaluates on real-text KV caches of Llama-3.1-8B and Qwen2-7B
(Section 3, "Models and Evaluation tasks"; Appendix Table "Dataset
statistics"): 10K-128K input tokens, batch 1.  Neither the weights nor the
datasets are available, so the workloads below keep the paper's geometry
(heads, head_dim, context lengths, K = L/16 .. L/8, strides 4-16) and draw the
values from stated distributions.

Everything is generated in fp32 from a ``torch.Generator`` whose seed is a pure
function of (base seed, workload id, layer, stream tag) and then rounded to
bf16 (round-to-nearest-even, torch's conversion).  A tensor may be generated on
the CPU or on the GPU; the two devices use different random streams, so a test
generates once and hands the same tensor to both sides.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np
import torch

BASE_SEED = 20241105

_TAG = {"k": 1, "v": 2, "q": 3, "newk": 4, "newv": 5, "plant": 6, "lens": 7,
        "topic": 8, "centroid": 9, "assign": 10, "weights": 11}


@dataclass(frozen=True)
class Workload:
    """One synthetic decode workload (geometry + schedule + value recipe)."""
    name: str
    wid: int                      # workload id, part of every seed
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int                  # L (max over the batch when ragged)
    k_small: int                  # K, size of the small cache
    stride: int                   # S: fixed stride, or QC stride when dynamic
    n_steps: int                  # decode steps after the t=0 initialisation
    dynamic: bool = False         # True: query-similarity trigger every S steps
    threshold: float = 0.0        # s of the trigger (dynamic only)
    pool_w: int = 7               # max-pool width used at selection
    kv_recipe: str = "normal"     # normal | planted | zipf | clustered
    q_recipe: str = "iid"         # iid | ar1 | topic_ar1
    q_rho: float = 0.95           # AR(1) coefficient
    q_sigma: float = 0.31         # AR(1) innovation scale
    ragged: Optional[Tuple[int, int]] = None   # (lo, hi) of Uniform context lengths
    extra: Dict[str, float] = field(default_factory=dict)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def capacity(self) -> int:
        """Rows allocated per (sequence, KV head): context + decode steps, padded."""
        need = self.context + self.n_steps + 1
        return (need + 63) // 64 * 64

    @property
    def scale(self) -> float:
        """Softmax scale 1/sqrt(head_dim), rounded once to fp32 for both sides."""
        return float(np.float32(1.0 / math.sqrt(self.head_dim)))

    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_kv_heads * self.head_dim * 2


LLAMA = dict(n_q_heads=32, n_kv_heads=8, head_dim=128)
QWEN = dict(n_q_heads=28, n_kv_heads=4, head_dim=128)

WORKLOADS: Dict[str, Workload] = {
    # Small correctness case: the oracle runs every step in seconds.
    "cfg1_llama_2k": Workload(
        name="cfg1_llama_2k", wid=1, n_layers=1, batch=1, **LLAMA, context=2048,
        k_small=256, stride=4, n_steps=32, kv_recipe="planted", q_recipe="iid",
        extra={"n_planted": 16, "plant_gain": 4.0}),
    # Headline case: the metric is quoted on this one.
    "cfg2_llama_32k": Workload(
        name="cfg2_llama_32k", wid=2, n_layers=32, batch=1, **LLAMA, context=32768,
        k_small=2048, stride=10, n_steps=200, kv_recipe="normal", q_recipe="ar1",
        q_rho=0.95, q_sigma=0.31),
    "cfg3_qwen_64k_dynamic": Workload(
        name="cfg3_qwen_64k_dynamic", wid=3, n_layers=28, batch=1, **QWEN, context=65536,
        k_small=4096, stride=5, n_steps=200, dynamic=True, threshold=0.9,
        kv_recipe="zipf", q_recipe="topic_ar1", q_rho=0.97, q_sigma=0.243,   # trigger fires every 10-15 steps
        extra={"n_affine": 512, "beta": 1.0, "topic_gain": 0.5}),
    "cfg4_llama_batch16_ragged": Workload(
        name="cfg4_llama_batch16_ragged", wid=4, n_layers=4, batch=16, **LLAMA,
        context=16384, k_small=1024, stride=8, n_steps=64, kv_recipe="normal",
        q_recipe="iid", ragged=(4096, 16384)),
    "cfg5_llama_128k": Workload(
        name="cfg5_llama_128k", wid=5, n_layers=32, batch=1, **LLAMA, context=131072,
        k_small=8192, stride=16, n_steps=100, kv_recipe="clustered", q_recipe="ar1",
        q_rho=0.95, q_sigma=0.31, extra={"n_centroids": 64, "cluster_sigma": 0.1}),
}


def shrink(w: Workload, **changes) -> Workload:
    """A smaller variant of a workload (tests use this to keep the recipe but cut sizes)."""
    return replace(w, **changes)


def _generator(w: Workload, layer: int, tag: str, device) -> torch.Generator:
    seed = (BASE_SEED * 1_000_003 + w.wid * 100_003 + layer * 1_009 + _TAG[tag]) % (2 ** 63 - 1)
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def seq_lens(w: Workload) -> torch.Tensor:
    """Initial context length of every sequence, int32 [B] on the CPU."""
    if w.ragged is None:
        return torch.full((w.batch,), w.context, dtype=torch.int32)
    lo, hi = w.ragged
    g = _generator(w, 0, "lens", "cpu")
    return torch.randint(lo, hi + 1, (w.batch,), generator=g, dtype=torch.int32)


def make_kv(w: Workload, layer: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """K and V of one layer, bf16 [B, Hkv, capacity, D]; rows >= context are zero."""
    B, H, C, D, L = w.batch, w.n_kv_heads, w.capacity, w.head_dim, w.context
    dev = torch.device(device)
    K = torch.zeros(B, H, C, D, dtype=torch.bfloat16, device=dev)
    V = torch.zeros(B, H, C, D, dtype=torch.bfloat16, device=dev)
    gk = _generator(w, layer, "k", dev)
    gv = _generator(w, layer, "v", dev)
    for b in range(B):                      # one sequence at a time bounds the fp32 scratch
        kb = torch.randn(H, L, D, generator=gk, device=dev, dtype=torch.float32)
        vb = torch.randn(H, L, D, generator=gv, device=dev, dtype=torch.float32)
        if w.kv_recipe == "planted":
            gp = _generator(w, layer * 4096 + b, "plant", "cpu")
            n = int(w.extra["n_planted"])
            for h in range(H):
                pos = torch.randperm(L, generator=gp)[:n].to(dev)
                kb[h, pos] *= float(w.extra["plant_gain"])
        elif w.kv_recipe == "zipf":
            gp = _generator(w, layer * 4096 + b, "plant", "cpu")
            gt = _generator(w, layer, "topic", "cpu")
            topic = torch.randn(H, D, generator=gt).to(dev)
            n = int(w.extra["n_affine"])
            rank = torch.arange(1, n + 1, dtype=torch.float32, device=dev)
            for h in range(H):
                pos = torch.randperm(L, generator=gp)[:n].to(dev)
                kb[h, pos] += float(w.extra["beta"]) * (1.0 / rank)[:, None] * topic[h][None, :]
        elif w.kv_recipe == "clustered":
            gc = _generator(w, layer, "centroid", "cpu")
            ga = _generator(w, layer * 4096 + b, "assign", "cpu")
            nc = int(w.extra["n_centroids"])
            cent = torch.randn(H, nc, D, generator=gc).to(dev)
            for h in range(H):
                clustered = (torch.rand(L, generator=ga) < 0.5).to(dev)
                which = torch.randint(0, nc, (L,), generator=ga).to(dev)
                near = cent[h][which] + float(w.extra["cluster_sigma"]) * kb[h]
                kb[h] = torch.where(clustered[:, None], near, kb[h])
        elif w.kv_recipe != "normal":
            raise ValueError(w.kv_recipe)
        K[b, :, :L] = kb.to(torch.bfloat16)
        V[b, :, :L] = vb.to(torch.bfloat16)
        del kb, vb
    return K, V


def make_new_rows(w: Workload, layer: int, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """The (k, v) row each decode step appends: bf16 [n_steps, B, Hkv, D], ~N(0,1)."""
    dev = torch.device(device)
    shape = (w.n_steps, w.batch, w.n_kv_heads, w.head_dim)
    nk = torch.randn(shape, generator=_generator(w, layer, "newk", "cpu"))
    nv = torch.randn(shape, generator=_generator(w, layer, "newv", "cpu"))
    return nk.to(torch.bfloat16).to(dev), nv.to(torch.bfloat16).to(dev)


def make_queries(w: Workload, layer: int, device="cpu") -> torch.Tensor:
    """Queries for t = 0..n_steps: bf16 [n_steps + 1, B, Hq, D].

    iid: every step ~N(0,1).  ar1: q_t = rho q_{t-1} + sigma eps, q_0 ~ N(0,1).
    topic_ar1: topic_gain * topic[kv head of h] + an AR(1) part as above.
    """
    T, B, Hq, D = w.n_steps + 1, w.batch, w.n_q_heads, w.head_dim
    g = _generator(w, layer, "q", "cpu")
    eps = torch.randn(T, B, Hq, D, generator=g)
    if w.q_recipe == "iid":
        q = eps
    elif w.q_recipe in ("ar1", "topic_ar1"):
        q = torch.empty_like(eps)
        q[0] = eps[0]
        for t in range(1, T):
            q[t] = w.q_rho * q[t - 1] + w.q_sigma * eps[t]
        if w.q_recipe == "topic_ar1":
            gt = _generator(w, layer, "topic", "cpu")
            topic = torch.randn(w.n_kv_heads, D, generator=gt)
            per_head = topic.repeat_interleave(w.group, dim=0)          # [Hq, D]
            q = q + float(w.extra["topic_gain"]) * per_head[None, None]
    else:
        raise ValueError(w.q_recipe)
    return q.to(torch.bfloat16).to(torch.device(device))


def make_weights(batch: int, n_q_heads: int, length: int, seed: int, kind: str = "lognormal",
                 device="cpu") -> torch.Tensor:
    """Stand-alone fp32 'attention weights' [B, Hq, length] for selection tests.

    lognormal: exp(N(0,1)) normalised per row by its sum (shape of real softmax rows).
    ties: values drawn from 8 distinct levels, so equal scores are the norm.
    plateaus: about 50 stretches of one value each (runs of equal pooled scores far longer than the window).
    narrow: all values within one part in a thousand of 0.5 (one bin of any coarse histogram).
    spiky: one position in a hundred carries a value of order 1, the rest of order 1e-6.
    zeros: all zero (every position ties with every other).
    """
    g = torch.Generator(device="cpu")
    g.manual_seed((BASE_SEED + 7919 * seed) % (2 ** 63 - 1))
    if kind == "lognormal":
        x = torch.randn(batch, n_q_heads, length, generator=g, dtype=torch.float64).exp()
        x = x / x.sum(dim=-1, keepdim=True)
    elif kind == "ties":
        x = torch.randint(0, 8, (batch, n_q_heads, length), generator=g).to(torch.float64) / 8.0
    elif kind == "plateaus":
        seg = max(length // 50, 1)
        x = torch.rand(batch, n_q_heads, (length + seg - 1) // seg, generator=g, dtype=torch.float64)
        x = x.repeat_interleave(seg, dim=-1)[..., :length]
    elif kind == "narrow":
        x = 0.5 + torch.rand(batch, n_q_heads, length, generator=g, dtype=torch.float64) * 1e-3
    elif kind == "spiky":
        x = torch.rand(batch, n_q_heads, length, generator=g, dtype=torch.float64) * 1e-6
        where = torch.randint(0, length, (batch, n_q_heads, max(length // 100, 1)), generator=g)
        x.scatter_(-1, where, torch.rand(where.shape, generator=g, dtype=torch.float64))
    elif kind == "zeros":
        x = torch.zeros(batch, n_q_heads, length, dtype=torch.float64)
    else:
        raise ValueError(kind)
    return x.to(torch.float32).to(torch.device(device))


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """A bf16 tensor as a numpy uint16 array of its bit patterns (CPU copy)."""
    return t.detach().to("cpu").contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_bf16(a: np.ndarray, device="cpu") -> torch.Tensor:
    """Inverse of :func:`bf16_bits`."""
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16)
    return t.to(torch.device(device))
