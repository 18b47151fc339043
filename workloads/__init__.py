"""Seeded synthetic inputs for the MoE expert-layer hot path.

This module only *draws inputs*: replayed routing (top-k expert ids and gates per
token), activations, expert weights and upstream gradients.  It holds none of the
method's arithmetic (no histogram, no plan, no permutation, no FFN), so the CPU
oracle and the HIP path can both be fed from it without sharing code.

Routing stands in for the RL routing traces the paper measures on (Section 2.2,
Table 1): a Zipf-biased router whose hot experts move between micro-batches
(Section 2.2, "load imbalance characterization").  Ids are *replayed* inputs
(Section 2.3): nothing downstream recomputes them from logits.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    """One MoE-layer workload; names follow the paper's notation (Table 2, Section 5.1)."""

    name: str
    index: int            # position in the list of configs (seed namespace)
    E: int                # experts in the layer
    k: int                # top-k
    h: int                # hidden size (d_model)
    hff: int              # expert intermediate size h' (d_ff)
    T: int                # tokens per micro-batch
    n_mb: int             # micro-batches per training batch
    EP: int               # simulated expert-parallel degree
    r: int                # replica slots per rank
    zipf_s: float         # Zipf exponent of the router bias
    routing: str          # "single" | "domains4" | "fresh" | "stress"
    ranks_per_node: int = field(default=0)

    @property
    def M(self) -> int:
        return self.E // self.EP

    @property
    def G(self) -> int:
        return self.EP * (self.M + self.r)

    @property
    def N(self) -> int:
        return self.T * self.k

    @property
    def rpn(self) -> int:
        return self.ranks_per_node if self.ranks_per_node > 0 else min(self.EP, 8)

    @property
    def flops_per_mb(self) -> float:
        # 6 h h' per routed row forward (Eq. 4), twice that backward (dgrad + wgrad).
        return 18.0 * self.h * self.hff * self.N


CONFIGS = [
    Config("tiny", 0, E=8, k=2, h=128, hff=256, T=512, n_mb=1, EP=4, r=1,
           zipf_s=1.2, routing="single"),
    Config("qwen3-30b-a3b", 1, E=128, k=8, h=2048, hff=768, T=8192, n_mb=16, EP=8, r=2,
           zipf_s=1.0, routing="domains4"),
    Config("mixtral-8x7b", 2, E=8, k=2, h=4096, hff=14336, T=4096, n_mb=8, EP=8, r=1,
           zipf_s=1.5, routing="fresh"),
    Config("deepseek-v3", 3, E=256, k=8, h=7168, hff=2048, T=4096, n_mb=8, EP=32, r=2,
           zipf_s=1.2, routing="domains4"),
    Config("qwen3-235b-a22b-stress", 4, E=128, k=8, h=4096, hff=1536, T=16384, n_mb=32,
           EP=16, r=2, zipf_s=1.5, routing="stress"),
]


def small_config(name="small", **kw) -> Config:
    """A free-form config for tests (defaults: a ragged mid-size layer)."""
    base = dict(index=99, E=16, k=4, h=256, hff=192, T=777, n_mb=3, EP=4, r=2,
                zipf_s=1.2, routing="domains4")
    base.update(kw)
    return Config(name, **base)


def _rng(cfg: Config, *stream) -> np.random.Generator:
    return np.random.default_rng([1000 + cfg.index, *[int(s) for s in stream]])


def _zipf_log_weights(E: int, s: float) -> np.ndarray:
    ranks = np.arange(1, E + 1, dtype=np.float64)
    w = ranks ** (-s)
    w /= w.sum()
    return np.log(w)


def domain_permutation(cfg: Config, mb: int) -> np.ndarray:
    """perm[i] = expert holding Zipf rank i+1 in micro-batch `mb`."""
    if cfg.routing == "single":
        return _rng(cfg, 1, 0).permutation(cfg.E)
    if cfg.routing == "domains4":
        dom = int(_rng(cfg, 2, mb).integers(0, 4))
        return _rng(cfg, 1, dom).permutation(cfg.E)
    if cfg.routing == "fresh":
        return _rng(cfg, 1, mb).permutation(cfg.E)
    if cfg.routing == "stress":
        return _rng(cfg, 1, mb % 4).permutation(cfg.E)
    raise ValueError(cfg.routing)


def _topk_and_gates(logits: np.ndarray, k: int):
    # top-k by logit, ties to the lowest expert id; order = descending logit.
    order = np.argsort(-logits, axis=1, kind="stable")[:, :k]
    sel = np.take_along_axis(logits, order, axis=1)
    sel = sel - sel.max(axis=1, keepdims=True)
    p = np.exp(sel)
    p /= p.sum(axis=1, keepdims=True)
    return order.astype(np.int32), p.astype(np.float32)


def make_routing(cfg: Config, mb: int):
    """Replayed routing of one micro-batch: ids[T,k] int32 (distinct per token), gates[T,k] f32."""
    seed_mb = mb
    rng = _rng(cfg, 3, seed_mb)
    perm = domain_permutation(cfg, mb)
    bias = np.empty(cfg.E, dtype=np.float64)
    bias[perm] = _zipf_log_weights(cfg.E, cfg.zipf_s)
    z = rng.standard_normal((cfg.T, cfg.E))
    logits = z + bias[None, :]
    if cfg.routing != "stress":
        return _topk_and_gates(logits, cfg.k)

    # stress: 5% of tokens forced onto the domain's hottest expert, and some experts empty.
    forced = rng.choice(cfg.T, size=max(1, (cfg.T * 5) // 100), replace=False)
    hot = int(perm[0])

    def route(lg):
        ids, _ = _topk_and_gates(lg, cfg.k)
        for t in forced:
            if hot not in ids[t]:
                ids[t, cfg.k - 1] = hot          # replace the lowest-scoring selected expert
        sel = np.take_along_axis(lg, ids.astype(np.int64), axis=1)
        sel = sel - sel.max(axis=1, keepdims=True)
        p = np.exp(sel)
        p /= p.sum(axis=1, keepdims=True)
        return ids, p.astype(np.float32)

    ids, gates = route(logits)
    if np.bincount(ids.ravel(), minlength=cfg.E).min() > 0:
        logits = logits.copy()
        logits[:, perm[-4:]] = -np.inf
        ids, gates = route(logits)
    return ids, gates


def _bf16(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)


def make_tokens(cfg: Config, mb: int):
    """X[T,h] and dOut[T,h], N(0,1), rounded once to bf16."""
    rng = _rng(cfg, 4, mb)
    X = _bf16(rng.standard_normal((cfg.T, cfg.h), dtype=np.float32))
    dOut = _bf16(rng.standard_normal((cfg.T, cfg.h), dtype=np.float32))
    return X, dOut


def make_weights(cfg: Config, device: str = "cpu"):
    """Wg, Wu [E,h',h] and Wd [E,h,h'], N(0,0.02), bf16.

    On "cpu" the draw is numpy's and reproducible anywhere.  On a GPU device the
    draw uses torch's device generator expert by expert (a 22 GB weight set is not
    drawn on the host); callers that need the same values on the host copy them back.
    """
    if device == "cpu":
        rng = _rng(cfg, 5)
        shp_in = (cfg.E, cfg.hff, cfg.h)
        Wg = _bf16(0.02 * rng.standard_normal(shp_in, dtype=np.float32))
        Wu = _bf16(0.02 * rng.standard_normal(shp_in, dtype=np.float32))
        Wd = _bf16(0.02 * rng.standard_normal((cfg.E, cfg.h, cfg.hff), dtype=np.float32))
        return Wg, Wu, Wd
    gen = torch.Generator(device=device)
    gen.manual_seed(5000 + cfg.index)
    out = []
    for shape in ((cfg.E, cfg.hff, cfg.h), (cfg.E, cfg.hff, cfg.h), (cfg.E, cfg.h, cfg.hff)):
        W = torch.empty(shape, dtype=torch.bfloat16, device=device)
        for e in range(cfg.E):
            W[e] = (0.02 * torch.randn(shape[1:], generator=gen, device=device,
                                       dtype=torch.float32)).to(torch.bfloat16)
        out.append(W)
    return tuple(out)


def make_tokens_device(cfg: Config, mb: int, device: str):
    """Device-side draw of X and dOut for the large configs (same distribution as make_tokens)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(4000 + 100 * cfg.index + mb)
    X = torch.randn((cfg.T, cfg.h), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    dOut = torch.randn((cfg.T, cfg.h), generator=gen, device=device, dtype=torch.float32).to(torch.bfloat16)
    return X, dOut
