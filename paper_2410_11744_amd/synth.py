"""Seeded synthetic inputs with the shapes and value distributions of the five benchmark
configurations (Llama-2-shaped attention tensors, draft/target logit tables).

This module holds no arithmetic of the method itself: it only draws random tensors.  Both
the GPU path and the CPU oracle are fed from here (the oracle receives host copies of the
very same tensors), so neither side generates inputs for the other.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    vocab: int
    dtype: str                    # "f32" or "bf16" (attention tensors)
    logit_kind: str               # "normal" or "zipf"
    logit_sigma: float            # std of draft logits ("normal") or of the Zipf noise
    target_sigma: Tuple[float, float]   # target = draft + N(0, s^2), s uniform in this range per sequence
    temps: Tuple[float, ...]      # temperature per sequence (draft and target alike)
    n_nodes: Tuple[int, ...]      # tree rows per sequence, root included
    prefix_len: Tuple[int, ...]
    seed: int


def _ragged_70b() -> Tuple[Tuple[int, ...], Tuple[int, ...]]:
    rng = np.random.default_rng(5)
    p = tuple(int(x) for x in rng.integers(1024, 8193, 8))
    n = tuple(int(x) for x in rng.integers(64, 769, 8))
    return n, p


_N5, _P5 = _ragged_70b()

CONFIGS = {
    "tiny_f32": Config("tiny_f32", 1, 8, 8, 64, 1000, "f32", "normal", 2.0, (0.5, 0.5), (1.0,), (32,), (128,), 0),
    "llama2_7b": Config("llama2_7b", 32, 32, 32, 128, 32000, "bf16", "normal", 3.0, (1.0, 1.0), (0.6,), (128,), (1024,), 1),
    "llama2_13b": Config("llama2_13b", 40, 40, 40, 128, 32000, "bf16", "zipf", 0.3, (1.5, 1.5), (1.0,), (256,), (2048,), 2),
    "llama2_70b": Config("llama2_70b", 80, 64, 8, 128, 32000, "bf16", "normal", 3.0, (0.8, 0.8), (0.6,), (512,), (4096,), 3),
    "llama2_70b_ragged8": Config("llama2_70b_ragged8", 80, 64, 8, 128, 32000, "bf16", "normal", 3.0, (0.5, 2.0),
                                 (0.6,) * 4 + (1.0,) * 4, _N5, _P5, 4),
}
ORDER = ["tiny_f32", "llama2_7b", "llama2_13b", "llama2_70b", "llama2_70b_ragged8"]
# supplementary point: the 70B shape with a tree so narrow (G*N = 256 rows per K/V byte) that
# tree attention is bound by the K/V stream from HBM, not by the matrix cores
CONFIGS["llama2_70b_n32"] = Config("llama2_70b_n32", 80, 64, 8, 128, 32000, "bf16", "normal", 3.0, (0.8, 0.8), (0.6,),
                                   (32,), (4096,), 3)


def make_logits(cfg: Config, seed: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Draft and target logit tables, fp32 [sum N, vocab], one row per tree node."""
    rng = np.random.default_rng((cfg.seed if seed is None else seed) * 7919 + 17)
    drafts, targets = [], []
    for s, n in enumerate(cfg.n_nodes):
        if cfg.logit_kind == "normal":
            d = rng.standard_normal((n, cfg.vocab), dtype=np.float32) * np.float32(cfg.logit_sigma)
        else:  # Zipf over a per-row random ranking: logit = -1.1 ln(rank) + noise
            base = (-1.1 * np.log(np.arange(1, cfg.vocab + 1))).astype(np.float32)
            d = np.empty((n, cfg.vocab), dtype=np.float32)
            for i in range(n):
                d[i] = base[rng.permutation(cfg.vocab)]
            d += rng.standard_normal((n, cfg.vocab), dtype=np.float32) * np.float32(cfg.logit_sigma)
        lo, hi = cfg.target_sigma
        sig = lo if hi == lo else float(rng.uniform(lo, hi))
        t = d + rng.standard_normal((n, cfg.vocab), dtype=np.float32) * np.float32(sig)
        drafts.append(d)
        targets.append(t.astype(np.float32))
    return np.concatenate(drafts), np.concatenate(targets)


def attention_shapes(cfg: Config):
    tn, tp = sum(cfg.n_nodes), sum(cfg.prefix_len)
    return ((tn, cfg.n_q_heads, cfg.head_dim), (tp, cfg.n_kv_heads, cfg.head_dim),
            (tn, cfg.n_kv_heads, cfg.head_dim))


def make_attention_inputs(cfg: Config, layer: int, device="cpu", seed: Optional[int] = None):
    """q, k_prefix, v_prefix, k_tree, v_tree ~ N(0,1), drawn in fp32 then rounded to the
    config's dtype.  Each layer has its own stream.  Returns torch tensors on `device`."""
    import torch
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    g = torch.Generator(device=device)
    g.manual_seed(((cfg.seed if seed is None else seed) + 1) * 1000003 + layer)
    qs, ps, ts = attention_shapes(cfg)
    mk = lambda sh: torch.randn(sh, generator=g, device=device, dtype=torch.float32).to(dt)
    return mk(qs), mk(ps), mk(ps), mk(ts), mk(ts)


def small_config(name: str, **kw) -> Config:
    """A config with overridden fields (tests use it for ragged and odd shapes)."""
    base = CONFIGS["tiny_f32"]
    fields = dict(base.__dict__)
    fields.update(name=name, **kw)
    return Config(**fields)
