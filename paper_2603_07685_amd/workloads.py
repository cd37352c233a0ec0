"""Seeded synthetic inputs for the MoE expert-layer path.

This module only *generates inputs*: Gaussian tensors rounded to the storage
format, router logits (the gate projection sits in front of the path, paper
Sec. 2.1.2 item 1 and Sec. 4.3.4: the GEMM is outside the fused router), and
forced routing maps with a prescribed per-expert load (the paper benchmarks
with force-balanced routing, Sec. 8.2).  It holds none of the layer's arithmetic and
imports neither the HIP binding nor the CPU oracle; both are fed from here.

Everything is numpy on the host.  `device_gaussian_bf16` is the one exception:
the big configurations (hundreds of millions of weights) are drawn with
torch's seeded device generator so that the GPU machine does not spend minutes in
a host RNG; tests copy the slices they need back to the host for the oracle.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

SOFTMAX = 0
SIGMOID = 1


# --------------------------------------------------------------------------
# storage-format helpers (bit-level conversions, no layer arithmetic)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 values that are exactly representable in bfloat16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# --------------------------------------------------------------------------
# configurations (the five workloads the benchmark definition names)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int                 # tokens on this GPU
    h: int                 # hidden size
    f: int                 # expert ffn width (SwiGLU: fc1 produces 2f)
    E: int                 # experts addressed by the grouped GEMM on this GPU
    k: int                 # top-k
    E_router: int          # experts the router scores (global count)
    score: int             # SOFTMAX / SIGMOID
    norm_topk: bool        # renormalise the k selected scores
    load: str              # "router" | "zipf" | "cv" | "zeros" | "hot"
    load_param: float = 0.0
    shared_f: int = 0      # width of the always-on shared expert (0: none)
    fp8: bool = False      # blockwise fp8 (1x128 / 128x128, fp32 scales) forward and data-gradient GEMMs
    mx: bool = False       # MXFP8 (1x32, E8M0 scales) forward and data-gradient GEMMs
    align: int = 1         # per-expert row padding (fp8 wgrad: 128)
    std: float = 0.02
    seed: int = 1234
    # router branches (group-limited top-k, load-balancing bias, score scaling); the defaults are the plain router
    n_group: int = 1       # expert groups of E_router / n_group
    topk_group: int = 1    # groups a token may draw its experts from
    route_scale: float = 1.0
    bias_std: float = 0.0  # > 0: a seeded N(0, bias_std^2) per-expert selection bias

    @property
    def grouped_router(self) -> bool:
        return self.n_group > 1 or self.bias_std > 0.0

    @property
    def R(self) -> int:
        return self.T * self.k

    @property
    def Rcap(self) -> int:
        """Worst-case padded row count: every expert may add align-1 pad rows."""
        return self.R + self.E * (self.align - 1)

    def model_flops(self) -> float:
        """fwd+bwd model FLOPs: 3 GEMM passes x 2 GEMMs x 2*R*h*(2f|f) = 18 R h f (+ shared)."""
        return 18.0 * self.R * self.h * self.f + 18.0 * self.T * self.h * self.shared_f


CONFIGS = {
    "C1": MoEConfig("C1-tiny", T=256, h=128, f=256, E=8, k=2, E_router=8, score=SOFTMAX,
                    norm_topk=False, load="router", seed=1235),
    "MID": MoEConfig("mid", T=2048, h=1024, f=512, E=8, k=2, E_router=8, score=SOFTMAX,
                     norm_topk=False, load="router", seed=1240),
    "C2": MoEConfig("C2-mixtral", T=8192, h=4096, f=14336, E=8, k=2, E_router=8, score=SOFTMAX,
                    norm_topk=False, load="router", seed=1236),
    "C3": MoEConfig("C3-qwen3-share", T=16384, h=4096, f=1536, E=16, k=8, E_router=128, score=SOFTMAX,
                    norm_topk=False, load="zipf", load_param=1.2, seed=1237),
    "C4": MoEConfig("C4-dsv3-share", T=16384, h=7168, f=2048, E=32, k=8, E_router=256, score=SIGMOID,
                    norm_topk=True, load="cv", load_param=0.3, shared_f=2048, seed=1238),
    # the C4 layer behind the published DeepSeek-V3 router: 8 groups of 32, 4 kept, bias, weights scaled by 2.5
    "C4G": MoEConfig("C4-dsv3-share-grouped-router", T=16384, h=7168, f=2048, E=32, k=8, E_router=256, score=SIGMOID,
                     norm_topk=True, load="cv", load_param=0.3, shared_f=2048, seed=1238,
                     n_group=8, topk_group=4, route_scale=2.5, bias_std=0.1),
    "C7S": MoEConfig("C7-small-grouped-router", T=1024, h=512, f=256, E=32, k=4, E_router=32, score=SIGMOID,
                     norm_topk=True, load="router", shared_f=256, seed=1243,
                     n_group=4, topk_group=2, route_scale=2.5, bias_std=0.1),
    "C5S": MoEConfig("C5-small-fp8", T=1024, h=512, f=256, E=8, k=4, E_router=32, score=SIGMOID,
                     norm_topk=True, load="cv", load_param=0.3, shared_f=256, fp8=True, align=128, seed=1241),
    "C6S": MoEConfig("C6-small-mxfp8", T=1024, h=512, f=256, E=8, k=4, E_router=32, score=SIGMOID,
                     norm_topk=True, load="cv", load_param=0.3, shared_f=256, mx=True, align=128, seed=1242),
    "C6": MoEConfig("C6-dsv3-share-mxfp8", T=16384, h=7168, f=2048, E=32, k=8, E_router=256, score=SIGMOID,
                    norm_topk=True, load="cv", load_param=0.3, shared_f=2048, mx=True, align=128, seed=1239),
    "C5": MoEConfig("C5-dsv3-share-fp8", T=16384, h=7168, f=2048, E=32, k=8, E_router=256, score=SIGMOID,
                    norm_topk=True, load="cv", load_param=0.3, shared_f=2048, fp8=True, align=128, seed=1239),
}


def expert_bias(cfg: "MoEConfig"):
    """The seeded selection bias of a config (None when it has none)."""
    if cfg.bias_std <= 0.0:
        return None
    return (rng(cfg.seed, 9).standard_normal(cfg.E_router, dtype=np.float32) * np.float32(cfg.bias_std)).astype(np.float32)


def rng(seed: int, stream: int = 0) -> np.random.Generator:
    """Counter-based generator; `stream` separates tensors drawn under one seed."""
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def gaussian_bf16(shape, std: float, seed: int, stream: int) -> np.ndarray:
    """N(0, std^2) fp32 values already rounded to bf16 precision (host)."""
    g = rng(seed, stream)
    x = g.standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return bf16_round(x)


def gaussian_f32(shape, std: float, seed: int, stream: int) -> np.ndarray:
    g = rng(seed, stream)
    return g.standard_normal(size=shape, dtype=np.float32) * np.float32(std)


def device_gaussian_bf16(shape, std: float, seed: int, stream: int, device="cuda"):
    """N(0, std^2) bf16 tensor drawn on the device with torch's seeded generator."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000003 + stream)
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    out.normal_(0.0, std, generator=g)
    return out


def router_logits(T: int, h: int, E: int, std: float, seed: int):
    """x ~ N(0, std^2), W_r ~ N(0, std^2) in fp32; logits = x @ W_r accumulated in fp64, stored fp32.

    The logits array (not x, W_r) is what both the oracle and the HIP router
    receive, so both select on identical fp32 values.
    """
    x = gaussian_f32((T, h), std, seed, 101)
    wr = gaussian_f32((h, E), std, seed, 102)
    logits = (x.astype(np.float64) @ wr.astype(np.float64)).astype(np.float32)
    return x, wr, logits


# --------------------------------------------------------------------------
# forced routing maps with a prescribed per-expert load
# --------------------------------------------------------------------------
def _largest_remainder(weights: np.ndarray, total: int) -> np.ndarray:
    w = np.asarray(weights, dtype=np.float64)
    w = w / w.sum() * total
    base = np.floor(w).astype(np.int64)
    rem = total - int(base.sum())
    order = np.argsort(-(w - base), kind="stable")
    base[order[:rem]] += 1
    return base


def load_zipf(R: int, E: int, s: float) -> np.ndarray:
    """m_e proportional to rank^-s, summing exactly to R."""
    return _largest_remainder(np.arange(1, E + 1, dtype=np.float64) ** (-s), R)


def load_cv(R: int, E: int, cv: float, seed: int) -> np.ndarray:
    """m_e = mean*(1 + cv*z_e), z ~ N(0,1) clipped to +-2.5, rescaled to sum exactly to R."""
    z = np.clip(rng(seed, 201).standard_normal(E), -2.5, 2.5)
    return _largest_remainder(np.maximum(1.0 + cv * z, 0.05), R)


def load_zeros(R: int, E: int, n_zero: int, seed: int) -> np.ndarray:
    """n_zero experts get no rows; the rest share R uniformly."""
    dead = rng(seed, 202).permutation(E)[:n_zero]
    w = np.ones(E)
    w[dead] = 0.0
    return _largest_remainder(w, R)


def load_hot(R: int, E: int, frac: float, seed: int) -> np.ndarray:
    """One expert gets `frac` of all rows; the rest share the remainder uniformly."""
    hot = int(rng(seed, 203).integers(E))
    w = np.full(E, (1.0 - frac) / (E - 1))
    w[hot] = frac
    return _largest_remainder(w, R)


def forced_routing(counts: np.ndarray, T: int, k: int, seed: int) -> np.ndarray:
    """idx[T,k] (int32) in which expert e appears exactly counts[e] times.

    Expert ids are listed in sorted order (e repeated counts[e] times), entry j
    is dealt to token pi(j mod T), slot j div T, then each token's slots are
    shuffled.  A token holds one expert twice only when counts[e] > T, which
    stands for rows that reach this GPU from other ranks' tokens under expert
    parallelism; the bytes and FLOPs are the same.
    """
    counts = np.asarray(counts, dtype=np.int64)
    assert counts.sum() == T * k
    g = rng(seed, 204)
    ids = np.repeat(np.arange(len(counts), dtype=np.int32), counts)
    pi = g.permutation(T)
    idx = np.empty((T, k), dtype=np.int32)
    j = np.arange(T * k)
    idx[pi[j % T], j // T] = ids
    # shuffle slot order per token
    keys = g.random((T, k))
    order = np.argsort(keys, axis=1)
    return np.take_along_axis(idx, order, axis=1)


def expert_load(cfg: MoEConfig, variant: Optional[str] = None) -> Optional[np.ndarray]:
    """Per-expert row counts for the forced map of `cfg` (None: use the router's own top-k)."""
    load = variant or cfg.load
    if load == "router":
        return None
    if load == "zipf":
        return load_zipf(cfg.R, cfg.E, cfg.load_param or 1.2)
    if load == "cv":
        return load_cv(cfg.R, cfg.E, cfg.load_param or 0.3, cfg.seed)
    if load == "zeros":
        return load_zeros(cfg.R, cfg.E, 4, cfg.seed)
    if load == "hot":
        return load_hot(cfg.R, cfg.E, 0.4, cfg.seed)
    if load == "uniform":
        return _largest_remainder(np.ones(cfg.E), cfg.R)
    raise ValueError(load)


def routing_map(cfg: MoEConfig, variant: Optional[str] = None) -> Optional[np.ndarray]:
    """Forced idx[T,k] for configs whose load is synthesised; None for router-driven ones."""
    counts = expert_load(cfg, variant)
    if counts is None:
        return None
    return forced_routing(counts, cfg.T, cfg.k, cfg.seed)


def forced_probs(T: int, k: int, seed: int) -> np.ndarray:
    """Positive combine weights summing to 1 per token (stand-in for router output on forced maps)."""
    p = rng(seed, 205).random((T, k), dtype=np.float32) + np.float32(0.25)
    return (p / p.sum(axis=1, keepdims=True)).astype(np.float32)
