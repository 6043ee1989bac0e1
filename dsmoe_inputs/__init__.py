"""Seeded synthetic inputs for the DS-MoE expert layer (shared by tests, bench and the CPU checker).

This module draws random tensors and rounds them to the storage precision.  It holds none of the
layer's arithmetic (no router, softmax, selection or FFN): callers that need routing statistics or
margin conditioning compute them with whichever implementation they are testing and ask this module
only to redraw rows.

The paper's workloads (a text corpus pushed through trained checkpoints, Sec. 4) are not available;
these inputs stand in for them.  Layer shapes follow the paper's Table 1 / Table 6 rows (32 experts,
per-expert hidden size 256..896, embedding size 2048..7168), sparsity follows the 30-40 % active
parameters reported in the abstract and Table 3, and the skewed case follows the remark in Sec. 1
that expert usage can be unbalanced.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20240405


@dataclass(frozen=True)
class LayerConfig:
    """Shape and recipe of one synthetic workload."""

    name: str
    index: int            # config number used in the seed
    T: int                # tokens
    d: int                # d_model
    E: int                # experts
    f: int                # d_ff per expert
    dtype: str            # "f32" | "bf16"
    mode: str             # "topk" | "threshold"
    k: int = 0
    eps: float = 0.0
    router_std: float = 0.02
    zipf_s: float = 0.0   # > 0: router bias -s*ln(rank) over a seeded permutation of experts
    weight_std: float = 0.02

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


def _c2_router_std(d: int) -> float:
    return 1.5 / np.sqrt(d)


CONFIGS: Dict[str, LayerConfig] = {
    # tiny fp32 correctness case
    "c1": LayerConfig("c1", 1, T=128, d=256, E=8, f=64, dtype="f32", mode="topk", k=2),
    # sparse prefill, threshold selection, ~36 % of experts active
    "c2": LayerConfig("c2", 2, T=4096, d=2048, E=32, f=512, dtype="bf16", mode="threshold",
                      eps=0.02, router_std=_c2_router_std(2048)),
    # decode on the same layer: T and selection are overridden per variant
    "c3": LayerConfig("c3", 3, T=128, d=2048, E=32, f=512, dtype="bf16", mode="topk", k=4,
                      eps=0.02, router_std=_c2_router_std(2048)),
    # dense training forward + backward
    "c4": LayerConfig("c4", 4, T=8192, d=2048, E=32, f=512, dtype="bf16", mode="threshold",
                      eps=0.02, router_std=_c2_router_std(2048)),
    # large, Zipf-skewed prefill
    "c5": LayerConfig("c5", 5, T=16384, d=4096, E=64, f=768, dtype="bf16", mode="threshold",
                      eps=0.01, router_std=1.0 / np.sqrt(4096), zipf_s=1.2),
}


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays in an fp32 array."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of fp32 values that are already exactly representable in bf16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(cfg: LayerConfig, variant: int, stream: int) -> np.random.Generator:
    seed = BASE_SEED + 1000 * cfg.index + variant
    return np.random.Generator(np.random.Philox(key=seed, counter=[0, 0, 0, stream]))


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    a = a.astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


@dataclass
class LayerInputs:
    """All tensors of one layer call, as fp32 arrays holding values exact in `cfg.dtype`."""

    cfg: LayerConfig
    variant: int
    x: np.ndarray                     # [T, d]
    w_r: np.ndarray                   # [d, E]
    b_r: Optional[np.ndarray]         # [E] or None
    w_gate: np.ndarray                # [E, d, f]
    w_up: np.ndarray                  # [E, d, f]
    w_down: np.ndarray                # [E, f, d]
    d_out: Optional[np.ndarray] = None  # [T, d] upstream gradient (dense training only)
    redraws: int = field(default=0)


# stream ids (one independent Philox counter block per tensor)
_S_X, _S_WR, _S_WG, _S_WU, _S_WD, _S_DO, _S_PERM, _S_REDRAW, _S_MOA_DO = range(9)


def make_router(cfg: LayerConfig, variant: int = 0):
    w_r = _store(_rng(cfg, variant, _S_WR).standard_normal((cfg.d, cfg.E), dtype=np.float32)
                 * np.float32(cfg.router_std), cfg.dtype)
    b_r = None
    if cfg.zipf_s > 0:
        perm = _rng(cfg, variant, _S_PERM).permutation(cfg.E)
        b = np.empty(cfg.E, dtype=np.float32)
        ranks = np.arange(1, cfg.E + 1, dtype=np.float64)
        b[perm] = (-cfg.zipf_s * np.log(ranks)).astype(np.float32)
        b_r = _store(b, cfg.dtype)
    return w_r, b_r


def make_tokens(cfg: LayerConfig, variant: int = 0, T: Optional[int] = None) -> np.ndarray:
    T = cfg.T if T is None else T
    return _store(_rng(cfg, variant, _S_X).standard_normal((T, cfg.d), dtype=np.float32), cfg.dtype)


def make_experts(cfg: LayerConfig, variant: int = 0):
    std = np.float32(cfg.weight_std)
    shp_in, shp_out = (cfg.E, cfg.d, cfg.f), (cfg.E, cfg.f, cfg.d)
    w_gate = _store(_rng(cfg, variant, _S_WG).standard_normal(shp_in, dtype=np.float32) * std, cfg.dtype)
    w_up = _store(_rng(cfg, variant, _S_WU).standard_normal(shp_in, dtype=np.float32) * std, cfg.dtype)
    w_down = _store(_rng(cfg, variant, _S_WD).standard_normal(shp_out, dtype=np.float32) * std, cfg.dtype)
    return w_gate, w_up, w_down


def make_upstream_grad(cfg: LayerConfig, variant: int = 0, T: Optional[int] = None) -> np.ndarray:
    T = cfg.T if T is None else T
    return _store(_rng(cfg, variant, _S_DO).standard_normal((T, cfg.d), dtype=np.float32), cfg.dtype)


def make_layer(cfg: LayerConfig, variant: int = 0, with_grad: bool = False) -> LayerInputs:
    w_r, b_r = make_router(cfg, variant)
    w_gate, w_up, w_down = make_experts(cfg, variant)
    return LayerInputs(cfg, variant, make_tokens(cfg, variant), w_r, b_r, w_gate, w_up, w_down,
                       make_upstream_grad(cfg, variant) if with_grad else None)


def redraw_rows(inp: LayerInputs, rows: np.ndarray) -> None:
    """Replace the given token rows of `inp.x` by fresh draws (used for margin conditioning).

    Each call uses a new sub-stream so repeated redraws of the same row differ; the sequence is a
    pure function of (config, variant, call number).
    """
    rows = np.asarray(rows, dtype=np.int64)
    if rows.size == 0:
        return
    inp.redraws += 1
    cfg = inp.cfg
    seed = BASE_SEED + 1000 * cfg.index + inp.variant
    g = np.random.Generator(np.random.Philox(key=seed, counter=[0, 0, inp.redraws, _S_REDRAW]))
    inp.x[rows] = _store(g.standard_normal((rows.size, cfg.d), dtype=np.float32), cfg.dtype)


# --------------------------------------------------------------------------------------------------
# Mixture-of-Attention-heads layer (Sec. 3.2).  Shapes follow Table 1: DS-MoE-1B has 16 attention experts
# of 2 heads of 64, DS-MoE-6B 8 experts of 4 heads of 128; the number of heads per expert is the number of
# shared key/value heads.  Keys and values are drawn directly (the paper takes the cache as given).
# --------------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class MoaConfig:
    name: str
    index: int
    T: int                # new tokens (the last T cache positions)
    L: int                # cache length
    d: int                # d_model
    E: int                # attention experts
    n_head: int           # heads per expert = shared key/value heads
    d_head: int
    dtype: str            # "f32" | "bf16"
    mode: str             # "dense" | "topk" | "threshold"
    k: int = 0
    eps: float = 0.0
    router_std: float = 0.02
    weight_std: float = 0.02

    def with_(self, **kw) -> "MoaConfig":
        return replace(self, **kw)


MOA_CONFIGS: Dict[str, MoaConfig] = {
    # tiny correctness case
    "m1": MoaConfig("m1", 11, T=48, L=80, d=128, E=8, n_head=2, d_head=64, dtype="bf16", mode="topk", k=2,
                    router_std=0.1),
    # prefill of the 6B shape (Table 1), every expert active: how the paper runs the attention layer at inference
    "m2": MoaConfig("m2", 12, T=2048, L=2048, d=4096, E=8, n_head=4, d_head=128, dtype="bf16", mode="dense",
                    router_std=1.0 / np.sqrt(4096)),
}


@dataclass
class MoaInputs:
    cfg: MoaConfig
    variant: int
    x: np.ndarray        # [T, d]
    w_r: np.ndarray      # [d, E]
    w_q: np.ndarray      # [E, d, n_head * d_head]
    k: np.ndarray        # [n_head, L, d_head]
    v: np.ndarray        # [n_head, L, d_head]
    w_o: np.ndarray      # [E, n_head * d_head, d]
    b_r: Optional[np.ndarray] = None
    redraws: int = field(default=0)


def make_moa(cfg: MoaConfig, variant: int = 0) -> MoaInputs:
    hd = cfg.n_head * cfg.d_head
    std = np.float32(cfg.weight_std)
    n = lambda stream, shape: _rng(cfg, variant, stream).standard_normal(shape, dtype=np.float32)
    return MoaInputs(
        cfg, variant,
        x=_store(n(_S_X, (cfg.T, cfg.d)), cfg.dtype),
        w_r=_store(n(_S_WR, (cfg.d, cfg.E)) * np.float32(cfg.router_std), cfg.dtype),
        w_q=_store(n(_S_WG, (cfg.E, cfg.d, hd)) * std, cfg.dtype),
        k=_store(n(_S_WU, (cfg.n_head, cfg.L, cfg.d_head)), cfg.dtype),
        v=_store(n(_S_DO, (cfg.n_head, cfg.L, cfg.d_head)), cfg.dtype),
        w_o=_store(n(_S_WD, (cfg.E, hd, cfg.d)) * std, cfg.dtype),
    )


def make_moa_upstream_grad(cfg: MoaConfig, variant: int = 0) -> np.ndarray:
    """Upstream gradient d_out [T, d] for the attention layer's dense-training backward."""
    return _store(_rng(cfg, variant, _S_MOA_DO).standard_normal((cfg.T, cfg.d), dtype=np.float32), cfg.dtype)
