"""Seeded draws of activations, weights, logits and the static placement.

Every tensor has its own child seed derived from (config seed, tensor id), so
any single expert can be regenerated alone.  Draws are made with torch on the
requested device, rounded once to the layer's working dtype; whoever needs a
CPU copy takes `.cpu()` of exactly those bits.

Distributions: x ~ N(0, 1); router and expert matrices ~ N(0, 1/H)
(variance 1/H), so router logits are ~ N(0, 1).
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Optional, Sequence

import numpy as np
import torch

from .configs import LayerConfig

_TENSOR_X, _TENSOR_ROUTER, _TENSOR_SHARED, _TENSOR_LOGITS, _TENSOR_EXPERT0 = 0, 1, 2, 3, 16
_TENSOR_SKEW = 7  # ids 4..6 belong to the shared expert


def work_dtype(cfg: LayerConfig) -> torch.dtype:
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[cfg.dtype]


def _gen(cfg: LayerConfig, tensor_id: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((cfg.seed * 1_000_003 + tensor_id) * 7919 + 12345)
    return g


def _normal(cfg, tensor_id, shape, std, device, dtype=None):
    g = _gen(cfg, tensor_id, device)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    return t.to(dtype if dtype is not None else work_dtype(cfg))


def draw_x(cfg: LayerConfig, device="cpu") -> torch.Tensor:
    """Token activations [T, H] in the working dtype."""
    return _normal(cfg, _TENSOR_X, (cfg.T, cfg.H), 1.0, device)


def draw_router(cfg: LayerConfig, device="cpu") -> torch.Tensor:
    """Router matrix [H, E] in the working dtype.

    With `cfg.router_skew` > 0 column e is scaled by exp(router_skew * z_e), z_e ~ N(0, 1): the
    logits of some experts spread wider than others', so top-k picks them more often and the rows
    per expert slot become uneven, as under real traffic.
    """
    if cfg.router_skew == 0.0:
        return _normal(cfg, _TENSOR_ROUTER, (cfg.H, cfg.E), cfg.H ** -0.5, device)
    w = _normal(cfg, _TENSOR_ROUTER, (cfg.H, cfg.E), cfg.H ** -0.5, device, torch.float32)
    z = _normal(cfg, _TENSOR_SKEW, (cfg.E,), 1.0, device, torch.float32)
    return (w * torch.exp(cfg.router_skew * z)).to(work_dtype(cfg))


def draw_logits(cfg: LayerConfig, device="cpu") -> torch.Tensor:
    """Stand-alone fp32 router logits [T, E] ~ N(0,1) (for tests that skip the router product)."""
    return _normal(cfg, _TENSOR_LOGITS, (cfg.T, cfg.E), 1.0, device, torch.float32)


def draw_expert(cfg: LayerConfig, e: int, device="cpu") -> Dict[str, torch.Tensor]:
    """One routed expert: gate [H, I], up [H, I], down [I, H] (y = (silu(x g) * (x u)) d)."""
    std = cfg.H ** -0.5
    base = _TENSOR_EXPERT0 + 3 * e
    return {"gate": _normal(cfg, base + 0, (cfg.H, cfg.I), std, device),
            "up": _normal(cfg, base + 1, (cfg.H, cfg.I), std, device),
            "down": _normal(cfg, base + 2, (cfg.I, cfg.H), std, device)}


def draw_shared(cfg: LayerConfig, device="cpu") -> Optional[Dict[str, torch.Tensor]]:
    """The always-on shared expert (width I_shared), or None."""
    if cfg.I_shared == 0:
        return None
    std = cfg.H ** -0.5
    # three separate ids inside the gap between the fixed ids and the experts
    return {"gate": _normal(cfg, _TENSOR_SHARED + 2, (cfg.H, cfg.I_shared), std, device),
            "up": _normal(cfg, _TENSOR_SHARED + 3, (cfg.H, cfg.I_shared), std, device),
            "down": _normal(cfg, _TENSOR_SHARED + 4, (cfg.I_shared, cfg.H), std, device)}


def failed_mask(cfg: LayerConfig, failed: Optional[Iterable[int]] = None) -> np.ndarray:
    """uint8[R], 1 where the rank is failed (default: the config's failed ranks)."""
    m = np.zeros(cfg.n_ranks, dtype=np.uint8)
    for r in (cfg.failed_ranks if failed is None else failed):
        m[r] = 1
    return m


def make_placement(cfg: LayerConfig) -> np.ndarray:
    """Static physical placement: int32[P], logical expert held by each slot.

    Rank r owns slots [r*S, (r+1)*S).  Its first E/R slots hold its primaries
    [r*E/R, (r+1)*E/R); the remaining slots are redundant copies.

    Round-robin rule (n_unprotected < 0): the j-th redundant slot of rank r
    copies the j-th primary of rank (r+1) mod R, so a copy never sits beside
    its primary.

    Targeted rule (n_unprotected >= 0): the primaries of the config's failed
    ranks, in ascending order and without the last `n_unprotected` of them,
    are copied into the redundant slots of the surviving ranks (ascending
    rank, ascending slot).  The unprotected ones get no copy anywhere.  Every
    redundant slot still free afterwards (including the failed ranks' own)
    follows the round-robin rule, skipping unprotected experts by moving on to
    the next expert id.
    """
    R, S, E = cfg.n_ranks, cfg.slots_per_rank, cfg.E
    assert E % R == 0, "experts must split evenly over ranks"
    per = E // R
    n_red = S - per
    assert n_red >= 0
    p2l = np.full(R * S, -1, dtype=np.int32)
    for r in range(R):
        for s in range(per):
            p2l[r * S + s] = r * per + s

    red_slots = [(r, r * S + per + j, j) for r in range(R) for j in range(n_red)]
    forbidden: set = set()
    if cfg.n_unprotected >= 0:
        failed = sorted(cfg.failed_ranks)
        lost_primaries: List[int] = [r * per + s for r in failed for s in range(per)]
        n_prot = len(lost_primaries) - cfg.n_unprotected
        protect, forbidden = lost_primaries[:n_prot], set(lost_primaries[n_prot:])
        free = [p for (r, p, j) in red_slots if r not in failed]
        assert len(protect) <= len(free), "not enough surviving redundant slots"
        for e, p in zip(protect, free):
            p2l[p] = e
    for (r, p, j) in red_slots:
        if p2l[p] >= 0:
            continue
        e = ((r + 1) % R) * per + (j % per)
        while e in forbidden:
            e = (e + 1) % E
        p2l[p] = e
    counts = np.bincount(p2l, minlength=E)
    assert counts.max() <= cfg.max_replicas, "placement exceeds max_replicas"
    return p2l
