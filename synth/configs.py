"""The five layer configurations the workloads are built from.

Shapes follow a DeepSeek-V3-style MoE layer (hidden 7168, 256 routed experts,
8 groups / top-4 groups / top-8 experts, SwiGLU width 2048, one shared expert)
and smaller relatives of it; expert-parallel ranks are simulated as contiguous
segments of physical expert slots inside one GPU's memory.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int                 # tokens
    H: int                 # hidden size
    E: int                 # logical routed experts
    k: int                 # experts per token
    I: int                 # routed expert intermediate width
    I_shared: int          # shared expert width (0 = no shared expert)
    n_ranks: int           # simulated expert-parallel ranks R
    slots_per_rank: int    # physical expert slots per rank S
    max_replicas: int      # upper bound on copies of one logical expert
    score_fn: str          # "softmax" | "sigmoid"
    n_group: int           # 1 = ungrouped
    topk_group: int
    dtype: str             # "fp32" | "bf16"
    failed_ranks: Tuple[int, ...]
    # placement recipe: experts that must own a copy on a surviving rank are
    # the primaries of the failed ranks, minus the last `n_unprotected` of them
    n_unprotected: int = -1   # -1: plain round-robin replicas (no targeting)
    seed: int = 0
    # skewed expert load: router column e is scaled by exp(router_skew * z_e), z_e ~ N(0, 1), so
    # that some experts' logits spread wider and win top-k more often (0 = near-uniform load)
    router_skew: float = 0.0

    @property
    def P(self) -> int:
        return self.n_ranks * self.slots_per_rank

    @property
    def N(self) -> int:
        return self.T * self.k


CONFIGS = {
    # tiny fp32 layer, rank 2 failed, round-robin replicas
    "c1": LayerConfig("c1", T=64, H=256, E=16, k=2, I=128, I_shared=0,
                      n_ranks=4, slots_per_rank=5, max_replicas=2,
                      score_fn="softmax", n_group=1, topk_group=1, dtype="fp32",
                      failed_ranks=(2,)),
    # mid-size bf16 layer; 63 surviving slots cannot hold 64 experts, so the
    # failed rank's last primary is the one unavoidable lost expert
    "c2": LayerConfig("c2", T=4096, H=2048, E=64, k=6, I=1408, I_shared=2816,
                      n_ranks=8, slots_per_rank=9, max_replicas=2,
                      score_fn="softmax", n_group=1, topk_group=1, dtype="bf16",
                      failed_ranks=(3,), n_unprotected=1),
    # DeepSeek-V3-shaped decode share, one failed rank, every lost primary
    # has a surviving copy: the pure remap case
    "c3": LayerConfig("c3", T=8192, H=7168, E=256, k=8, I=2048, I_shared=2048,
                      n_ranks=32, slots_per_rank=9, max_replicas=2,
                      score_fn="sigmoid", n_group=8, topk_group=4, dtype="bf16",
                      failed_ranks=(5,), n_unprotected=0),
    # same shapes, three failed ranks, five experts lose every copy
    "c4": LayerConfig("c4", T=8192, H=7168, E=256, k=8, I=2048, I_shared=2048,
                      n_ranks=32, slots_per_rank=9, max_replicas=4,
                      score_fn="sigmoid", n_group=8, topk_group=4, dtype="bf16",
                      failed_ranks=(5, 13, 22), n_unprotected=5),
    # large-expert-count prefill chunk; the mask flips from no failure to two
    # failed ranks between two replays of one captured graph
    "c5": LayerConfig("c5", T=32768, H=7168, E=384, k=8, I=2048, I_shared=2048,
                      n_ranks=48, slots_per_rank=9, max_replicas=2,
                      score_fn="softmax", n_group=1, topk_group=1, dtype="bf16",
                      failed_ranks=(7, 29)),
}


def get_config(name: str) -> LayerConfig:
    return CONFIGS[name]


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some sizes replaced (reduced-size test variants)."""
    return replace(cfg, **kw)
