"""Shared test harness: builds a layer on the GPU from the seeded workloads and gives the oracle
the very same bits.  Holds no arithmetic of the method: the GPU side goes through the binding,
the CPU side through oracle/."""
from __future__ import annotations

from typing import Dict, Iterable, List, Optional

import numpy as np
import torch

import synth
from oracle import revive_oracle as orc
from synth.resident import ResidentLayer

TOL = {"fp32": 1e-4, "bf16": 1e-2}


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    """Per-tensor relative error: max |gpu - ref| / max |ref|."""
    denom = float(np.abs(ref).max())
    return float(np.abs(gpu - ref).max()) / (denom if denom > 0 else 1.0)


class GpuLayer(ResidentLayer):
    """The resident GPU layer plus oracle-side (fp64, CPU) views of the very same bits."""

    # ---- oracle-side views of the same bits ------------------------------------------------
    def oracle_map(self) -> orc.ExpertMap:
        c = self.cfg
        return orc.build_map(self.p2l, self.failed, c.slots_per_rank, c.E, c.max_replicas,
                             expert_failed=self.expert_failed)

    # The oracle's weights are drawn again from the seeded generator (same seed, same device, hence
    # the same bits the layer packed), never read back through the library's packers: a mistake in
    # the packed layout then shows up as a parity failure instead of cancelling out.
    def expert_f64(self, e: int) -> Dict[str, np.ndarray]:
        """Expert e's matrices in math layout, fp64."""
        return {n: f64(t) for n, t in synth.draw_expert(self.cfg, int(e), self.device).items()}

    def slot_expert_f64(self, p: int) -> Dict[str, np.ndarray]:
        """The matrices of the expert that slot p holds."""
        return self.expert_f64(int(self.p2l[p]))

    def shared_f64(self) -> Optional[Dict[str, np.ndarray]]:
        sh = synth.draw_shared(self.cfg, self.device)
        return None if sh is None else {n: f64(t) for n, t in sh.items()}


def compare_selection(cfg, gpu_top: np.ndarray, sel: np.ndarray, ref_top: np.ndarray, gap_limit=1e-5):
    """Tokens where the two ordered selections differ, split into near-ties and real mismatches.

    `sel` are the oracle's fp64 selection scores.  A disagreement is a near-tie when the scores of
    the experts the two lists differ on are within gap_limit of each other, or (grouped) when the
    kept groups differ and the scores of the groups in dispute are within gap_limit."""
    near, bad = [], []
    for t in np.nonzero((gpu_top != ref_top).any(axis=1))[0]:
        gap = orc.selection_gap(sel[t], ref_top[t], gpu_top[t])
        if cfg.n_group > 1:
            gsz = cfg.E // cfg.n_group
            gs = orc.group_scores(sel[t], cfg.n_group)
            kept = set(int(g) for g in orc.kept_groups(sel[t], cfg.n_group, cfg.topk_group))
            stray = set(int(e) // gsz for e in gpu_top[t]) - kept
            if stray:   # the GPU kept a group the oracle dropped: compare it with the weakest kept group
                gap = max(min(gs[g] for g in kept) - gs[g] for g in stray)
        (near if gap < gap_limit else bad).append(int(t))
    return near, bad
