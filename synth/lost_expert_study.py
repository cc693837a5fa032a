"""Routing side of the paper's lost-expert study (Sec. 4.2) on a synthetic workload.

For failing fractions r in {1/64 ... 1/2} and both ways of choosing the failed experts
("every nth" and "task-based": the most activated experts by the GPU's activation counts) this
prints how much of the routing changes: the share of tokens that lose at least one of their
experts, the share of (token, choice) pairs that move, and the share of the unfailed layer's
combine weight that sat on failed experts.  The paper's accuracy numbers need DeepSeek V3 weights
and benchmark datasets and are not reproduced; this only exercises the masks through the library.

Usage: python -m synth.lost_expert_study [--workload c3]
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

import synth

from paper_2602_21140_amd.binding import mask_every_nth, mask_most_activated
from synth.resident import ResidentLayer


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c3")
    args = ap.parse_args()
    cfg = synth.get_config(args.workload)
    g = ResidentLayer(cfg, device="cuda:0", with_weights=False, failed=[])
    L, T, k, E = g.layer, cfg.T, cfg.k, cfg.E
    logits, top0, w0, _phys = L.route(g.x, g.w_router_packed, T)
    assert logits.shape == (T, E) and logits.dtype == torch.float32
    top0, w0 = top0.clone(), w0.clone()
    counts = L.expert_counts(top0, T).cpu().numpy()
    rows = []
    for den in (64, 32, 16, 8, 4, 2):
        for kind in ("every_nth", "task_based"):
            mask = mask_every_nth(E, den) if kind == "every_nth" else mask_most_activated(counts, E // den)
            try:
                stats = g.set_failed([], expert_failed=mask)
            except Exception as exc:  # not enough live experts reachable for this mask
                rows.append({"r": f"1/{den}", "kind": kind, "error": str(exc)})
                continue
            _lg, top, w, _phys = L.route(None, None, T, logits=logits, logits_given=True)
            dead = torch.from_numpy(mask.astype(bool)).to(top0.device)
            on_failed = dead[top0.long()]
            rows.append({"r": f"1/{den}", "kind": kind, "lost_experts": stats["n_lost_experts"],
                         "tokens_affected": float(on_failed.any(dim=1).float().mean()),
                         "choices_moved": float(on_failed.float().mean()),
                         "weight_mass_moved": float((w0 * on_failed).sum() / w0.sum()),
                         "routes_to_failed_after": int(dead[top.long()].sum())})
    g.close()
    for r in rows:
        print(json.dumps(r))


if __name__ == "__main__":
    main()
