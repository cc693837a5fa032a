"""GPU parity over randomly drawn layer configurations.

Each configuration stays inside the limits the library documents (fp32 or bf16, 1-16 ranks, with or
without spare slots, grouped or not, softmax or sigmoid, any token count from 1 to a few thousand,
even or uneven load, random failed ranks) and is first checked on the host to leave at least k
reachable experts.  The whole layer is compared with the oracle stage by stage: indices bit for
bit, values within the dtype's tolerance."""
import numpy as np
import pytest
import torch

import synth
from oracle import revive_oracle as orc
from harness import GpuLayer, TOL, f64, rel_err

pytestmark = pytest.mark.gpu

N_CASES = 60
TOKEN_COUNTS = [1, 2, 7, 31, 33, 63, 64, 65, 127, 255, 256, 257, 300, 511, 513, 777, 1023, 1024, 1025, 1500, 2049, 3000]


def _i(t):
    return t.cpu().numpy()


def _random_cfg(rng, idx):
    dtype = "bf16" if rng.random() < 0.75 else "fp32"
    R = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
    per = int(rng.choice([1, 2, 3, 4, 8]))
    E = R * per
    n_red = min(per, int(rng.choice([0, 1, 1, 2])))
    k = int(rng.integers(1, min(E, 8) + 1))
    n_group = int(rng.choice([g for g in (1, 2, 4, 8) if E % g == 0]))
    topk_group = int(rng.integers(1, n_group + 1))
    if dtype == "bf16":
        H, I, I_s = 64 * int(rng.integers(1, 9)), 64 * int(rng.integers(1, 7)), 64 * int(rng.integers(0, 5))
    else:
        H, I, I_s = 8 * int(rng.integers(1, 33)), 4 * int(rng.integers(1, 49)), 4 * int(rng.integers(0, 33))
    n_fail = int(rng.integers(0, max(1, R // 2) + 1)) if R > 1 else 0
    failed = tuple(sorted(int(r) for r in rng.choice(R, size=n_fail, replace=False)))
    return synth.LayerConfig(f"random{idx}", T=int(rng.choice(TOKEN_COUNTS)), H=H, E=E, k=k, I=I, I_shared=I_s,
                             n_ranks=R, slots_per_rank=per + n_red, max_replicas=1 + n_red,
                             score_fn=str(rng.choice(["softmax", "sigmoid"])), n_group=n_group, topk_group=topk_group,
                             dtype=dtype, failed_ranks=failed, n_unprotected=-1, seed=int(rng.integers(0, 1000)),
                             router_skew=float(rng.choice([0.0, 0.0, 0.4, 0.8])))


def _usable(cfg):
    m = orc.build_map(synth.make_placement(cfg), synth.failed_mask(cfg), cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    return orc.enough_live_experts(m.l2p_count, cfg.k, cfg.n_group, cfg.topk_group)


def test_random_configurations_match_the_oracle():
    rng = np.random.default_rng(2024)
    ran = 0
    idx = 0
    while ran < N_CASES:
        cfg = _random_cfg(rng, idx)
        idx += 1
        if not _usable(cfg):
            continue
        print(f"case {ran}: {cfg}", flush=True)
        g = GpuLayer(cfg)
        try:
            r = g.forward()
            torch.cuda.synchronize()
            experts = {e: g.expert_f64(e) for e in range(cfg.E)}
            tr = orc.layer_staged(f64(g.x), None, experts, g.shared_f64(), g.p2l, g.oracle_map(), cfg.k, cfg.score_fn,
                                  cfg.n_group, cfg.topk_group, logits=f64(r["logits"]))
            assert rel_err(f64(r["logits"]), orc.router_logits(f64(g.x), f64(g.w_router))) < 1e-5, cfg
            for name, ref in (("topk_logical", tr.topk_logical), ("topk_phys", tr.topk_phys),
                              ("slot_offsets", tr.slot_offsets), ("dst_row", tr.dst_row), ("src_of", tr.src_of)):
                assert np.array_equal(_i(r[name]), ref), (name, cfg)
            assert np.array_equal(f64(r["x_perm"]), tr.x_perm), cfg
            tol = TOL[cfg.dtype]
            assert rel_err(f64(r["y_perm"]), tr.y_perm) < tol, cfg
            assert rel_err(f64(r["out"]), tr.out) < tol, cfg
            if tr.y_shared is not None:
                assert rel_err(f64(r["y_shared"]), tr.y_shared) < tol, cfg
        finally:
            g.close()
        ran += 1
