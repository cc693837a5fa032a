"""GPU tests of what follows the hot path in the paper: a failed rank's slots coming back
(Sec. 3.4 "Role switch", Sec. 4.3) and the lost-expert study's masks and activation counts (Sec. 4.2)."""
import numpy as np
import pytest
import torch

import synth
from oracle import revive_oracle as orc
from harness import GpuLayer, TOL, f64, rel_err

pytestmark = pytest.mark.gpu

CFG = synth.scaled(synth.get_config("c4"), T=900, H=512, I=256, I_shared=256)


def _i(t):
    return t.cpu().numpy()


def _experts_f64(g):
    return {e: g.expert_f64(e) for e in range(g.cfg.E)}


def test_failed_rank_is_never_read_and_comes_back():
    """While a rank is failed its weights may be garbage (the device is lost) and must not be
    touched; after new weights have been written in the background and the rank is un-failed,
    the masked experts return and the output is the unfailed layer's."""
    cfg = CFG
    g = GpuLayer(cfg, failed=[])
    try:
        experts = _experts_f64(g)
        base = orc.layer_staged(f64(g.x), f64(g.w_router), experts, g.shared_f64(), g.p2l, g.oracle_map(), cfg.k,
                                cfg.score_fn, cfg.n_group, cfg.topk_group)
        S = cfg.slots_per_rank
        lost_slots = [p for r in cfg.failed_ranks for p in range(r * S, (r + 1) * S)]
        saved = {p: (g.gu[p].clone(), g.dn[p].clone()) for p in lost_slots}
        stats = g.set_failed(cfg.failed_ranks)
        assert stats["n_lost_experts"] == 5
        for p in lost_slots:                     # the failed devices' memory is gone
            g.gu[p].fill_(float("nan"))
            g.dn[p].fill_(float("nan"))
        r = g.forward()
        out_failed = r["out"].clone()
        assert torch.isfinite(out_failed.float()).all()
        tr = orc.layer_staged(f64(g.x), None, experts, g.shared_f64(), g.p2l, g.oracle_map(), cfg.k, cfg.score_fn,
                              cfg.n_group, cfg.topk_group, logits=f64(r["logits"]))
        assert np.array_equal(_i(r["topk_phys"]), tr.topk_phys)
        assert rel_err(f64(out_failed), tr.out) < TOL[cfg.dtype]
        # role switch: replacement weights arrive on a side stream while the layer keeps serving
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for p in lost_slots:
                g.gu[p].copy_(saved[p][0], non_blocking=True)
                g.dn[p].copy_(saved[p][1], non_blocking=True)
        r = g.forward()                          # still under the failure map: unaffected by the copies
        assert torch.equal(r["out"], out_failed)
        side.synchronize()
        stats = g.set_failed([])
        assert stats["n_lost_experts"] == 0 and stats["n_live_slots"] == cfg.P
        r = g.forward()
        assert np.array_equal(_i(r["topk_logical"]), orc.select_topk(
            orc.masked_selection_scores(orc.scores(f64(r["logits"]), cfg.score_fn), g.oracle_map().l2p_count),
            cfg.k, cfg.n_group, cfg.topk_group))
        assert rel_err(f64(r["out"]), base.out) < TOL[cfg.dtype]
    finally:
        g.close()


@pytest.mark.parametrize("n", [2, 4, 32])
def test_every_nth_masks_on_the_gpu(n):
    import paper_2602_21140_amd as pk
    cfg = CFG
    g = GpuLayer(cfg, failed=[], with_weights=False)
    try:
        mask = pk.mask_every_nth(cfg.E, n)
        assert np.array_equal(mask, orc.every_nth_mask(cfg.E, n))
        stats = g.set_failed([], expert_failed=mask)
        assert stats["n_lost_experts"] == cfg.E // n
        logits = synth.draw_logits(cfg, g.device)
        _, top_l, top_w, top_p = g.layer.route(None, None, cfg.T, logits=logits, logits_given=True)
        m = g.oracle_map()
        s = orc.scores(f64(logits), cfg.score_fn)
        ref = orc.select_topk(orc.masked_selection_scores(s, m.l2p_count), cfg.k, cfg.n_group, cfg.topk_group)
        assert np.array_equal(_i(top_l), ref)
        assert np.array_equal(_i(top_p), orc.remap(ref, m))
        assert not mask[_i(top_l)].any()
        if n == 2:
            assert np.all(_i(top_l) % 2 == 1)    # Sec. 4.2: every even-indexed expert has failed
    finally:
        g.close()


def test_task_based_mask_from_gpu_activation_counts():
    import paper_2602_21140_amd as pk
    cfg = CFG
    g = GpuLayer(cfg, failed=[], with_weights=False)
    try:
        L = g.layer
        counts = torch.zeros(cfg.E, dtype=torch.int64, device=g.device)
        ref_counts = np.zeros(cfg.E, dtype=np.int64)
        for layer in range(3):                   # "aggregate the counts across layers"
            logits = synth.draw_logits(synth.scaled(cfg, seed=layer + 1), g.device)
            _, top_l, _, _ = L.route(None, None, cfg.T, logits=logits, logits_given=True)
            L.expert_counts(top_l, cfg.T, counts=counts)
            ref_counts += orc.activation_counts(_i(top_l), cfg.E)
        assert np.array_equal(_i(counts), ref_counts) and ref_counts.sum() == 3 * cfg.T * cfg.k
        for frac in (64, 32, 8):
            n_fail = cfg.E // frac
            mask = pk.mask_most_activated(_i(counts), n_fail)
            assert np.array_equal(mask, orc.most_activated_mask(ref_counts, n_fail))
            stats = g.set_failed([], expert_failed=mask)
            assert stats["n_lost_experts"] == n_fail
            logits = synth.draw_logits(cfg, g.device)
            _, top_l, top_w, _ = L.route(None, None, cfg.T, logits=logits, logits_given=True)
            assert not mask[_i(top_l)].any()
            assert np.abs(f64(top_w).sum(axis=1) - 1).max() < 1e-6
    finally:
        g.close()


def test_dense_ffn_group_rebalancing_on_the_gpu():
    """Sec. 3.4, dense FFN layers: one FFN replicated over G groups; when groups are compromised
    the tokens are spread evenly over the healthy ones.  Through the same map: one logical expert,
    one replica per group, k = 1, replica t mod (healthy groups)."""
    import paper_2602_21140_amd as pk
    G, T, H, I = 6, 1000, 512, 320
    cfg = synth.LayerConfig("dense_groups", T=T, H=H, E=1, k=1, I=I, I_shared=0, n_ranks=G, slots_per_rank=1,
                            max_replicas=G, score_fn="softmax", n_group=1, topk_group=1, dtype="bf16", failed_ranks=(1, 4))
    L = pk.ReviveLayer(cfg)
    try:
        p2l = np.zeros(G, dtype=np.int32)
        L.set_placement(p2l)
        failed = synth.failed_mask(cfg)
        stats = L.update_map(failed)
        assert stats["n_live_slots"] == 4 and stats["n_lost_experts"] == 0
        x = synth.draw_x(cfg, "cuda:0")
        w_r = pk.pack_router(synth.draw_router(cfg, "cuda:0"))
        w = synth.draw_expert(cfg, 0, "cuda:0")
        gu, dn = pk.pack_expert(w["gate"], w["up"], w["down"])
        nan = torch.full_like(gu, float("nan")), torch.full_like(dn, float("nan"))
        gus = [gu.clone() if not failed[p] else nan[0] for p in range(G)]
        dns = [dn.clone() if not failed[p] else nan[1] for p in range(G)]
        L.set_expert_weights(gus, dns)
        lg, top_l, top_w, top_p = L.route(x, w_r, T)
        x_perm, offs, dst, src = L.dispatch(x, top_p, T)
        y_perm, _ = L.expert_ffn(x_perm, offs, T, shared=False)
        out = L.combine(y_perm, dst, top_w, None, T)
        m = orc.build_map(p2l, failed, 1, 1, G)
        assert np.array_equal(_i(top_p).ravel(), m.l2p_table[0, np.arange(T) % 4])
        counts = np.diff(_i(offs))
        assert counts.tolist() == [250, 0, 250, 250, 0, 250]
        ref = orc.swiglu_ffn(f64(x), f64(w["gate"]), f64(w["up"]), f64(w["down"]))
        assert rel_err(f64(out), ref) < TOL["bf16"]
    finally:
        L.close()


def test_empty_slots_are_never_routed_to_and_can_be_filled_later():
    """A slot that holds no expert (placement -1: spare capacity for a later role switch, Sec. 3.4)
    takes no rows and its weight pointers are never followed; once weights are written into it and
    the placement names it, it serves as one more replica."""
    cfg = synth.scaled(synth.get_config("c2"), T=1100, H=512, I=320, I_shared=192, E=16, k=4, n_ranks=4,
                       slots_per_rank=6, max_replicas=3, failed_ranks=(1,), n_unprotected=-1)
    g = GpuLayer(cfg)
    try:
        S = cfg.slots_per_rank
        spare = [r * S + S - 1 for r in range(cfg.n_ranks)]          # last (redundant) slot of every rank
        held = {p: int(g.p2l[p]) for p in spare}
        p2l = g.p2l.copy()
        p2l[spare] = -1
        saved = {p: (g.gu[p].clone(), g.dn[p].clone()) for p in spare}
        for p in spare:
            g.gu[p].fill_(float("nan"))
            g.dn[p].fill_(float("nan"))
        g.layer.set_placement(p2l)
        g.p2l = p2l
        g.set_failed(cfg.failed_ranks)
        experts = {e: g.expert_f64(e) for e in range(cfg.E)}
        r = g.forward()
        tr = orc.layer_staged(f64(g.x), None, experts, g.shared_f64(), g.p2l, g.oracle_map(), cfg.k, cfg.score_fn,
                              cfg.n_group, cfg.topk_group, logits=f64(r["logits"]))
        assert np.array_equal(_i(r["topk_phys"]), tr.topk_phys)
        assert not np.isin(_i(r["topk_phys"]), spare).any()
        offs = _i(r["slot_offsets"])
        assert all(offs[p + 1] == offs[p] for p in spare)
        assert torch.isfinite(r["out"].float()).all()
        assert rel_err(f64(r["out"]), tr.out) < TOL[cfg.dtype]
        # fill the spare slots of the surviving ranks again and name them in the placement
        for p in spare:
            g.gu[p].copy_(saved[p][0])
            g.dn[p].copy_(saved[p][1])
        torch.cuda.synchronize()
        p2l = g.p2l.copy()
        for p in spare:
            p2l[p] = held[p]
        g.layer.set_placement(p2l)
        g.p2l = p2l
        g.set_failed(cfg.failed_ranks)
        r = g.forward()
        tr = orc.layer_staged(f64(g.x), None, experts, g.shared_f64(), g.p2l, g.oracle_map(), cfg.k, cfg.score_fn,
                              cfg.n_group, cfg.topk_group, logits=f64(r["logits"]))
        assert np.array_equal(_i(r["topk_phys"]), tr.topk_phys)
        live_spares = [p for p in spare if p // S not in cfg.failed_ranks]
        assert np.isin(_i(r["topk_phys"]), live_spares).any()
        assert rel_err(f64(r["out"]), tr.out) < TOL[cfg.dtype]
    finally:
        g.close()


def _golden_route_cases():
    import os
    from fractions import Fraction
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_route.txt")
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, fn, shape, ratios, masked, ids, weights = [f.strip() for f in line.split("|")]
        n_group, topk_group, k = (int(v) for v in shape.split())
        yield (name, fn, n_group, topk_group, k, [float(v) for v in ratios.split()],
               [] if masked == "-" else [int(v) for v in masked.split()],
               [int(v) for v in ids.split()], [float(Fraction(v)) for v in weights.split()])


@pytest.mark.parametrize("case", list(_golden_route_cases()), ids=lambda c: c[0])
def test_hand_worked_gating_examples_on_the_gpu(case):
    """The routing kernel against tests/golden/tiny_route.txt (values worked out by hand, no oracle in
    between): scores, mask before top-k, next-best experts, group-limited selection, weights."""
    name, fn, n_group, topk_group, k, ratios, masked, ids, weights = case
    E = len(ratios)
    cfg = synth.LayerConfig(name, T=3, H=64, E=E, k=k, I=64, I_shared=0, n_ranks=1, slots_per_rank=E, max_replicas=1,
                            score_fn=fn, n_group=n_group, topk_group=topk_group, dtype="fp32", failed_ranks=())
    g = GpuLayer(cfg, with_weights=False)
    try:
        ef = np.zeros(E, dtype=np.uint8)
        ef[masked] = 1
        g.set_failed([], expert_failed=ef)
        logits = torch.log(torch.tensor([ratios] * cfg.T, dtype=torch.float64)).to(torch.float32).to(g.device)
        _, top_l, top_w, top_p = g.layer.route(None, None, cfg.T, logits=logits, logits_given=True)
        for t in range(cfg.T):
            assert top_l[t].cpu().tolist() == ids
            assert top_p[t].cpu().tolist() == ids          # one slot per expert, slot id = expert id
            assert np.allclose(top_w[t].cpu().numpy(), weights, rtol=0, atol=2e-6)
    finally:
        g.close()


def test_hand_worked_dispatch_example_on_the_gpu():
    """The dispatch kernels against tests/golden/tiny_dispatch.txt (worked out by hand)."""
    import os
    rows = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "tiny_dispatch.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            key, rest = line.split(None, 1)
            rows[key] = rest
    phys = np.array([[int(v) for v in tok.split()] for tok in rows["topk_phys"].split("|")], dtype=np.int32)
    cfg = synth.LayerConfig("tiny_dispatch", T=4, H=64, E=5, k=2, I=64, I_shared=0, n_ranks=5, slots_per_rank=1,
                            max_replicas=1, score_fn="softmax", n_group=1, topk_group=1, dtype="fp32", failed_ranks=())
    g = GpuLayer(cfg, with_weights=False)
    try:
        x_perm, offs, dst, src = g.layer.dispatch(g.x, torch.from_numpy(phys).to(g.device), cfg.T)
        assert offs.cpu().tolist() == [int(v) for v in rows["slot_offsets"].split()]
        assert src.cpu().tolist() == [int(v) for v in rows["src_of"].split()]
        assert dst.cpu().tolist() == [int(v) for v in rows["dst_row"].split()]
        assert torch.equal(x_perm, g.x[torch.tensor([int(v) // cfg.k for v in rows["src_of"].split()], device=g.device)])
    finally:
        g.close()
