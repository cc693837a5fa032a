"""Pins for the oracle's expert FFN, combine and the whole layer."""
import numpy as np
import pytest
import torch

import synth
from oracle import revive_oracle as orc


def _np(t):
    return t.to(torch.float64).numpy()


def _tiny(score_fn="softmax", n_group=1, topk_group=1, I_shared=24, failed=(2,), seed=0):
    cfg = synth.scaled(synth.get_config("c1"), T=12, H=32, I=16, I_shared=I_shared, score_fn=score_fn,
                       n_group=n_group, topk_group=topk_group, failed_ranks=tuple(failed), seed=seed)
    x = _np(synth.draw_x(cfg))
    wr = _np(synth.draw_router(cfg))
    experts = {e: {n: _np(v) for n, v in synth.draw_expert(cfg, e).items()} for e in range(cfg.E)}
    sh = synth.draw_shared(cfg)
    shared = None if sh is None else {n: _np(v) for n, v in sh.items()}
    p2l = synth.make_placement(cfg)
    return cfg, x, wr, experts, shared, p2l


def _map(cfg, p2l, failed=None):
    return orc.build_map(p2l, synth.failed_mask(cfg, failed), cfg.slots_per_rank, cfg.E, cfg.max_replicas)


def test_swiglu_against_library():
    """One expert, one choice: the layer is a textbook SwiGLU MLP (torch's silu and matmul)."""
    r = np.random.default_rng(0)
    x, g, u, d = r.normal(size=(5, 8)), r.normal(size=(8, 6)), r.normal(size=(8, 6)), r.normal(size=(6, 8))
    ref = (torch.nn.functional.silu(torch.from_numpy(x) @ torch.from_numpy(g)) * (torch.from_numpy(x) @ torch.from_numpy(u))) @ torch.from_numpy(d)
    assert np.allclose(orc.swiglu_ffn(x, g, u, d), ref.numpy(), rtol=1e-13, atol=1e-13)
    experts = {0: {"gate": g, "up": u, "down": d}}
    out = orc.layer_definition(x, r.normal(size=(8, 1)), experts, None, np.array([1]), 1, "softmax")
    assert np.allclose(out, ref.numpy(), rtol=1e-13, atol=1e-13)
    tr = orc.layer_staged(x, r.normal(size=(8, 1)), experts, None, np.array([0]), _one_slot_map(), 1, "sigmoid")
    assert np.allclose(tr.out, ref.numpy(), rtol=1e-13, atol=1e-13)
    # silu pin: silu(0) = 0, silu(z) -> z for large z, silu(-z) = -z sigmoid(-z)
    assert orc.silu(np.array([0.0]))[0] == 0.0 and abs(orc.silu(np.array([40.0]))[0] - 40.0) < 1e-12
    assert np.isclose(orc.silu(np.array([-1.0]))[0], -1.0 / (1.0 + np.e))


def _one_slot_map():
    return orc.build_map(np.array([0], np.int32), np.zeros(1, np.uint8), 1, 1, 1)


def test_ffn_special_cases():
    r = np.random.default_rng(1)
    x, g, u, d = r.normal(size=(4, 8)), r.normal(size=(8, 6)), r.normal(size=(8, 6)), r.normal(size=(6, 8))
    assert np.all(orc.swiglu_ffn(x, g, u, np.zeros_like(d)) == 0)
    assert np.all(orc.swiglu_ffn(np.zeros_like(x), g, u, d) == 0)
    # gate and up are not interchangeable
    assert not np.allclose(orc.swiglu_ffn(x, g, u, d), orc.swiglu_ffn(x, u, g, d))
    # rows are independent: permuting the input rows permutes the output rows
    perm = np.array([2, 0, 3, 1])
    assert np.allclose(orc.swiglu_ffn(x[perm], g, u, d), orc.swiglu_ffn(x, g, u, d)[perm], atol=1e-14)


@pytest.mark.parametrize("score_fn,ng,tg", [("softmax", 1, 1), ("sigmoid", 4, 2), ("sigmoid", 1, 1)])
def test_staged_equals_dense_definition(score_fn, ng, tg):
    cfg, x, wr, experts, shared, p2l = _tiny(score_fn, ng, tg)
    m = _map(cfg, p2l)
    dense = orc.layer_definition(x, wr, experts, shared, m.l2p_count, cfg.k, score_fn, ng, tg)
    tr = orc.layer_staged(x, wr, experts, shared, p2l, m, cfg.k, score_fn, ng, tg)
    assert np.allclose(tr.out, dense, rtol=1e-12, atol=1e-12)
    assert np.allclose(tr.topk_weight.sum(axis=1), 1.0, atol=1e-12)
    assert np.abs(dense).max() > 0.01


def test_no_failure_equals_unfailed_layer_and_pure_remap_is_invisible():
    """Sec. 3.4: removing replicas changes only the map; as long as every expert keeps one
    replica the layer output is the unfailed layer's."""
    cfg, x, wr, experts, shared, p2l = _tiny(failed=())
    full = _map(cfg, p2l, [])
    base = orc.layer_staged(x, wr, experts, shared, p2l, full, cfg.k, cfg.score_fn)
    # unfailed layer written without any map: plain top-k over all experts
    plain = orc.layer_definition(x, wr, experts, shared, np.ones(cfg.E, np.int32), cfg.k, cfg.score_fn)
    assert np.allclose(base.out, plain, rtol=1e-12, atol=1e-12)
    # a placement where rank 2's four experts each have a copy elsewhere: pure remap
    cfg2 = synth.scaled(cfg, slots_per_rank=6, max_replicas=3, n_unprotected=0, failed_ranks=(2,))
    p2l2 = synth.make_placement(cfg2)
    m2 = _map(cfg2, p2l2)
    assert m2.n_lost_experts == 0 and m2.n_degraded_experts > 0
    before = orc.layer_staged(x, wr, experts, shared, p2l2, _map(cfg2, p2l2, []), cfg.k, cfg.score_fn)
    tr = orc.layer_staged(x, wr, experts, shared, p2l2, m2, cfg.k, cfg.score_fn)
    assert np.array_equal(tr.topk_logical, base.topk_logical)
    assert not np.array_equal(tr.topk_phys, before.topk_phys)
    assert np.allclose(tr.out, base.out, rtol=1e-12, atol=1e-12)
    S = cfg2.slots_per_rank
    assert np.diff(tr.slot_offsets)[2 * S:3 * S].sum() == 0


def test_masking_changes_output_only_through_lost_experts():
    cfg, x, wr, experts, shared, p2l = _tiny()
    full, m = _map(cfg, p2l, []), _map(cfg, p2l)
    a = orc.layer_staged(x, wr, experts, shared, p2l, full, cfg.k, cfg.score_fn)
    b = orc.layer_staged(x, wr, experts, shared, p2l, m, cfg.k, cfg.score_fn)
    lost = set(np.nonzero(m.l2p_count == 0)[0])
    hit = np.array([bool(lost & set(row)) for row in a.topk_logical])
    assert hit.any() and not hit.all()
    assert np.allclose(a.out[~hit], b.out[~hit], rtol=1e-12, atol=1e-12)
    assert not np.allclose(a.out[hit], b.out[hit], rtol=1e-6, atol=1e-6)
    assert not (set(b.topk_logical.ravel()) & lost)


def test_identical_experts_make_routing_irrelevant():
    cfg, x, wr, experts, shared, p2l = _tiny()
    same = {e: experts[0] for e in range(cfg.E)}
    m = _map(cfg, p2l)
    tr = orc.layer_staged(x, wr, same, None, p2l, m, cfg.k, cfg.score_fn)
    ref = orc.swiglu_ffn(x, experts[0]["gate"], experts[0]["up"], experts[0]["down"])
    assert np.allclose(tr.out, ref, rtol=1e-12, atol=1e-12)


def test_combine_by_hand():
    y = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, 2.0], [5.0, 7.0]])
    dst = np.array([2, 0, 3, 1], dtype=np.int32)           # token0 -> rows 2,0 ; token1 -> rows 3,1
    w = np.array([[0.25, 0.75], [0.5, 0.5]])
    sh = np.array([[10.0, 10.0], [0.0, 0.0]])
    out = orc.combine(y, dst, w, sh)
    assert np.allclose(out, [[0.25 * 2 + 0.75 * 1 + 10, 0.25 * 2 + 10], [2.5, 4.0]])
    assert np.allclose(orc.combine(y, dst, w, None), out - sh)


def test_supplied_logits_are_used():
    cfg, x, wr, experts, shared, p2l = _tiny()
    m = _map(cfg, p2l)
    lg = synth.draw_logits(cfg).numpy()
    tr = orc.layer_staged(x, wr, experts, shared, p2l, m, cfg.k, cfg.score_fn, logits=lg)
    s = orc.scores(lg, cfg.score_fn)
    assert np.array_equal(tr.topk_logical, orc.select_topk(orc.masked_selection_scores(s, m.l2p_count), cfg.k))


def test_selection_gap():
    row = np.array([0.5, 0.4, 0.4 + 1e-7, 0.1])
    assert orc.selection_gap(row, [0, 2], [0, 2]) == 0.0
    assert orc.selection_gap(row, [0, 2], [0, 1]) == pytest.approx(1e-7)
    assert orc.selection_gap(row, [0, 2], [0, 3]) > 0.29


def test_dense_ffn_group_rebalancing_is_the_same_remap():
    """Sec. 3.4 (last paragraph): a dense FFN replicated over several groups; tokens are spread
    evenly over the healthy groups.  One logical 'expert' with one replica per group, k = 1."""
    G, T, H, I = 6, 50, 16, 8
    r = np.random.default_rng(5)
    x = r.normal(size=(T, H))
    w = {"gate": r.normal(size=(H, I)), "up": r.normal(size=(H, I)), "down": r.normal(size=(I, H))}
    p2l = np.zeros(G, dtype=np.int32)
    failed = np.zeros(G, np.uint8)
    failed[[1, 4]] = 1
    m = orc.build_map(p2l, failed, 1, 1, G)
    assert m.l2p_table[0, :4].tolist() == [0, 2, 3, 5]
    tr = orc.layer_staged(x, r.normal(size=(H, 1)), {0: w}, None, p2l, m, 1, "softmax")
    counts = np.diff(tr.slot_offsets)
    assert counts[[1, 4]].sum() == 0 and counts[[0, 2, 3, 5]].max() - counts[[0, 2, 3, 5]].min() <= 1
    assert np.allclose(tr.topk_weight, 1.0)
    assert np.allclose(tr.out, orc.swiglu_ffn(x, w["gate"], w["up"], w["down"]), atol=1e-12)


def test_grouped_ffn_is_one_textbook_mlp_per_slot():
    """grouped_expert_ffn: the rows of slot p go through the expert slot p holds, nothing else;
    empty slots contribute nothing; rows keep their positions (row-order independence)."""
    rng = np.random.default_rng(5)
    H, I = 12, 7
    p2l = np.array([2, 0, 1, 0], dtype=np.int32)               # slot 3 is a second copy of expert 0
    experts = {e: {"gate": rng.standard_normal((H, I)), "up": rng.standard_normal((H, I)),
                   "down": rng.standard_normal((I, H))} for e in range(3)}
    offsets = np.array([0, 3, 3, 8, 10], dtype=np.int32)        # slot 1 is empty
    x = rng.standard_normal((10, H))
    y = orc.grouped_expert_ffn(x, offsets, p2l, experts)
    for p in range(4):
        a, b = offsets[p], offsets[p + 1]
        w = experts[int(p2l[p])]
        g, u = x[a:b] @ w["gate"], x[a:b] @ w["up"]
        ref = ((g / (1.0 + np.exp(-g))) * u) @ w["down"]         # SwiGLU written out with library matmuls
        assert np.allclose(y[a:b], ref, rtol=1e-12, atol=1e-12)
    # permuting the rows inside a slot permutes its outputs identically
    perm = np.array([2, 0, 1, 7, 3, 6, 4, 5, 9, 8])
    assert np.allclose(orc.grouped_expert_ffn(x[perm], offsets, p2l, experts), y[perm], rtol=1e-12, atol=1e-12)
    # a mistake that a plain reading would make: using the slot id as the expert id
    wrong = orc.grouped_expert_ffn(x, offsets, np.arange(4, dtype=np.int32) % 3, experts)
    assert not np.allclose(wrong[0:3], y[0:3])
