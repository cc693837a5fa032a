"""Pins for the oracle's lost-expert study helpers (Sec. 4.2 of the paper)."""
import numpy as np
import pytest

import synth
from oracle import revive_oracle as orc


def test_every_nth_examples():
    # the paper's example: r = 1/2 fails every even-indexed expert
    assert orc.every_nth_mask(8, 2).tolist() == [1, 0, 1, 0, 1, 0, 1, 0]
    assert orc.every_nth_mask(8, 4).tolist() == [1, 0, 0, 0, 1, 0, 0, 0]
    assert orc.every_nth_mask(6, 1).tolist() == [1] * 6
    for n in (2, 4, 8, 16, 32, 64):
        m = orc.every_nth_mask(256, n)
        assert m.sum() * n == 256                      # exactly the target fraction 1/n
        assert np.all(np.diff(np.nonzero(m)[0]) == n)  # a constant step


def test_every_nth_half_routes_only_to_odd_experts():
    cfg = synth.get_config("c1")
    p2l = synth.make_placement(cfg)
    mask = orc.every_nth_mask(cfg.E, 2)
    m = orc.build_map(p2l, synth.failed_mask(cfg, []), cfg.slots_per_rank, cfg.E, cfg.max_replicas, expert_failed=mask)
    assert m.n_lost_experts == cfg.E // 2
    assert np.array_equal(m.l2p_count > 0, mask == 0)
    assert not m.slot_alive[np.isin(p2l, np.nonzero(mask)[0])].any()
    s = orc.scores(synth.draw_logits(cfg).numpy(), "softmax")
    top = orc.select_topk(orc.masked_selection_scores(s, m.l2p_count), cfg.k)
    assert np.all(top % 2 == 1)


def test_expert_and_rank_failures_compose():
    cfg = synth.get_config("c1")
    p2l = synth.make_placement(cfg)
    mask = np.zeros(cfg.E, np.uint8)
    mask[[0, 8]] = 1
    both = orc.build_map(p2l, synth.failed_mask(cfg), cfg.slots_per_rank, cfg.E, cfg.max_replicas, expert_failed=mask)
    ranks_only = orc.build_map(p2l, synth.failed_mask(cfg), cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    assert both.l2p_count[0] == 0 and both.l2p_count[8] == 0
    keep = np.ones(cfg.E, bool)
    keep[[0, 8]] = False
    assert np.array_equal(both.l2p_count[keep], ranks_only.l2p_count[keep])
    assert np.array_equal(both.l2p_table[keep], ranks_only.l2p_table[keep])
    assert both.n_lost_experts == ranks_only.n_lost_experts + 2


def test_activation_counts_match_bincount():
    r = np.random.default_rng(0)
    top = r.integers(0, 37, size=(500, 6))
    c = orc.activation_counts(top, 37)
    assert c.sum() == top.size
    assert np.array_equal(c, np.bincount(top.ravel(), minlength=37))
    assert orc.activation_counts(np.zeros((0, 4), np.int32), 5).tolist() == [0] * 5


def test_most_activated_mask_properties():
    counts = np.array([5, 9, 9, 1, 0, 9, 3, 5])
    assert orc.most_activated_mask(counts, 0).sum() == 0
    assert orc.most_activated_mask(counts, 2).tolist() == [0, 1, 1, 0, 0, 0, 0, 0]      # tie of three 9s: lower ids
    assert orc.most_activated_mask(counts, 4).tolist() == [1, 1, 1, 0, 0, 1, 0, 0]      # then the first 5
    r = np.random.default_rng(1)
    for _ in range(20):
        c = r.integers(0, 6, size=24)
        n = int(r.integers(0, 25))
        m = orc.most_activated_mask(c, n)
        assert m.sum() == n
        if 0 < n < 24:
            assert c[m == 1].min() >= c[m == 0].max()   # no survivor is more activated than a failed expert
            # brute force: the lexicographically first set among those with the largest total count
            worst_in = c[m == 1].min()
            tied_in = [e for e in range(24) if m[e] and c[e] == worst_in]
            tied_out = [e for e in range(24) if not m[e] and c[e] == worst_in]
            assert not tied_out or max(tied_in) < min(tied_out)


def test_rank_compaction_follows_the_papers_description():
    """Sec. 3.5: device B with rank l_A + 1 takes l_A and later ranks are decremented; with a role
    switch device C takes l_A and any gap left behind is closed the same way."""
    assert orc.compact_ranks([0, 1, 2, 3, 4], 2) == [0, 1, -1, 2, 3]
    assert orc.compact_ranks([0, 1, 2, 3, 4], 4) == [0, 1, 2, 3, -1]
    assert orc.compact_ranks([0, 1, 2, 3, 4], 0) == [-1, 0, 1, 2, 3]
    # a device from outside the domain (an attention device) is switched in: nobody else moves
    assert orc.compact_ranks([0, 1, 2, 3, -1], 1, 4) == [0, -1, 2, 3, 1]
    # a device of the domain is switched: it takes the hole, the hole it leaves is closed
    assert orc.compact_ranks([0, 1, 2, 3, 4], 2, 4) == [0, 1, -1, 3, 2]
    assert orc.compact_ranks([0, 1, 2, 3, 4], 3, 0) == [2, 0, 1, -1, 3]
    r = np.random.default_rng(4)
    for _ in range(50):
        n = int(r.integers(2, 12))
        ranks = list(r.permutation(n))
        out_of_domain = r.random(n) < 0.2
        live = [d for d in range(n) if not out_of_domain[d]]
        if len(live) < 2:
            continue
        ranks = [-1] * n
        for i, d in enumerate(r.permutation(live)):
            ranks[d] = i
        f = int(r.choice(live))
        sw = int(r.integers(-1, n))
        if sw == f:
            sw = -1
        new = orc.compact_ranks(ranks, f, sw)
        members = [d for d in range(n) if new[d] >= 0]
        assert sorted(new[d] for d in members) == list(range(len(members)))     # compact: 0..m-1
        assert new[f] == -1
        others = [d for d in members if d != sw]
        assert sorted(others, key=lambda d: ranks[d]) == sorted(others, key=lambda d: new[d])   # order kept
        if sw >= 0 and ranks[sw] < 0:
            assert new[sw] == ranks[f] and all(new[d] == ranks[d] for d in others)


def test_compacted_rank_offsets_by_hand():
    """Sec. 3.5: after compaction the failed ranks are no part of the layout.  Four devices with
    two slots each, rows per slot 3,1 | 0,0 | 2,2 | 5,0; device 1 failed (it holds no rows)."""
    offs = [0, 3, 4, 4, 4, 6, 8, 13, 13]
    assert orc.compacted_rank_offsets(offs, [0, -1, 1, 2], 2) == [0, 4, 8, 13, 13]
    # nobody failed: the plain rank boundaries
    offs_all = [0, 3, 4, 5, 5, 7, 9, 14, 14]
    assert orc.compacted_rank_offsets(offs_all, [0, 1, 2, 3], 2) == [0, 4, 5, 9, 14]
    # a switched-in device that took logical rank 1 while physically sitting last
    assert orc.compacted_rank_offsets(offs, [0, -1, 2, 1], 2) == [0, 8, 4, 13, 13]
    with pytest.raises(AssertionError):
        orc.compacted_rank_offsets(offs_all, [0, -1, 1, 2], 2)      # a device outside the domain holding rows


def test_removing_failed_ranks_one_at_a_time_gives_the_same_table_in_any_order():
    r = np.random.default_rng(9)
    for _ in range(30):
        R = int(r.integers(2, 20))
        failed = [int(d) for d in r.choice(R, size=int(r.integers(0, R)), replace=False)]
        ranks = list(range(R))
        for f in failed:
            ranks = orc.compact_ranks(ranks, f)
        again = list(range(R))
        for f in sorted(failed):
            again = orc.compact_ranks(again, f)
        assert ranks == again
        live = [d for d in range(R) if d not in failed]
        assert [ranks[d] for d in live] == list(range(len(live))) and all(ranks[f] == -1 for f in failed)


def _golden_compaction():
    import os
    vals = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "rank_compaction.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *rest = line.split()
        vals[key] = [int(v) for v in rest]
    return vals


def test_hand_worked_rank_compaction():
    """tests/golden/rank_compaction.txt against the oracle and against the library's host code."""
    g = _golden_compaction()
    failed = g["rank_failed"]
    ranks = list(range(len(failed)))
    for d in (1, 4):                                   # in the order the fixture describes
        ranks = orc.compact_ranks(ranks, d)
    assert ranks == g["logical_rank"] and sum(r >= 0 for r in ranks) == g["n_live"][0]
    assert orc.compacted_rank_offsets(g["slot_offsets"], g["logical_rank"], 2) == g["rank_offsets"]
    import paper_2602_21140_amd as pk
    step = pk.compact_ranks(list(range(len(failed))), 1)
    assert pk.compact_ranks(step, 4).tolist() == g["logical_rank"]
