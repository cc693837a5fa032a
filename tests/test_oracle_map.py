"""Pins for the oracle's map construction (Sec. 3.4 of the paper)."""
import os

import numpy as np
import pytest

import synth
from oracle import revive_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "c1_map.txt")


def _read_golden():
    lists, totals = {}, None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b = line.split(None, 1)
        if a == "totals":
            totals = [int(v) for v in b.split()]
        else:
            lists[int(a)] = [] if b == "-" else [int(v) for v in b.split(",")]
    return lists, totals


def test_c1_hand_worked_map():
    cfg = synth.get_config("c1")
    p2l = synth.make_placement(cfg)
    m = orc.build_map(p2l, synth.failed_mask(cfg), cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    lists, totals = _read_golden()
    for e in range(cfg.E):
        c = m.l2p_count[e]
        assert list(m.l2p_table[e, :c]) == lists[e]
        assert np.all(m.l2p_table[e, c:] == -1)
    assert [m.n_live_slots, m.n_live_experts, m.n_lost_experts, m.n_degraded_experts] == totals
    # a failed device is never touched: none of its slots is alive or listed
    assert not m.slot_alive[10:15].any()
    assert not np.isin(m.l2p_table, np.arange(10, 15)).any()


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_map_invariants(name):
    cfg = synth.get_config(name)
    p2l = synth.make_placement(cfg)
    none = orc.build_map(p2l, synth.failed_mask(cfg, []), cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    # no failure: the table is the full replica list of the placement
    for e in range(cfg.E):
        assert list(none.l2p_table[e, :none.l2p_count[e]]) == list(np.nonzero(p2l == e)[0])
    assert none.n_lost_experts == 0 and none.n_degraded_experts == 0 and none.n_live_slots == cfg.P
    m = orc.build_map(p2l, synth.failed_mask(cfg), cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    assert m.l2p_count.sum() == m.n_live_slots == cfg.P - len(cfg.failed_ranks) * cfg.slots_per_rank
    for e in range(cfg.E):
        on_failed = [p // cfg.slots_per_rank in cfg.failed_ranks for p in np.nonzero(p2l == e)[0]]
        assert (m.l2p_count[e] == 0) == all(on_failed)
        lst = m.l2p_table[e, :m.l2p_count[e]]
        assert np.all(np.diff(lst) > 0) and np.all(p2l[lst] == e) and np.all(m.slot_alive[lst] == 1)
    assert orc.enough_live_experts(m.l2p_count, cfg.k, cfg.n_group, cfg.topk_group)


def test_config_failure_outcomes():
    """The outcomes the workload recipes are engineered for."""
    want = {"c1": (3, 2), "c2": (1, 8), "c3": (0, 9), "c4": (5, None), "c5": (14, 4)}
    for name, (lost, degraded) in want.items():
        cfg = synth.get_config(name)
        m = orc.build_map(synth.make_placement(cfg), synth.failed_mask(cfg), cfg.slots_per_rank,
                          cfg.E, cfg.max_replicas)
        assert m.n_lost_experts == lost, name
        if degraded is not None:
            assert m.n_degraded_experts == degraded, name


def test_unreplicated_rank_failure_loses_one_over_R():
    """Sec. 4.2: with EP = R and no redundancy one failed device loses a 1/R fraction of the experts."""
    R, per = 8, 4
    p2l = np.arange(R * per, dtype=np.int32)
    failed = np.zeros(R, np.uint8)
    failed[5] = 1
    m = orc.build_map(p2l, failed, per, R * per, 1)
    assert m.n_lost_experts == per and m.n_live_experts == (R - 1) * per
    assert list(np.nonzero(m.l2p_count == 0)[0]) == [20, 21, 22, 23]


def test_empty_slots_and_bad_mask():
    p2l = np.array([0, -1, 1, 0], dtype=np.int32)
    m = orc.build_map(p2l, np.zeros(2, np.uint8), 2, 2, 2)
    assert list(m.l2p_count) == [2, 1] and list(m.slot_alive) == [1, 0, 1, 1]
    with pytest.raises(AssertionError):
        orc.build_map(p2l, np.array([0, 2], np.uint8), 2, 2, 2)


def test_enough_live_experts_grouped():
    # 4 groups of 2; keep 2 groups; k = 3
    assert orc.enough_live_experts(np.array([1, 1, 1, 1, 1, 1, 1, 1]), 3, 4, 2)
    # two groups with one live expert each could both be kept -> only 2 experts
    assert not orc.enough_live_experts(np.array([1, 0, 1, 0, 1, 1, 1, 1]), 3, 4, 2)
    # a dead group is never preferred to a live one: kept groups are live ones
    assert orc.enough_live_experts(np.array([0, 0, 1, 1, 1, 1, 1, 1]), 3, 4, 2)
    # fewer live groups than topk_group: all live groups are kept
    assert orc.enough_live_experts(np.array([0, 0, 0, 0, 0, 0, 1, 1]), 2, 4, 2)
    assert not orc.enough_live_experts(np.array([0, 0, 0, 0, 0, 0, 1, 1]), 3, 4, 2)
    assert not orc.enough_live_experts(np.array([1, 0, 0, 0]), 2, 1, 1)
