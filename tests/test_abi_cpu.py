"""CPU checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
map construction agrees bit for bit with the oracle.  No GPU call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

import synth
from oracle import revive_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _pk():
    import paper_2602_21140_amd as pk
    if not os.path.exists(pk.lib_path()):
        from paper_2602_21140_amd import build
        build.build(verbose=False)
    return pk


def _declared():
    text = open(os.path.join(ROOT, "include", "revive.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(revive_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    pk = _pk()
    L = pk.lib()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), f"{n} declared in revive.h but not exported"
    from paper_2602_21140_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_status_and_kernel_names():
    L = _pk().lib()
    assert L.revive_status_name(0) == b"REVIVE_OK" and L.revive_status_name(-4) == b"REVIVE_EINSUFFICIENT_EXPERTS"
    from paper_2602_21140_amd import binding
    for i, n in enumerate(binding.KERNEL_NAMES):
        assert L.revive_kernel_name(i).decode() == n


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_host_map_build_matches_oracle(name):
    pk = _pk()
    cfg = synth.get_config(name)
    p2l = synth.make_placement(cfg)
    rng = np.random.default_rng(5)
    cases = [synth.failed_mask(cfg), synth.failed_mask(cfg, [])]
    for _ in range(4):
        cases.append(synth.failed_mask(cfg, rng.choice(cfg.n_ranks, size=rng.integers(1, 3), replace=False)))
    for failed in cases:
        rc, table, count, alive, stats = pk.build_map_host(cfg, p2l, failed)
        m = orc.build_map(p2l, failed, cfg.slots_per_rank, cfg.E, cfg.max_replicas)
        ok = orc.enough_live_experts(m.l2p_count, cfg.k, cfg.n_group, cfg.topk_group)
        assert (rc == 0) == ok
        assert np.array_equal(table, m.l2p_table) and np.array_equal(count, m.l2p_count)
        assert np.array_equal(alive, m.slot_alive)
        assert stats == dict(n_live_slots=m.n_live_slots, n_live_experts=m.n_live_experts,
                             n_lost_experts=m.n_lost_experts, n_degraded_experts=m.n_degraded_experts)


def test_host_map_build_rejects_bad_input():
    pk = _pk()
    cfg = synth.get_config("c1")
    p2l = synth.make_placement(cfg)
    bad = synth.failed_mask(cfg)
    bad[0] = 2
    assert pk.build_map_host(cfg, p2l, bad)[0] == -1                      # byte not 0/1
    assert pk.build_map_host(cfg, p2l, np.ones(cfg.n_ranks, np.uint8))[0] == -4   # nothing left alive
    p2 = p2l.copy()
    p2[3] = cfg.E
    assert pk.build_map_host(cfg, p2, synth.failed_mask(cfg))[0] == -1    # expert id out of range
    p3 = p2l.copy()
    p3[:3] = 0
    assert pk.build_map_host(cfg, p3, synth.failed_mask(cfg))[0] == -1    # more copies than max_replicas
    # grouped sufficiency: 4 groups of 4, keep 2, k = 4; leave two groups with one live expert each
    g = synth.scaled(cfg, n_group=4, topk_group=2, k=4, score_fn="sigmoid", slots_per_rank=1, max_replicas=1,
                     n_ranks=16)
    pg = np.arange(16, dtype=np.int32)
    failed = np.zeros(16, np.uint8)
    failed[[1, 2, 3, 5, 6, 7]] = 1
    assert pk.build_map_host(g, pg, failed)[0] == -4
    failed[5] = 0
    assert pk.build_map_host(g, pg, failed)[0] == -4     # 1 + 2 < 4
    failed[[1, 2]] = 0
    assert pk.build_map_host(g, pg, failed)[0] == 0      # groups hold 3, 2, 4, 4: worst pair 2 + 3 >= 4


def test_mask_generators_match_oracle():
    pk = _pk()
    for E, n in ((8, 2), (256, 32), (384, 64), (10, 3), (6, 1)):
        assert np.array_equal(pk.mask_every_nth(E, n), orc.every_nth_mask(E, n))
    rng = np.random.default_rng(9)
    for _ in range(30):
        E = int(rng.integers(1, 60))
        counts = rng.integers(0, 5, size=E)          # many ties
        n_fail = int(rng.integers(0, E + 1))
        assert np.array_equal(pk.mask_most_activated(counts, n_fail), orc.most_activated_mask(counts, n_fail))


def test_host_map_build_with_failed_experts_matches_oracle():
    pk = _pk()
    rng = np.random.default_rng(11)
    for name in ("c1", "c3", "c5"):
        cfg = synth.get_config(name)
        p2l = synth.make_placement(cfg)
        for n in (2, 4, 64):
            if name == "c1" and n > 4:
                continue
            ef = orc.every_nth_mask(cfg.E, n)
            for failed in (synth.failed_mask(cfg, []), synth.failed_mask(cfg)):
                rc, table, count, alive, stats = pk.build_map_host(cfg, p2l, failed, expert_failed=ef)
                m = orc.build_map(p2l, failed, cfg.slots_per_rank, cfg.E, cfg.max_replicas, expert_failed=ef)
                assert (rc == 0) == orc.enough_live_experts(m.l2p_count, cfg.k, cfg.n_group, cfg.topk_group)
                assert np.array_equal(table, m.l2p_table) and np.array_equal(count, m.l2p_count)
                assert np.array_equal(alive, m.slot_alive) and stats["n_lost_experts"] == m.n_lost_experts
    bad = np.zeros(16, np.uint8)
    bad[3] = 7
    cfg = synth.get_config("c1")
    assert pk.build_map_host(cfg, synth.make_placement(cfg), synth.failed_mask(cfg, []), expert_failed=bad)[0] == -1


def test_compact_ranks_matches_oracle():
    pk = _pk()
    rng = np.random.default_rng(13)
    for _ in range(100):
        n = int(rng.integers(2, 16))
        live = [d for d in range(n) if rng.random() > 0.2]
        if len(live) < 2:
            continue
        ranks = [-1] * n
        for i, d in enumerate(rng.permutation(live)):
            ranks[d] = i
        f = int(rng.choice(live))
        sw = int(rng.integers(-1, n))
        if sw == f:
            sw = -1
        assert pk.compact_ranks(ranks, f, sw).tolist() == orc.compact_ranks(ranks, f, sw)
    with pytest.raises(pk.ReviveError):
        pk.compact_ranks([0, -1, 1], 1)


def test_library_sufficiency_test_over_every_live_mask():
    """The library's refusal (REVIVE_EINSUFFICIENT_EXPERTS) against the oracle's sufficiency test,
    itself pinned by brute force over rankings, for every set of live experts of an 8-expert layer in
    4 groups and every (k, topk_group)."""
    pk = _pk()
    base = synth.get_config("c1")
    p2l = np.arange(8, dtype=np.int32)
    none = np.zeros(8, np.uint8)
    for topk_group in (1, 2, 3, 4):
        for k in range(1, 2 * topk_group + 1):
            cfg = synth.scaled(base, E=8, k=k, n_group=4, topk_group=topk_group, n_ranks=8, slots_per_rank=1,
                               max_replicas=1, score_fn="sigmoid")
            for bits in range(1 << 8):
                ef = np.array([1 - ((bits >> e) & 1) for e in range(8)], dtype=np.uint8)
                rc, _t, count, _a, _s = pk.build_map_host(cfg, p2l, none, expert_failed=ef)
                assert rc in (0, -4)
                assert (rc == 0) == orc.enough_live_experts(count, k, 4, topk_group), (bits, k, topk_group)
