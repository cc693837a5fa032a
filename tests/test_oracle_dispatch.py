"""Pins for the oracle's dispatch indices and row permutation."""
import numpy as np
import pytest

import synth
from oracle import revive_oracle as orc


def _routing(name, T=None):
    cfg = synth.get_config(name)
    if T is not None:
        cfg = synth.scaled(cfg, T=T)
    p2l = synth.make_placement(cfg)
    m = orc.build_map(p2l, synth.failed_mask(cfg), cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    logits = synth.draw_logits(cfg).numpy()
    s = orc.scores(logits, cfg.score_fn)
    top = orc.select_topk(orc.masked_selection_scores(s, m.l2p_count), cfg.k, cfg.n_group, cfg.topk_group)
    return cfg, p2l, m, top, orc.remap(top, m)


@pytest.mark.parametrize("name,T", [("c1", None), ("c2", 300), ("c4", 200), ("c5", 150)])
def test_dispatch_invariants(name, T):
    cfg, p2l, m, top, phys = _routing(name, T)
    offsets, dst_row, src_of = orc.dispatch_indices(phys, cfg.P)
    N = cfg.T * cfg.k
    # every (token, choice) lands exactly once, on a surviving slot
    assert sorted(dst_row.tolist()) == list(range(N))
    assert np.array_equal(src_of[dst_row], np.arange(N))
    assert offsets[0] == 0 and offsets[-1] == N                      # per-slot counts sum to T*k
    counts = np.diff(offsets)
    assert np.array_equal(counts, np.bincount(phys.ravel(), minlength=cfg.P))
    S = cfg.slots_per_rank
    for r in cfg.failed_ranks:                                        # failed ranks receive nothing
        assert counts[r * S:(r + 1) * S].sum() == 0
    assert np.all(counts[m.slot_alive == 0] == 0)
    for p in range(cfg.P):                                            # stable inside a slot
        seg = src_of[offsets[p]:offsets[p + 1]]
        assert np.all(np.diff(seg) > 0)
        assert np.all(phys.ravel()[seg] == p)
    # library routine: a stable argsort by slot is the same permutation
    assert np.array_equal(src_of, np.argsort(phys.ravel(), kind="stable"))


def test_permute_rows_moves_exact_rows():
    cfg, p2l, m, top, phys = _routing("c1")
    x = synth.draw_x(cfg).numpy()
    offsets, dst_row, src_of = orc.dispatch_indices(phys, cfg.P)
    xp = orc.permute_rows(x, dst_row, cfg.k)
    for i in range(cfg.T * cfg.k):
        assert np.array_equal(xp[dst_row[i]], x[i // cfg.k])
    assert np.array_equal(xp, x[src_of // cfg.k])


def test_dispatch_tiny_by_hand():
    phys = np.array([[3, 1], [1, 3], [1, 0]], dtype=np.int32)
    offsets, dst_row, src_of = orc.dispatch_indices(phys, 5)
    assert offsets.tolist() == [0, 1, 4, 4, 6, 6]
    assert dst_row.tolist() == [4, 1, 2, 5, 3, 0]
    assert src_of.tolist() == [5, 1, 2, 4, 0, 3]


def test_dispatch_empty():
    offsets, dst_row, src_of = orc.dispatch_indices(np.zeros((0, 2), np.int32), 4)
    assert offsets.tolist() == [0] * 5 and dst_row.size == 0 and src_of.size == 0


def test_dispatch_indices_on_random_slot_lists():
    """Property check on many random inputs (any slot distribution, empty slots, one slot only):
    dst_row is the permutation of a stable sort by slot, src_of its inverse, offsets the exclusive
    scan of the counts; checked against a plain Python bucket fill."""
    rng = np.random.default_rng(9)
    for case in range(200):
        P = int(rng.integers(1, 40))
        T, k = int(rng.integers(0, 60)), int(rng.integers(1, 5))
        if case % 7 == 0:
            phys = np.full((T, k), int(rng.integers(0, P)), dtype=np.int32)      # everything on one slot
        else:
            phys = rng.integers(0, P, size=(T, k)).astype(np.int32)
        offsets, dst_row, src_of = orc.dispatch_indices(phys, P)
        buckets = [[] for _ in range(P)]
        for i, p in enumerate(phys.ravel().tolist()):
            buckets[p].append(i)
        flat = [i for b in buckets for i in b]
        assert src_of.tolist() == flat
        assert offsets.tolist() == np.concatenate([[0], np.cumsum([len(b) for b in buckets])]).tolist()
        inv = np.empty(T * k, dtype=np.int64)
        inv[np.array(flat, dtype=np.int64)] = np.arange(T * k)
        assert dst_row.tolist() == inv.tolist()


def test_hand_worked_dispatch_example():
    """tests/golden/tiny_dispatch.txt."""
    import os
    rows = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "tiny_dispatch.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            key, rest = line.split(None, 1)
            rows[key] = rest
    phys = np.array([[int(v) for v in tok.split()] for tok in rows["topk_phys"].split("|")], dtype=np.int32)
    offsets, dst_row, src_of = orc.dispatch_indices(phys, 5)
    assert offsets.tolist() == [int(v) for v in rows["slot_offsets"].split()]
    assert src_of.tolist() == [int(v) for v in rows["src_of"].split()]
    assert dst_row.tolist() == [int(v) for v in rows["dst_row"].split()]
