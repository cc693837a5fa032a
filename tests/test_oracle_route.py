"""Pins for the oracle's scores, masked (grouped) top-k, weights and remap."""
import itertools

import numpy as np
import pytest

import synth
from oracle import revive_oracle as orc


def _rng(seed):
    return np.random.default_rng(seed)


def _brute_topk(row, k):
    """Best k-subset by total score; ties by lexicographically smallest sorted id tuple."""
    live = [e for e in range(len(row)) if np.isfinite(row[e])]
    best, best_key = None, None
    for sub in itertools.combinations(live, k):
        key = (-sum(row[e] for e in sub), sub)
        if best_key is None or key < best_key:
            best, best_key = sub, key
    return set(best)


@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force_ungrouped(seed):
    r = _rng(seed)
    T, E = 4, 8
    for k in (1, 2, 3):
        logits = np.round(r.normal(size=(T, E)), 1)      # coarse values: ties do occur
        count = (r.random(E) < 0.7).astype(np.int32)
        if count.sum() < k:
            count[:k] = 1
        for fn in ("softmax", "sigmoid"):
            s = orc.scores(logits, fn)
            sel = orc.masked_selection_scores(s, count)
            top = orc.select_topk(sel, k)
            for t in range(T):
                # distinct-sum brute force is only unambiguous without exact ties in the row
                assert set(top[t]) .isdisjoint(np.nonzero(count == 0)[0])   # Sec. 3.4: never a missing expert
                vals = sel[t][top[t]]
                assert np.all(np.diff(vals) <= 0)
                if len(np.unique(sel[t][np.isfinite(sel[t])])) == int(count.sum()):
                    assert set(top[t]) == _brute_topk(sel[t], k)


def test_topk_is_topk_of_live_subvector():
    """Sec. 3.4: the next-best experts take the place of the masked ones."""
    r = _rng(1)
    T, E, k = 32, 24, 4
    logits = r.normal(size=(T, E))
    count = np.ones(E, np.int32)
    count[[0, 5, 6, 17, 23]] = 0
    s = orc.scores(logits, "softmax")
    top = orc.select_topk(orc.masked_selection_scores(s, count), k)
    live = np.nonzero(count)[0]
    for t in range(T):
        sub = np.argsort(-logits[t, live], kind="stable")[:k]
        assert list(top[t]) == list(live[sub])


def test_no_mask_equals_argsort():
    r = _rng(2)
    logits = r.normal(size=(50, 64))
    s = orc.scores(logits, "softmax")
    top = orc.select_topk(orc.masked_selection_scores(s, np.ones(64, np.int32)), 6)
    ref = np.argsort(-s, axis=1, kind="stable")[:, :6]
    assert np.array_equal(top, ref)


def test_every_nth_half_selects_only_odd():
    """Sec. 4.2: failing every even-indexed expert leaves only odd ids selectable."""
    r = _rng(3)
    E = 32
    count = np.ones(E, np.int32)
    count[0::2] = 0
    for fn, ng, tg in (("softmax", 1, 1), ("sigmoid", 4, 2)):
        s = orc.scores(r.normal(size=(40, E)), fn)
        top = orc.select_topk(orc.masked_selection_scores(s, count), 4, ng, tg)
        assert np.all(top % 2 == 1)


def test_all_equal_logits_pick_lowest_live_ids():
    E, k = 12, 3
    count = np.ones(E, np.int32)
    count[[0, 2]] = 0
    for fn in ("softmax", "sigmoid"):
        s = orc.scores(np.zeros((3, E)), fn)
        top = orc.select_topk(orc.masked_selection_scores(s, count), k)
        assert np.array_equal(top, np.tile([1, 3, 4], (3, 1)))
        w = orc.gate_weights(s, top)
        assert np.allclose(w, 1.0 / k, atol=1e-15)


def _brute_grouped(row, k, n_group, topk_group):
    E = len(row)
    gsz = E // n_group
    gs = []
    for g in range(n_group):
        part = sorted([v for v in row[g * gsz:(g + 1) * gsz] if np.isfinite(v)], reverse=True)
        gs.append(sum(part[:2]) if part else -np.inf)
    best, best_key = None, None
    for sub in itertools.combinations(range(n_group), topk_group):
        if any(not np.isfinite(gs[g]) for g in sub) and sum(np.isfinite(gs)) >= topk_group:
            continue
        key = (-sum(gs[g] for g in sub if np.isfinite(gs[g])), sub)
        if best_key is None or key < best_key:
            best, best_key = sub, key
    allowed = [e for g in best for e in range(g * gsz, (g + 1) * gsz)]
    masked = np.full(E, -np.inf)
    masked[allowed] = row[allowed]
    return set(best), _brute_topk(masked, k)


@pytest.mark.parametrize("seed", range(6))
def test_grouped_brute_force(seed):
    r = _rng(100 + seed)
    T, E, k, ng, tg = 4, 8, 2, 4, 2
    logits = r.normal(size=(T, E))
    count = (r.random(E) < 0.75).astype(np.int32)
    if not orc.enough_live_experts(count, k, ng, tg):
        count[:] = 1
    s = orc.scores(logits, "sigmoid")
    sel = orc.masked_selection_scores(s, count)
    top = orc.select_topk(sel, k, ng, tg)
    for t in range(T):
        groups, experts = _brute_grouped(sel[t], k, ng, tg)
        assert set(orc.kept_groups(sel[t], ng, tg)) == groups
        assert set(top[t]) == experts


def test_grouped_reductions():
    r = _rng(7)
    s = orc.scores(r.normal(size=(16, 32)), "sigmoid")
    sel = orc.masked_selection_scores(s, np.ones(32, np.int32))
    # one group, or keeping every group, is the ungrouped rule
    assert np.array_equal(orc.select_topk(sel, 4, 1, 1), orc.select_topk(sel, 4))
    assert np.array_equal(orc.select_topk(sel, 4, 8, 8), orc.select_topk(sel, 4))
    # group score: two best; one live -> that one; none -> -inf
    row = np.array([0.9, 0.2, 0.5, -np.inf, -np.inf, 0.3, -np.inf, -np.inf])
    assert np.allclose(orc.group_scores(row, 2)[0], 1.4) and np.allclose(orc.group_scores(row, 4), [1.1, 0.5, 0.3, -np.inf], equal_nan=False)
    assert list(orc.kept_groups(row, 4, 2)) == [0, 1]
    # a tie between groups goes to the lower group id
    tie = np.array([0.5, 0.25, 0.25, 0.5, 0.1, 0.1, 0.0, 0.0])
    assert list(orc.kept_groups(tie, 4, 1)) == [0]


def test_too_few_live_experts_is_an_error():
    s = orc.scores(np.zeros((1, 4)), "softmax")
    sel = orc.masked_selection_scores(s, np.array([1, 0, 0, 0]))
    with pytest.raises(AssertionError):
        orc.select_topk(sel, 2)


def test_weights_closed_forms():
    r = _rng(11)
    T, E, k = 20, 16, 3
    logits = r.normal(size=(T, E)) * 3
    count = np.ones(E, np.int32)
    count[[2, 9]] = 0
    s = orc.scores(logits, "softmax")
    top = orc.select_topk(orc.masked_selection_scores(s, count), k)
    w = orc.gate_weights(s, top)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-12)
    # renormalised softmax = softmax restricted to the selected logits
    picked = np.take_along_axis(logits, top.astype(np.int64), axis=1)
    ref = np.exp(picked - picked.max(axis=1, keepdims=True))
    ref /= ref.sum(axis=1, keepdims=True)
    assert np.allclose(w, ref, atol=1e-14)
    # masking the logits before the softmax gives the same set and weights
    ml = np.where(count[None, :] > 0, logits, -np.inf)
    s2 = orc.scores(ml, "softmax")
    top2 = orc.select_topk(np.where(count[None, :] > 0, s2, -np.inf), k)
    assert np.array_equal(top, top2)
    assert np.allclose(orc.gate_weights(s2, top2), w, atol=1e-14)
    # sigmoid: weights are the picked sigmoids over their sum; scale multiplies
    sg = orc.scores(logits, "sigmoid")
    assert np.allclose(sg, 0.5 * (1 + np.tanh(logits / 2)), atol=1e-15)
    tg = orc.select_topk(orc.masked_selection_scores(sg, count), k)
    wg = orc.gate_weights(sg, tg, route_scale=2.5)
    assert np.allclose(wg.sum(axis=1), 2.5, atol=1e-12)


def test_scores_textbook():
    z = np.array([[0.0, np.log(2.0), np.log(5.0)]])
    assert np.allclose(orc.scores(z, "softmax"), [[1 / 8, 2 / 8, 5 / 8]], atol=1e-15)
    assert np.allclose(orc.scores(np.array([[0.0, np.log(3.0)]]), "sigmoid"), [[0.5, 0.75]], atol=1e-15)


def test_remap_rule():
    cfg = synth.get_config("c1")
    p2l = synth.make_placement(cfg)
    m = orc.build_map(p2l, synth.failed_mask(cfg), cfg.slots_per_rank, cfg.E, cfg.max_replicas)
    top = np.array([[0, 8], [0, 8], [4, 12], [4, 12], [15, 1]], dtype=np.int32)
    phys = orc.remap(top, m)
    # two replicas: even token -> lower slot, odd token -> higher; one replica: the survivor
    assert phys.tolist() == [[0, 9], [19, 9], [4, 15], [5, 15], [18, 1]]
    assert np.all(m.slot_alive[phys] == 1) and np.array_equal(p2l[phys], top)
    with pytest.raises(AssertionError):
        orc.remap(np.array([[9, 0]], dtype=np.int32), m)


def test_router_logits_transposition_pin():
    x = np.array([[1.0, 2.0, 3.0]])
    w = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    assert orc.router_logits(x, w).tolist() == [[4.0, 5.0]]


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
def test_hand_worked_gating_examples(case):
    """tests/golden/tiny_route.txt: scores, mask before top-k, next-best experts, groups, weights."""
    name, fn, n_group, topk_group, k, ratios, masked, ids, weights = case
    logits = np.log(np.array([ratios]))
    count = np.ones(len(ratios), dtype=np.int32)
    count[masked] = 0
    s = orc.scores(logits, fn)
    top = orc.select_topk(orc.masked_selection_scores(s, count), k, n_group, topk_group)
    assert top[0].tolist() == ids
    assert np.allclose(orc.gate_weights(s, top)[0], weights, rtol=0, atol=1e-12)


def test_enough_live_experts_against_every_possible_ranking():
    """The sufficiency test of the map update is a worst case over all logits.  Brute force on 6
    experts in 3 groups: for every set of live experts and every (k, topk_group), a token can always
    be given k live experts exactly when no ranking of the experts' scores makes the selection run
    out of live experts (select_topk asserts when it does).  Scores 1..6 in every order reach every
    ranking of experts and of group sums that matters here."""
    import itertools
    E, n_group = 6, 3
    perms = np.array(list(itertools.permutations(range(1, E + 1))), dtype=np.float64)
    checked = refused = 0
    for bits in range(1, 1 << E):
        count = np.array([(bits >> e) & 1 for e in range(E)], dtype=np.int32)
        sel = orc.masked_selection_scores(perms, count)
        for topk_group in (1, 2, 3):
            for k in (1, 2, 3, 4):
                if k > (E // n_group) * topk_group:
                    continue                    # more experts than the kept groups hold at all: not a valid layer
                try:
                    top = orc.select_topk(sel, k, n_group, topk_group)
                    always = bool((count[top] > 0).all())
                except AssertionError:
                    always = False
                assert orc.enough_live_experts(count, k, n_group, topk_group) == always, (bits, k, topk_group)
                checked += 1
                refused += not always
    assert checked > 500 and 0 < refused < checked
    # ungrouped: plain count of live experts, against the same brute force
    for bits in range(1, 1 << E):
        count = np.array([(bits >> e) & 1 for e in range(E)], dtype=np.int32)
        sel = orc.masked_selection_scores(perms[:120], count)
        for k in (1, 2, 3, 6):
            try:
                orc.select_topk(sel, k)
                always = True
            except AssertionError:
                always = False
            assert orc.enough_live_experts(count, k, 1, 1) == always


def test_enough_live_experts_by_keepable_group_subsets():
    """8 experts in 4 groups, every live mask and every (k, topk_group): enumerate every set of
    groups the gate can end up keeping (any topk_group live groups; when fewer groups are live, all
    of them padded with dead ones) and ask whether each holds k live experts."""
    import itertools
    E, n_group, gsz = 8, 4, 2
    for bits in range(1 << E):
        live = np.array([(bits >> e) & 1 for e in range(E)], dtype=np.int32)
        per_group = live.reshape(n_group, gsz).sum(axis=1)
        live_groups = [g for g in range(n_group) if per_group[g] > 0]
        for topk_group in range(1, n_group + 1):
            if len(live_groups) >= topk_group:
                keepable = list(itertools.combinations(live_groups, topk_group))
            else:
                keepable = [tuple(live_groups)]          # the dead groups that pad the set add no expert
            worst = min(sum(per_group[g] for g in G) for G in keepable)
            for k in range(1, gsz * topk_group + 1):
                assert orc.enough_live_experts(live, k, n_group, topk_group) == (worst >= k), (bits, k, topk_group)
