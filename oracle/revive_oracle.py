"""CPU oracle for the failure-remapped MoE layer (TEST INFRASTRUCTURE ONLY).

A plain, slow, fp64 numpy statement of what the layer computes after failed
expert ranks have been taken out of service.  It exists to check the GPU
library; it shares no code with it and nothing on the product path may call
it.  Parity status: every function below is pinned by the CPU tests
(brute-force enumeration on tiny inputs, closed forms, invariants and the
hand-worked placement example); nothing here is "parity unpinned".

What the paper fixes (ReviveMoE, arXiv 2602.21140):
  * Sec. 2.1: a gating function scores the experts per token, tokens go to
    their top-k experts, each expert is an FFN.
  * Sec. 2.3: dispatch routes tokens to their top-k experts using the gating
    scores; combine aggregates the expert outputs back, weighted by them.
  * Sec. 3.4 "Redundant experts": recovery removes the failed replicas from
    the logical-to-physical map; weights are untouched.
  * Sec. 3.4 "Missing experts" and Sec. 4.2: experts with no replica left are
    masked to -inf immediately before top-k, so the next-best live experts
    are chosen in their place.
  * Sec. 3.5: a failed device still exists but is never touched again.
The paper gives no formula for the score function, the grouping, the weight
normalisation, the replica choice or the expert FFN; those follow the layer
shapes of the workloads (softmax or sigmoid scores, DeepSeek-V3 style group
limited top-k, renormalised top-k weights, SwiGLU experts, replica
`t mod count`), as listed with the functions below.

All floating point is fp64 on inputs that were already rounded to the layer's
working dtype.  Integer outputs are int64/int32 numpy arrays.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

NEG_INF = -np.inf


# --------------------------------------------------------------------------
# a0  logical -> physical map (Sec. 3.4 "Redundant experts" / "Missing experts")
# --------------------------------------------------------------------------
@dataclass
class ExpertMap:
    l2p_table: np.ndarray   # int32 [E, max_replicas], surviving slots ascending, -1 padded
    l2p_count: np.ndarray   # int32 [E], number of surviving replicas (0 = masked expert)
    slot_alive: np.ndarray  # uint8 [P], 1 where the slot holds an expert on a live rank
    n_live_slots: int
    n_live_experts: int
    n_lost_experts: int      # experts with no surviving replica
    n_degraded_experts: int  # experts that lost some but not all replicas


def build_map(phys_to_logical: np.ndarray, rank_failed: np.ndarray, slots_per_rank: int,
              E: int, max_replicas: int, expert_failed: Optional[np.ndarray] = None) -> ExpertMap:
    """Remove every replica that sits on a failed rank from the map.

    A slot p belongs to rank p // slots_per_rank.  Slot p survives when its
    rank is not failed and it holds an expert (phys_to_logical[p] >= 0).  For
    each logical expert the surviving slots are listed in ascending order.

    `expert_failed` (Sec. 4.2: a failed expert i is treated as failed wherever
    it is chosen) additionally removes every replica of the flagged experts.
    """
    p2l = np.asarray(phys_to_logical, dtype=np.int64)
    failed = np.asarray(rank_failed, dtype=np.uint8)
    P = p2l.shape[0]
    assert P == failed.shape[0] * slots_per_rank
    assert set(np.unique(failed)).issubset({0, 1})
    table = np.full((E, max_replicas), -1, dtype=np.int32)
    count = np.zeros(E, dtype=np.int32)
    full = np.zeros(E, dtype=np.int32)
    alive = np.zeros(P, dtype=np.uint8)
    for p in range(P):
        e = int(p2l[p])
        if e < 0:
            continue
        assert e < E
        full[e] += 1
        if failed[p // slots_per_rank]:
            continue
        if expert_failed is not None and expert_failed[e]:
            continue
        alive[p] = 1
        assert count[e] < max_replicas, "more replicas than max_replicas"
        table[e, count[e]] = p
        count[e] += 1
    return ExpertMap(table, count, alive,
                     n_live_slots=int(alive.sum()),
                     n_live_experts=int((count > 0).sum()),
                     n_lost_experts=int((count == 0).sum()),
                     n_degraded_experts=int(((count > 0) & (count < full)).sum()))


# --------------------------------------------------------------------------
# Lost-expert study (Sec. 4.2): which experts to fail, and activation counts
# --------------------------------------------------------------------------
def every_nth_mask(E: int, n: int) -> np.ndarray:
    """"Every nth": experts fail at a step of n, targeting a fraction 1/n.

    The experts whose index is a multiple of n fail; n = 2 fails every
    even-indexed expert, as the paper's example says.  uint8 [E].
    """
    assert n >= 1
    m = np.zeros(E, dtype=np.uint8)
    for e in range(E):
        if e % n == 0:
            m[e] = 1
    return m


def activation_counts(topk_logical: np.ndarray, E: int) -> np.ndarray:
    """How often each expert was selected (int64 [E]); counts of several layers or batches add."""
    c = np.zeros(E, dtype=np.int64)
    for e in np.asarray(topk_logical).ravel():
        c[int(e)] += 1
    return c


def most_activated_mask(counts: np.ndarray, n_fail: int) -> np.ndarray:
    """"Task-based": fail the n_fail most frequently activated experts.

    Experts are ranked by descending count, equal counts by ascending id.
    """
    counts = np.asarray(counts)
    order = sorted(range(len(counts)), key=lambda e: (-int(counts[e]), e))
    m = np.zeros(len(counts), dtype=np.uint8)
    for e in order[:n_fail]:
        m[e] = 1
    return m


# --------------------------------------------------------------------------
# Logical-rank compaction (Sec. 3.5 "Recreating Communications")
# --------------------------------------------------------------------------
def compact_ranks(logical_rank: Sequence[int], failed_device: int, switched_device: int = -1) -> List[int]:
    """New logical ranks after one device fails.

    `logical_rank[d]` is device d's current logical rank (-1 = not in the
    domain).  Without a role switch the failed device leaves a gap: the device
    that had the next rank takes its rank and every later rank is decremented.
    With a role switch, device `switched_device` (in the domain or not) takes
    the failed device's rank; the gap it leaves behind, if it had a rank, is
    closed the same way.  The failed device ends with rank -1.
    """
    ranks = list(logical_rank)
    gap = ranks[failed_device]
    assert gap >= 0, "the failed device had no rank"
    ranks[failed_device] = -1
    if switched_device >= 0:
        assert switched_device != failed_device
        old = ranks[switched_device]
        ranks[switched_device] = gap
        gap = old                       # the rank the switched device gives up (-1: none)
    if gap >= 0:
        for d in range(len(ranks)):
            if ranks[d] > gap:
                ranks[d] -= 1
    return ranks


def compacted_rank_offsets(slot_offsets: Sequence[int], logical_rank: Sequence[int], slots_per_rank: int) -> List[int]:
    """Segment boundaries of a dispatched buffer in compacted rank order (Sec. 3.5).

    Device d owns slots [d*S, (d+1)*S), i.e. rows [slot_offsets[d*S], slot_offsets[(d+1)*S]).
    Entry l (l < number of live devices) is the first row of the device whose logical
    rank is l; entries from the number of live devices up to len(logical_rank) hold N.
    A device without a logical rank must have received no rows.
    """
    R, S = len(logical_rank), slots_per_rank
    N = int(slot_offsets[R * S])
    out = [N] * (R + 1)
    for d in range(R):
        a, b = int(slot_offsets[d * S]), int(slot_offsets[(d + 1) * S])
        if logical_rank[d] < 0:
            assert a == b, "a device outside the domain holds rows"
        else:
            out[logical_rank[d]] = a
    return out


def enough_live_experts(l2p_count: np.ndarray, k: int, n_group: int, topk_group: int) -> bool:
    """True when every token can always be given k live experts.

    Ungrouped: at least k live experts.  Grouped: groups holding no live
    expert are only kept when fewer than topk_group groups have one, so the
    worst case keeps the topk_group *live* groups with the fewest live
    experts (or all live groups if there are fewer than topk_group).
    """
    live = np.asarray(l2p_count) > 0
    if n_group <= 1:
        return int(live.sum()) >= k
    per_group = live.reshape(n_group, -1).sum(axis=1)
    nonzero = np.sort(per_group[per_group > 0])
    return int(nonzero[:topk_group].sum()) >= k


# --------------------------------------------------------------------------
# a1  router logits (Sec. 2.1: the gating function's scores start from x W_r)
# --------------------------------------------------------------------------
def router_logits(x: np.ndarray, w_router: np.ndarray) -> np.ndarray:
    """logits[t, e] = sum_h x[t, h] * W_r[h, e], in fp64."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(w_router, dtype=np.float64)


# --------------------------------------------------------------------------
# a2  scores and failure mask (Sec. 3.4 "Missing experts", Sec. 4.2)
# --------------------------------------------------------------------------
def scores(logits: np.ndarray, score_fn: str) -> np.ndarray:
    """Per-token gating scores over all E experts, before any mask."""
    z = np.asarray(logits, dtype=np.float64)
    if score_fn == "softmax":
        z = z - z.max(axis=1, keepdims=True)
        ez = np.exp(z)
        return ez / ez.sum(axis=1, keepdims=True)
    if score_fn == "sigmoid":
        return 1.0 / (1.0 + np.exp(-z))
    raise ValueError(score_fn)


def masked_selection_scores(s: np.ndarray, l2p_count: np.ndarray) -> np.ndarray:
    """Selection score = gating score, or -inf for an expert with no replica left."""
    live = np.asarray(l2p_count) > 0
    return np.where(live[None, :], s, NEG_INF)


# --------------------------------------------------------------------------
# a3  top-k, optionally limited to the best groups
# --------------------------------------------------------------------------
def _top_desc(values: np.ndarray, n: int) -> np.ndarray:
    """Indices of the n largest entries, larger value first, equal values by lower index."""
    order = sorted(range(len(values)), key=lambda i: (-values[i], i))
    return np.array(order[:n], dtype=np.int64)


def group_scores(sel_row: np.ndarray, n_group: int) -> np.ndarray:
    """Score of each contiguous expert group for one token.

    The sum of the group's two largest finite selection scores; a single
    score if only one expert of the group is live; -inf if none is.
    """
    E = sel_row.shape[0]
    gsz = E // n_group
    out = np.empty(n_group)
    for g in range(n_group):
        part = sel_row[g * gsz:(g + 1) * gsz]
        finite = np.sort(part[np.isfinite(part)])[::-1]
        out[g] = NEG_INF if finite.size == 0 else finite[:2].sum()
    return out


def kept_groups(sel_row: np.ndarray, n_group: int, topk_group: int) -> np.ndarray:
    """The topk_group best groups of one token, best first, ties to the lower group id."""
    return _top_desc(group_scores(sel_row, n_group), topk_group)


def select_topk(sel: np.ndarray, k: int, n_group: int = 1, topk_group: int = 1) -> np.ndarray:
    """Ordered top-k expert ids per token, int32 [T, k].

    Ungrouped (n_group == 1): the k largest selection scores, ties to the
    lower expert id, listed by descending score then ascending id.

    Grouped: experts are split into n_group contiguous groups, the
    topk_group best groups are kept (see `group_scores`) and the top-k is
    taken over the experts of the kept groups only.

    A masked expert (-inf) must never be returned: that would mean fewer than
    k live experts were reachable, which is an error.
    """
    sel = np.asarray(sel, dtype=np.float64)
    T, E = sel.shape
    out = np.empty((T, k), dtype=np.int32)
    for t in range(T):
        row = sel[t]
        if n_group > 1:
            gsz = E // n_group
            allowed = np.zeros(E, dtype=bool)
            for g in kept_groups(row, n_group, topk_group):
                allowed[g * gsz:(g + 1) * gsz] = True
            row = np.where(allowed, row, NEG_INF)
        idx = _top_desc(row, k)
        assert np.all(np.isfinite(row[idx])), "fewer than k live experts reachable"
        out[t] = idx
    return out


# --------------------------------------------------------------------------
# a4  combine weights (Sec. 2.3: combine uses the gating scores)
# --------------------------------------------------------------------------
def gate_weights(s: np.ndarray, topk_logical: np.ndarray, route_scale: float = 1.0) -> np.ndarray:
    """w[t, j] = s[t, e_j] / sum_j' s[t, e_j'] * route_scale, using unmasked scores."""
    picked = np.take_along_axis(np.asarray(s, dtype=np.float64), topk_logical.astype(np.int64), axis=1)
    return picked / picked.sum(axis=1, keepdims=True) * route_scale


# --------------------------------------------------------------------------
# a5  logical -> physical remap (Sec. 3.4 "Redundant experts")
# --------------------------------------------------------------------------
def remap(topk_logical: np.ndarray, emap: ExpertMap) -> np.ndarray:
    """Physical slot of each (token, choice): the (t mod count)-th surviving replica."""
    T, k = topk_logical.shape
    out = np.empty((T, k), dtype=np.int32)
    for t in range(T):
        for j in range(k):
            e = int(topk_logical[t, j])
            c = int(emap.l2p_count[e])
            assert c > 0, "token routed to an expert with no replica"
            out[t, j] = emap.l2p_table[e, t % c]
    return out


# --------------------------------------------------------------------------
# a6/a7  dispatch (Sec. 2.3): count, scan, stable placement, row permute
# --------------------------------------------------------------------------
def dispatch_indices(topk_phys: np.ndarray, P: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """slot_offsets [P+1], dst_row [N], src_of [N] of the stable sort by slot.

    Flat routed-row index i = t*k + j.  Rows of slot p occupy
    [slot_offsets[p], slot_offsets[p+1]) in ascending i (a stable counting
    sort); slots are laid out in ascending id, i.e. rank by rank.
    """
    flat = np.asarray(topk_phys, dtype=np.int64).ravel()
    N = flat.shape[0]
    counts = np.zeros(P, dtype=np.int64)
    for p in flat:
        counts[p] += 1
    offsets = np.zeros(P + 1, dtype=np.int32)
    for p in range(P):
        offsets[p + 1] = offsets[p] + counts[p]
    cursor = offsets[:-1].astype(np.int64).copy()
    dst_row = np.empty(N, dtype=np.int32)
    src_of = np.empty(N, dtype=np.int32)
    for i in range(N):
        p = flat[i]
        dst_row[i] = cursor[p]
        src_of[cursor[p]] = i
        cursor[p] += 1
    return offsets, dst_row, src_of


def permute_rows(x: np.ndarray, dst_row: np.ndarray, k: int) -> np.ndarray:
    """x_perm[dst_row[i], :] = x[i // k, :]."""
    N = dst_row.shape[0]
    xp = np.empty((N, x.shape[1]), dtype=x.dtype)
    for i in range(N):
        xp[dst_row[i]] = x[i // k]
    return xp


# --------------------------------------------------------------------------
# a8  expert FFN (Sec. 2.1: each expert acts as an FFN; SwiGLU from the layer shapes)
# --------------------------------------------------------------------------
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def swiglu_ffn(v: np.ndarray, gate: np.ndarray, up: np.ndarray, down: np.ndarray) -> np.ndarray:
    """(silu(v @ gate) * (v @ up)) @ down, gate/up [H, I], down [I, H], fp64."""
    v = np.asarray(v, dtype=np.float64)
    g = v @ np.asarray(gate, dtype=np.float64)
    u = v @ np.asarray(up, dtype=np.float64)
    return (silu(g) * u) @ np.asarray(down, dtype=np.float64)


def grouped_expert_ffn(x_perm: np.ndarray, slot_offsets: np.ndarray, phys_to_logical: np.ndarray,
                       experts: Dict[int, Dict[str, np.ndarray]]) -> np.ndarray:
    """y_perm rows of slot p = FFN of the expert slot p holds, applied to x_perm's rows of p."""
    y = np.zeros((x_perm.shape[0], x_perm.shape[1]), dtype=np.float64)
    for p in range(len(slot_offsets) - 1):
        a, b = int(slot_offsets[p]), int(slot_offsets[p + 1])
        if b > a:
            w = experts[int(phys_to_logical[p])]
            y[a:b] = swiglu_ffn(x_perm[a:b], w["gate"], w["up"], w["down"])
    return y


# --------------------------------------------------------------------------
# a9  combine (Sec. 2.3)
# --------------------------------------------------------------------------
def combine(y_perm: np.ndarray, dst_row: np.ndarray, topk_weight: np.ndarray,
            y_shared: Optional[np.ndarray]) -> np.ndarray:
    """out[t] = sum_j w[t, j] * y_perm[dst_row[t*k + j]] (+ y_shared[t])."""
    T, k = topk_weight.shape
    out = np.zeros((T, y_perm.shape[1]), dtype=np.float64)
    for t in range(T):
        for j in range(k):
            out[t] += topk_weight[t, j] * y_perm[dst_row[t * k + j]]
        if y_shared is not None:
            out[t] += y_shared[t]
    return out


# --------------------------------------------------------------------------
# whole layer, two ways
# --------------------------------------------------------------------------
def layer_definition(x, w_router, experts, shared, l2p_count, k, score_fn,
                     n_group=1, topk_group=1, route_scale=1.0, logits=None) -> np.ndarray:
    """The layer as its plain definition: a dense gate matrix times every expert.

    out[t] = sum_e g[t, e] * FFN_e(x[t]) + FFN_shared(x[t]) with g[t, e] the
    renormalised score for the selected experts and 0 elsewhere.  Physical
    slots, replicas, dispatch and permutation do not appear: which replica
    serves a token cannot change the result (replicas hold identical weights).
    Every expert is evaluated on every token (use tiny inputs).
    """
    x = np.asarray(x, dtype=np.float64)
    if logits is None:
        logits = router_logits(x, w_router)
    s = scores(logits, score_fn)
    sel = masked_selection_scores(s, l2p_count)
    top = select_topk(sel, k, n_group, topk_group)
    w = gate_weights(s, top, route_scale)
    T, E = s.shape
    g = np.zeros((T, E))
    for t in range(T):
        for j in range(k):
            g[t, top[t, j]] = w[t, j]
    out = np.zeros_like(x)
    for e in range(E):
        we = experts[e]
        out += g[:, e:e + 1] * swiglu_ffn(x, we["gate"], we["up"], we["down"])
    if shared is not None:
        out += swiglu_ffn(x, shared["gate"], shared["up"], shared["down"])
    return out


@dataclass
class LayerTrace:
    logits: np.ndarray
    topk_logical: np.ndarray
    topk_weight: np.ndarray
    topk_phys: np.ndarray
    slot_offsets: np.ndarray
    dst_row: np.ndarray
    src_of: np.ndarray
    x_perm: np.ndarray
    y_perm: np.ndarray
    y_shared: Optional[np.ndarray]
    out: np.ndarray


def layer_staged(x, w_router, experts, shared, phys_to_logical, emap: ExpertMap, k, score_fn,
                 n_group=1, topk_group=1, route_scale=1.0, logits=None) -> LayerTrace:
    """The layer as the sequence of steps the library performs (a1..a9).

    `logits` may be supplied (e.g. the GPU's fp32 logits) so that the integer
    steps can be compared with zero tolerance independent of GEMM rounding.
    """
    x = np.asarray(x, dtype=np.float64)
    if logits is None:
        logits = router_logits(x, w_router)
    logits = np.asarray(logits, dtype=np.float64)
    s = scores(logits, score_fn)
    sel = masked_selection_scores(s, emap.l2p_count)
    top = select_topk(sel, k, n_group, topk_group)
    w = gate_weights(s, top, route_scale)
    phys = remap(top, emap)
    offsets, dst_row, src_of = dispatch_indices(phys, len(phys_to_logical))
    x_perm = permute_rows(x, dst_row, k)
    y_perm = grouped_expert_ffn(x_perm, offsets, phys_to_logical, experts)
    y_sh = None if shared is None else swiglu_ffn(x, shared["gate"], shared["up"], shared["down"])
    out = combine(y_perm, dst_row, w, y_sh)
    return LayerTrace(logits, top, w, phys, offsets, dst_row, src_of, x_perm, y_perm, y_sh, out)


# --------------------------------------------------------------------------
# near-tie accounting for comparisons against a lower-precision selection
# --------------------------------------------------------------------------
def selection_gap(sel_row: np.ndarray, mine: Sequence[int], theirs: Sequence[int]) -> float:
    """Largest absolute score gap between experts the two selections disagree on.

    `sel_row` are this oracle's fp64 selection scores of one token.  When the
    two ordered lists differ, the disagreement is explained by a near-tie if
    the scores of the differing experts (position by position) are within a
    small gap of each other; the caller compares the returned gap to 1e-5.
    """
    gap = 0.0
    for a, b in zip(mine, theirs):
        if a != b:
            gap = max(gap, abs(float(sel_row[a]) - float(sel_row[b])))
    return gap
