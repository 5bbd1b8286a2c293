"""Pins for the oracle's capacity assignment with Random Token Selection.

Hand-worked cases (tests/golden), an independent sort-then-enumerate router in
pure Python, exhaustive enumeration of tiny top-1 problems, structural
invariants, and the statistical property RTS is introduced for (Sec. 3.1):
keep-probability independent of token position.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import moe_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "route_worked_cases.txt")


def sorted_router(expert_idx, keys, E, C):
    """Independent statement: per expert, sort its candidates with Python's
    sort on (choice, -key, token) and hand out slots in that order."""
    T, k = expert_idx.shape
    slot = np.full((T, k), -1, np.int32)
    src = np.full((E, C), -1, np.int32)
    demand = np.zeros(E, np.int32)
    for e in range(E):
        cands = [(j, -(0.0 if keys is None else float(keys[t])), t)
                 for t in range(T) for j in range(k) if expert_idx[t, j] == e]
        demand[e] = len(cands)
        for s, (j, _, t) in enumerate(sorted(cands)[:C]):
            slot[t, j] = s
            src[e, s] = t * k + j
    return slot, np.minimum(demand, C).astype(np.int32), demand, src


def load_golden():
    cases, cur = [], {}
    for line in open(GOLDEN):
        line = line.strip()
        if line.startswith("#"):
            continue
        if not line:
            if cur:
                cases.append(cur)
                cur = {}
            continue
        key, *vals = line.split()
        cur[key] = vals
    if cur:
        cases.append(cur)
    return cases


@pytest.mark.parametrize("case", load_golden(), ids=lambda c: c["name"][0])
def test_hand_worked_cases(case):
    E, C, k = int(case["E"][0]), int(case["C"][0]), int(case["k"][0])
    eidx = np.array(case["expert_idx"], np.int32).reshape(-1, k)
    keys = None if case["keys"] == ["none"] else np.array(case["keys"], np.float32)
    slot, count, demand, src = O.route(eidx, keys, E, C)
    assert slot.reshape(-1).tolist() == [int(v) for v in case["slot"]]
    assert count.tolist() == [int(v) for v in case["count"]]
    assert demand.tolist() == [int(v) for v in case["demand"]]
    assert src.reshape(-1).tolist() == [int(v) for v in case["slot_src"]]


def random_choices(r, T, E, k):
    if k == 1:
        return r.integers(0, E, size=(T, 1)).astype(np.int32)
    a = r.integers(0, E, size=T)
    b = (a + r.integers(1, E, size=T)) % E
    return np.stack([a, b], axis=1).astype(np.int32)


@pytest.mark.parametrize("k", [1, 2])
@pytest.mark.parametrize("keymode", ["none", "uniform", "ties"])
def test_counting_definition_equals_sort_then_enumerate(k, keymode):
    r = np.random.default_rng(11 + k)
    for T, E, C in [(1, 2, 1), (7, 3, 2), (40, 4, 7), (64, 5, 30), (64, 2, 1)]:
        eidx = random_choices(r, T, E, k)
        keys = {"none": None, "uniform": r.random(T, dtype=np.float32),
                "ties": r.integers(0, 3, T).astype(np.float32)}[keymode]
        got = O.route(eidx, keys, E, C)
        want = sorted_router(eidx, keys, E, C)
        for g, w in zip(got, want):
            assert np.array_equal(g, w)


def test_exhaustive_tiny_top1():
    key_patterns = [None, [0.3, 0.1, 0.9, 0.5, 0.5, 0.7], [1.0] * 6, [0.1, 0.2, 0.3, 0.4, 0.5, 0.6]]
    n = 0
    for T in range(1, 7):
        for E in range(1, 4):
            for C in (1, 2):
                for assign in itertools.product(range(E), repeat=T):
                    eidx = np.array(assign, np.int32).reshape(T, 1)
                    for kp in key_patterns[: 2 if T > 4 else 4]:
                        keys = None if kp is None else np.array(kp[:T], np.float32)
                        got = O.route(eidx, keys, E, C)
                        want = sorted_router(eidx, keys, E, C)
                        assert all(np.array_equal(g, w) for g, w in zip(got, want))
                        n += 1
    assert n > 3000


@pytest.mark.parametrize("k", [1, 2])
def test_structural_invariants(k):
    r = np.random.default_rng(5)
    T, E, C = 600, 7, (90 if k == 1 else 150)
    # skewed choice so some experts overflow and some underfill
    pvals = np.array([0.4, 0.25, 0.15, 0.1, 0.05, 0.04, 0.01])
    first = r.choice(E, size=T, p=pvals)
    eidx = first[:, None].astype(np.int32)
    if k == 2:
        second = (first + r.integers(1, E, size=T)) % E
        eidx = np.stack([first, second], 1).astype(np.int32)
    keys = r.random(T, dtype=np.float32)
    slot, count, demand, src = O.route(eidx, keys, E, C)
    assert np.all(count <= C)
    assert demand.sum() == k * T
    assert np.array_equal(count, np.minimum(demand, C))
    assert count.max() == C and count.min() < C          # both regimes present
    for e in range(E):
        s = np.sort(slot[(eidx == e) & (slot >= 0)])
        assert np.array_equal(s, np.arange(count[e]))      # slots 0..n_e-1 once each
        assert np.all(src[e, count[e]:] == -1)
        for sl in range(count[e]):
            t, j = divmod(int(src[e, sl]), k)
            assert eidx[t, j] == e and slot[t, j] == sl    # slot_src inverts slot
        for j in range(k):
            cand = np.nonzero(eidx[:, j] == e)[0]
            kept = cand[slot[cand, j] >= 0]
            dropped = cand[slot[cand, j] < 0]
            if kept.size and dropped.size:
                assert keys[kept].min() >= keys[dropped].max()   # higher priority wins
    if k == 2:
        # a second choice is only kept if every first choice of that expert is
        for e in range(E):
            if np.any((eidx[:, 1] == e) & (slot[:, 1] >= 0)):
                assert np.all(slot[eidx[:, 0] == e, 0] >= 0)


def test_no_keys_keeps_the_first_candidates_in_position_order():
    r = np.random.default_rng(9)
    T, E, C = 300, 4, 40
    eidx = random_choices(r, T, E, 2)
    slot, count, _, _ = O.route(eidx, None, E, C)
    for e in range(E):
        order = [(j, t) for j in range(2) for t in range(T) if eidx[t, j] == e]
        for rank, (j, t) in enumerate(order):
            assert slot[t, j] == (rank if rank < C else -1)


def test_enough_capacity_drops_nothing():
    r = np.random.default_rng(10)
    eidx = random_choices(r, 128, 4, 2)
    slot, count, demand, _ = O.route(eidx, r.random(128, dtype=np.float32), 4, 256)
    assert np.all(slot >= 0) and np.array_equal(count, demand)


def _keep_by_decile(use_keys, seeds):
    T, E, C = 1000, 2, 270
    kept = np.zeros(10)
    cand = np.zeros(10)
    for s in seeds:
        r = np.random.default_rng(1000 + s)
        eidx = (r.random(T) < 0.2).astype(np.int32)[:, None]     # expert 0 takes ~80 %
        keys = r.random(T, dtype=np.float32) if use_keys else None
        slot, *_ = O.route(eidx, keys, E, C)
        on0 = eidx[:, 0] == 0
        dec = np.arange(T) // (T // 10)
        kept += np.bincount(dec[on0 & (slot[:, 0] >= 0)], minlength=10)
        cand += np.bincount(dec[on0], minlength=10)
    return kept, cand


def test_rts_keep_rate_is_flat_in_position_and_plain_priority_is_a_step():
    kept, cand = _keep_by_decile(True, range(40))
    rate = kept.sum() / cand.sum()
    expected = cand * rate
    chi2 = float(((kept - expected) ** 2 / (expected * (1 - rate))).sum())
    assert chi2 < 27.9          # chi-square, 9 dof, p = 0.001
    kept, cand = _keep_by_decile(False, range(5))
    r = kept / cand
    assert np.all(r[:3] == 1.0) and np.all(r[4:] == 0.0)       # prefix kept, suffix dropped


def test_utilisation_counts_every_routed_candidate_and_sums_the_demands():
    """Sec. 3.3 pruning statistic: over several batches the count per expert is
    the sum of the per-batch demands (a bincount of the choices), whatever the
    capacity dropped."""
    rng = np.random.default_rng(9)
    E, batches, demands = 6, [], []
    for T in (50, 1, 77):
        lg = rng.standard_normal((T, E))
        eidx = O.top_k(lg, 2)
        _, _, demand, _ = O.route(eidx, rng.random(T), E, 5)     # tight capacity: many drops
        batches.append(eidx); demands.append(demand)
    u = O.utilisation(batches, E)
    assert u.dtype == np.int64 and u.sum() == 2 * (50 + 1 + 77)
    assert np.array_equal(u, np.sum(demands, axis=0))
    assert np.array_equal(u, np.bincount(np.concatenate([b.ravel() for b in batches]), minlength=E))
    assert np.array_equal(O.utilisation([], E), np.zeros(E, np.int64))


# ---------------------------------------------------------------------------
# grouped token selection (Sec. 3.1 group dimension, Sec. 5.5 ablation arm)
# ---------------------------------------------------------------------------
def brute_grouped(expert_idx, keys, E, C, G):
    """Independent statement: sort each (group, expert)'s candidates by
    (choice, -key, token) with Python's sort, keep the first C/G, and lay the
    groups' kept rows one after another in the expert's buffer."""
    T, k = expert_idx.shape
    Tg, Cg = T // G, C // G
    slot = np.full((T, k), -1, np.int32)
    slot_src = np.full((E, C), -1, np.int32)
    count = np.zeros(E, np.int32)
    for e in range(E):
        nxt = 0
        for g in range(G):
            cands = [(j, -(0.0 if keys is None else float(keys[t])), t)
                     for t in range(g * Tg, (g + 1) * Tg) for j in range(k) if expert_idx[t, j] == e]
            for (j, _, t) in sorted(cands)[:Cg]:
                slot[t, j] = nxt
                slot_src[e, nxt] = t * k + j
                nxt += 1
        count[e] = nxt
    return slot, count, slot_src


@pytest.mark.parametrize("k", [1, 2])
@pytest.mark.parametrize("use_keys", [True, False])
def test_grouped_selection_matches_brute_force(k, use_keys):
    rng = np.random.default_rng(40 + k)
    T, E, G, C = 96, 5, 4, 24
    lg = rng.standard_normal((T, E)); lg[:, 0] += 1.0
    eidx = O.top_k(lg, k)
    keys = rng.random(T) if use_keys else None
    if use_keys:
        keys[10:14] = keys[10]                      # duplicate keys -> token order
    slot, count, demand, slot_src = O.route_grouped(eidx, keys, E, C, G)
    bs, bc, bsrc = brute_grouped(eidx, keys, E, C, G)
    assert np.array_equal(slot, bs) and np.array_equal(count, bc) and np.array_equal(slot_src, bsrc)
    assert np.array_equal(demand, np.bincount(eidx.ravel(), minlength=E))
    assert (slot < 0).any()                         # the hot expert overflows its group capacity


def test_grouped_with_one_group_is_plain_routing_and_groups_confine_the_position_bias():
    rng = np.random.default_rng(7)
    T, E, C = 128, 4, 32
    eidx = O.top_k(rng.standard_normal((T, E)), 1)
    a = O.route(eidx, None, E, C)
    b = O.route_grouped(eidx, None, E, C, 1)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    # every token wants expert 2, position priority: plain routing keeps the first C
    # tokens of the batch, grouped routing the first C/G tokens of every group
    allsame = np.full((T, 1), 2, np.int32)
    sp = O.route(allsame, None, E, C)[0][:, 0]
    sg, cg, dg, srcg = O.route_grouped(allsame, None, E, C, 4)
    assert np.array_equal(np.nonzero(sp >= 0)[0], np.arange(C))
    kept = np.nonzero(sg[:, 0] >= 0)[0]
    assert np.array_equal(kept, np.concatenate([np.arange(g * 32, g * 32 + 8) for g in range(4)]))
    assert np.array_equal(sg[kept, 0], np.arange(C)) and cg[2] == C and dg[2] == T
    assert np.array_equal(srcg[2], kept)            # k = 1: t*k+j = t
    # per group and expert never more than C/G rows
    eidx2 = O.top_k(rng.standard_normal((T, E)), 2)
    s2, c2, _, src2 = O.route_grouped(eidx2, rng.random(T), E, C, 4)
    for g in range(4):
        for e in range(E):
            assert ((s2[g * 32:(g + 1) * 32] >= 0) & (eidx2[g * 32:(g + 1) * 32] == e)).sum() <= C // 4
    # slot_src is the inverse of slot on the rows in use, which form a prefix
    for e in range(E):
        assert np.all(src2[e, :c2[e]] >= 0) and np.all(src2[e, c2[e]:] == -1)
        for s in range(c2[e]):
            t, j = divmod(int(src2[e, s]), 2)
            assert eidx2[t, j] == e and s2[t, j] == s
