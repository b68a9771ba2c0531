"""Pins of the scheduler oracle (oracle/scheduler_oracle.py) against things it does not compute itself.

Section 3.3 (Eq. 6, Alg. 1, Migrate) and Section 3.4 (Alg. 2, Eq. 5 / Eq. 7 / Eq. 9) of the paper.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import flexmoe_oracle as fo
from oracle import scheduler_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------------------
# independent restatements used as the other side of a pin
# ----------------------------------------------------------------------------------------
def dealt_gpu_loads(I, slot_owner, G):
    """Deal every expert's tokens one at a time, cyclically, over its vExperts; count per GPU."""
    S = len(slot_owner) // G
    per_gpu = [0] * G
    for e, I_e in enumerate(I):
        slots = [s for s in range(len(slot_owner)) if slot_owner[s] == e]
        for t in range(int(I_e)):
            per_gpu[slots[t % len(slots)] // S] += 1
    return per_gpu


def dealt_cost(I, slot_owner, G, token_cost, sync_cost=None):
    S = len(slot_owner) // G
    t = [x * token_cost for x in dealt_gpu_loads(I, slot_owner, G)]
    if sync_cost is not None:
        for e in range(len(I)):
            gpus = {s // S for s in range(len(slot_owner)) if slot_owner[s] == e}
            for g in gpus:
                t[g] += sync_cost[len(gpus)]
    return max(t)


def random_cluster(rng, E, G, S, fill=1.0, hot=4.0):
    """Every expert gets one slot, the rest of the occupied slots go to random experts."""
    V = G * S
    assert V >= E
    used = max(E, int(round(V * fill)))
    slots = rng.permutation(V)[:used]
    owner = [so.FREE] * V
    for e in range(E):
        owner[slots[e]] = e
    for s in slots[E:]:
        owner[s] = int(rng.integers(E))
    p = rng.dirichlet(np.full(E, 1.0 / hot))
    I = rng.multinomial(int(rng.integers(50, 400)), p).tolist()
    return I, owner


# ----------------------------------------------------------------------------------------
# Eq. 6
# ----------------------------------------------------------------------------------------
def test_balance_ratio_of_the_papers_worked_example():
    """Figure 1(b): expert loads 10 and 8 on two GPUs, one expert each -> max/mean = 10/9."""
    with open(os.path.join(GOLDEN, "fig1b_expert_loads.txt")) as fh:
        row = [ln for ln in fh if not ln.startswith("#")][0].split()
    load_e0, load_e1 = int(row[4]), int(row[5])
    J = [[load_e0, 0], [0, load_e1]]
    assert so.balance_ratio_exact(J) == Fraction(10, 9)
    assert abs(so.balance_ratio(J) - 1.1111111111111112) < 1e-15
    # the same through the slot model: one slot per GPU, expert e on GPU e
    assert so.expert_gpu_loads([load_e0, load_e1], [0, 1], 2) == J


def test_balance_ratio_closed_forms():
    G = 5
    assert so.balance_ratio([[7] * G, [3] * G]) == 1.0                 # even -> 1
    assert so.balance_ratio([[0, 0, 9, 0, 0], [0, 0, 4, 0, 0]]) == G   # all on one GPU -> |G|
    assert so.balance_ratio([[0] * G]) == 1.0                          # no tokens (reading S5)
    rng = np.random.default_rng(5)
    for _ in range(50):
        J = rng.integers(0, 100, size=(4, G))
        if J.sum() == 0:
            continue
        r = so.balance_ratio_exact(J.tolist())
        assert 1 <= r <= G
        assert r == Fraction(int(J.sum(0).max()) * G, int(J.sum()))
        assert so.balance_ratio_exact((3 * J).tolist()) == r                  # scale-free
        assert so.balance_ratio_exact(J[:, rng.permutation(G)].tolist()) == r  # GPUs unordered
        assert so.balance_ratio_exact(J[rng.permutation(4)].tolist()) == r     # experts unordered


# ----------------------------------------------------------------------------------------
# shares and loads
# ----------------------------------------------------------------------------------------
def test_shares_equal_token_by_token_dealing_and_the_routers_counts():
    rng = np.random.default_rng(11)
    for trial in range(60):
        E, G, S = int(rng.integers(1, 6)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
        if G * S < E:
            continue
        I, owner = random_cluster(rng, E, G, S, fill=rng.choice([0.7, 1.0]))
        share = so.vexpert_shares(I, owner)
        assert sum(share) == sum(I)
        for e in range(E):
            mine = [share[s] for s in so.slots_of(owner, e)]
            assert sum(mine) == I[e] and max(mine) - min(mine) <= 1
            assert mine == sorted(mine, reverse=True)
        assert so.gpu_loads(I, owner, G) == dealt_gpu_loads(I, owner, G)
        # the exported table gives the router (pinned on its own) the same per-vExpert counts
        rep_off, rep_ids = so.placement_table(owner, E)
        V = fo.check_placement(E, np.array(rep_off), np.array(rep_ids))
        idx = np.repeat(np.arange(E), I).astype(np.int32)[:, None]
        r = fo.route(idx, E, np.array(rep_off), np.array(rep_ids))
        occupied = [s for s in range(G * S) if owner[s] != so.FREE]
        assert V == len(occupied)
        assert r["vexpert_count"].tolist() == [share[s] for s in occupied]
        assert r["vexpert_owner"].tolist() == [owner[s] for s in occupied]


def test_cost_equals_dealt_cost():
    rng = np.random.default_rng(12)
    for trial in range(60):
        E, G, S = int(rng.integers(1, 6)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
        if G * S < E:
            continue
        I, owner = random_cluster(rng, E, G, S, fill=rng.choice([0.7, 1.0]))
        c = int(rng.integers(1, 9))
        sync = [0, 0] + sorted(rng.integers(1, 50, size=G - 1).tolist()) if trial % 2 else None
        assert so.step_cost(I, owner, G, c, sync) == dealt_cost(I, owner, G, c, sync)
    # Eq. 7 alone: cost = largest GPU load / TPS
    assert so.step_cost([30, 10], [0, 0, 1, 1], 2, 7) == 30 * 7
    # Eq. 9: an expert on two GPUs pays the two-GPU synchronisation on both
    assert so.step_cost([30, 10], [0, 1, 0, 1], 2, 1, [0, 0, 100]) == 15 + 5 + 200
    assert so.replica_spread([0, 1, 0, 1], 2, 0) == 2 and so.replica_spread([0, 0, 1, 1], 2, 0) == 1


# ----------------------------------------------------------------------------------------
# Alg. 2
# ----------------------------------------------------------------------------------------
def test_policy_maker_on_a_hand_computed_case():
    """Two GPUs x two slots, expert 0 on GPU 0 (30 tokens), expert 1 on GPU 1 (10 tokens).

    cap = (15, 5): expand 0, shrink 1.  Releasing either slot of expert 1 and giving it to
    expert 0 yields shares 10/10/10 for expert 0 and 10 for expert 1: both GPUs compute 20.
    """
    plan = so.make_scheduling_plan([30, 10], [0, 0, 1, 1], 2, 1)
    assert plan == {"e0": 0, "e1": 1, "t0": 30, "t1": 20, "released": 2, "target": 2, "source": 0}
    assert so.apply_plan([0, 0, 1, 1], plan) == [0, 0, 0, 1]
    # already even: nothing to gain
    assert so.make_scheduling_plan([20, 20], [0, 0, 1, 1], 2, 1) is None
    # the coldest expert owns a single vExpert and no other expert can shrink (reading S1)
    assert so.make_scheduling_plan([30, 1], [0, 1], 2, 1) is None
    # ties of capacity go to the lowest expert id (reading S6): caps (20, 20, 2, 2); GPU 0 computes
    # 40 tokens before, 10 + 20 after expert 0 got a second vExpert on GPU 1
    plan = so.make_scheduling_plan([20, 20, 4, 4], [0, 1, 2, 2, 3, 3], 3, 1)
    assert (plan["e0"], plan["e1"], plan["t0"], plan["t1"], plan["released"]) == (0, 2, 40, 30, 2)
    # the greedy step can stall: two GPUs tie for the maximum, relieving one of them gains nothing
    assert so.make_scheduling_plan([20, 20, 4, 4], [0, 0, 1, 1, 2, 2, 3, 3], 4, 1) is None


def test_policy_maker_picks_the_cheapest_pair_of_slots():
    """t1 is the minimum over every (released vExpert, free target) pair, by exhaustive search."""
    rng = np.random.default_rng(13)
    seen_plan = seen_none = 0
    for trial in range(150):
        E, G, S = int(rng.integers(2, 5)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        if G * S < E:
            continue
        I, owner = random_cluster(rng, E, G, S, fill=rng.choice([0.8, 1.0]))
        c = int(rng.integers(1, 5))
        sync = [0, 0] + sorted(rng.integers(1, 30, size=G - 1).tolist()) if trial % 3 == 0 else None
        plan = so.make_scheduling_plan(I, owner, G, c, sync)
        # capacities by exact fractions, choices restated here
        n = [owner.count(e) for e in range(E)]
        caps = [Fraction(I[e], n[e]) for e in range(E)]
        e0 = min(range(E), key=lambda e: (-caps[e], e))
        shrinkable = [e for e in range(E) if n[e] >= 2]
        if not shrinkable or min(shrinkable, key=lambda e: (caps[e], e)) == e0:
            assert plan is None
            seen_none += 1
            continue
        e1 = min(shrinkable, key=lambda e: (caps[e], e))
        t0 = dealt_cost(I, owner, G, c, sync)
        best = None
        for released in [s for s in range(G * S) if owner[s] == e1]:
            trial_owner = list(owner)
            trial_owner[released] = so.FREE
            for target in [s for s in range(G * S) if trial_owner[s] == so.FREE]:
                cand = list(trial_owner)
                cand[target] = e0
                t = dealt_cost(I, cand, G, c, sync)
                best = t if best is None else min(best, t)
        if best < t0:
            assert plan is not None and (plan["e0"], plan["e1"]) == (e0, e1)
            assert plan["t0"] == t0 and plan["t1"] == best
            assert dealt_cost(I, so.apply_plan(owner, plan), G, c, sync) == best
            assert owner[plan["source"]] == e0
            seen_plan += 1
        else:
            assert plan is None
            seen_none += 1
    assert seen_plan > 20 and seen_none > 20


# ----------------------------------------------------------------------------------------
# Migrate
# ----------------------------------------------------------------------------------------
def test_migrate_on_a_hand_computed_case():
    """Both experts straddle both GPUs; a two-GPU synchronisation costs 5, tokens cost 1.

    Before: each GPU computes 5 + 5 tokens and pays two synchronisations: 20.  Exchanging slot 0
    (expert 0's only vExpert on GPU 0) with slot 3 leaves each expert on one GPU: cost 10.
    """
    I, owner, sync = [10, 10], [0, 1, 0, 1], [0, 0, 5]
    assert so.step_cost(I, owner, 2, 1, sync) == 20
    mig = so.make_migrate_plan(I, owner, 2, 1, sync)
    assert (mig["a"], mig["b"], mig["t0"], mig["t1"]) == (0, 3, 20, 10)
    # without a synchronisation cost the exchange gains nothing and is not made
    assert so.make_migrate_plan(I, owner, 2, 1, None) is None
    # an expert that lives on one GPU only is never moved
    assert so.make_migrate_plan([10, 10], [0, 0, 1, 1], 2, 1, sync) is None


def test_migrate_candidates_by_exhaustive_search():
    rng = np.random.default_rng(14)
    hits = 0
    for trial in range(120):
        E, G, S = int(rng.integers(2, 5)), int(rng.integers(2, 4)), int(rng.integers(1, 4))
        if G * S < E:
            continue
        I, owner = random_cluster(rng, E, G, S, fill=rng.choice([0.8, 1.0]))
        sync = [0, 0] + sorted(rng.integers(1, 60, size=G - 1).tolist())
        mig = so.make_migrate_plan(I, owner, G, 1, sync)
        t0 = dealt_cost(I, owner, G, 1, sync)
        best = None
        for a, b in itertools.permutations(range(G * S), 2):
            e = owner[a]
            if e == so.FREE or owner[b] == e or a // S == b // S:
                continue
            on_ga = [s for s in range(G * S) if owner[s] == e and s // S == a // S]
            on_gb = [s for s in range(G * S) if owner[s] == e and s // S == b // S]
            if len(on_ga) != 1 or not on_gb:
                continue
            cand = list(owner)
            cand[a], cand[b] = cand[b], cand[a]
            t = dealt_cost(I, cand, G, 1, sync)
            best = t if best is None else min(best, t)
        if best is not None and best < t0:
            assert mig is not None and mig["t1"] == best and mig["t0"] == t0
            hits += 1
        else:
            assert mig is None
    assert hits > 10


# ----------------------------------------------------------------------------------------
# Alg. 1
# ----------------------------------------------------------------------------------------
def replay(owner, ops):
    P = list(owner)
    for kind, e, a, b in ops:
        if kind == so.SHRINK:
            assert P[a] == e
            P[a] = so.FREE
        elif kind == so.EXPAND:
            assert P[b] == so.FREE and P[a] == e
            P[b] = e
        else:
            assert P[a] == e
            P[a], P[b] = P[b], P[a]
    return P


def test_scheduler_invariants():
    rng = np.random.default_rng(15)
    moved = 0
    for trial in range(80):
        E, G, S = int(rng.integers(2, 7)), int(rng.integers(2, 5)), int(rng.integers(1, 4))
        if G * S < E:
            continue
        I, owner = random_cluster(rng, E, G, S, fill=rng.choice([0.8, 1.0]))
        threshold = float(rng.choice([1.0, 1.05, 1.3]))
        ops, P, before, after = so.schedule(I, owner, G, 1, threshold, 64)
        assert replay(owner, ops) == P
        assert all(P.count(e) >= 1 for e in range(E))
        assert sum(o != so.FREE for o in P) == sum(o != so.FREE for o in owner)
        assert before == so.balance_ratio(so.expert_gpu_loads(I, owner, G))
        assert after == so.balance_ratio(so.expert_gpu_loads(I, P, G))
        assert after <= before
        if before <= threshold:
            assert not [op for op in ops if op[0] != so.MIGRATE]
        # every Shrink/Expand pair lowers the estimated cost (Alg. 2 returns nothing otherwise)
        cur, cost = list(owner), dealt_cost(I, owner, G, 1)
        for i in range(0, len(ops) - 1, 2):
            if ops[i][0] != so.SHRINK:
                break
            cur = replay(cur, ops[i:i + 2])
            new_cost = dealt_cost(I, cur, G, 1)
            assert new_cost < cost
            cost = new_cost
        # stopping is for a reason: balanced enough, or the Policy Maker has nothing left
        if after > threshold and len(ops) + 2 <= 64:
            assert so.make_scheduling_plan(I, P, G, 1) is None
        moved += bool(ops)
    assert moved > 20


def test_scheduler_respects_the_operation_budget_and_the_threshold():
    I, owner = [90, 5, 5, 5], [0, 1, 1, 1, 2, 2, 2, 3, 3, 3, 3, 3]
    ops, P, before, after = so.schedule(I, owner, 4, 1, 1.0, 2)
    assert len(ops) == 2 and [op[0] for op in ops] == [so.SHRINK, so.EXPAND]
    ops, P, before, after = so.schedule(I, owner, 4, 1, 1.0, 1)
    assert not ops and P == owner
    ops, P, before, after = so.schedule(I, owner, 4, 1, before, 64)     # ratio == threshold: no trigger
    assert not ops
    ops, P, before, after = so.schedule(I, owner, 4, 1, 1.0, 64)
    assert after < before and P.count(0) > 1


def test_scheduler_reaches_the_ideal_capacity_when_it_exists():
    """Section 3.2: B/(G*S) tokens per vExpert is the ideal; reachable loads are reached.

    4 GPUs x 2 slots, 8 experts, expert 0 takes 5/8 of 640 tokens, experts 1..3 take 1/8 each and the
    rest nothing -- but every expert must keep one vExpert, so the best placement gives expert 0
    all spare capacity.
    """
    I = [400, 80, 80, 80, 0, 0, 0, 0]
    owner = [0, 1, 2, 3, 4, 5, 6, 7]
    ops, P, before, after = so.schedule(I, owner, 4, 1, 1.0, 64)
    assert P == owner and not ops           # no expert can shrink: nothing to do
    # 16 slots: the idle experts own two each and can give one away
    owner = [0, 1, 2, 3, 4, 4, 5, 5, 6, 6, 7, 7, 1, 2, 3, 0]
    ops, P, before, after = so.schedule(I, owner, 8, 1, 1.0, 64)
    assert after < before
    assert [P.count(e) for e in range(4, 8)] == [1, 1, 1, 1]
    assert P.count(0) == 2 + 4


def test_scheduler_is_never_worse_than_where_it_started_and_bounded_by_the_optimum():
    """Exhaustive optimum over all placements of a tiny cluster (3 experts, 2 GPUs x 2 slots)."""
    rng = np.random.default_rng(16)
    E, G, S = 3, 2, 2
    placements = [list(p) for p in itertools.product(range(E), repeat=G * S) if len(set(p)) == E]
    for trial in range(25):
        I = rng.multinomial(120, rng.dirichlet(np.full(E, 0.5))).tolist()
        optimum = min(dealt_cost(I, p, G, 1) for p in placements)
        owner = placements[int(rng.integers(len(placements)))]
        ops, P, before, after = so.schedule(I, owner, G, 1, 1.0, 64)
        assert optimum <= dealt_cost(I, P, G, 1) <= dealt_cost(I, owner, G, 1)


def test_placement_table_numbers_occupied_slots_in_order():
    rep_off, rep_ids = so.placement_table([1, so.FREE, 0, 1, so.FREE, 0], 2)
    assert rep_off == [0, 2, 4] and rep_ids == [1, 3, 0, 2]
    rep_off, rep_ids = so.placement_table([0, 1, 2, 0], 3)
    assert rep_off == [0, 2, 3, 4] and rep_ids == [0, 3, 1, 2]
    with pytest.raises(ValueError):
        so.placement_table([0, 0], 2)
