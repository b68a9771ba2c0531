"""CPU oracle for the host-side placement scheduler (balance ratio, Policy Maker, Scheduler).

TEST INFRASTRUCTURE ONLY.  A plain, slow statement of the steps of Section 3.3
(balance ratio Eq. 6, the Expand / Shrink / Migrate primitives, Alg. 1) and
Section 3.4 (Alg. 2 with the cost of Eq. 5 built from Eq. 7 and, when the caller
supplies its table, Eq. 9), written from the paper (arXiv 2304.03946).  It shares
no code with the library and must never be imported by the product path; only
the tests and the benchmark's baseline leg use it.

Model of the cluster (Section 3.2): G GPUs with S vExpert slots each; slot
s = g*S + i lives on GPU g.  The placement P is `slot_owner[G*S]`: the expert a
slot replicates, or -1 for a free slot.  An expert's I_e tokens are partitioned
evenly over its vExperts (third vExpert property): floor(I_e/n_e) each, the
first I_e mod n_e of them in ascending slot id taking one more -- the same
integer shares the router hands out -- so after Alg. 3's routing GPU g computes
the sum of the shares of its slots.

All decisions are taken in integers: times are integer multiples of a caller's
unit (`token_cost` = time per token = 1/TPS of Eq. 7, `sync_cost[m]` = time of
one gradient synchronisation over m GPUs, Eq. 9), capacities cap_e = I_e/n_e are
compared as exact fractions.  Only the balance ratio is a float.

Readings of what the paper leaves open (each also taken by the library):
  S1  Alg. 2 shrinks the expert with the smallest capacity among those that own
      at least two vExperts (an expert must keep one), and returns the empty
      plan when there is none, or when it is the expert to expand.
  S2  Alg. 2 does not say where.  Every vExpert of e1 is a candidate to release;
      the new vExpert of e0 goes into the released slot or into the lowest free
      slot of any GPU; the pair with the smallest estimated cost t1 wins, the
      first in (released slot, target slot) order among equals.
  S3  Eq. 5 per GPU: sum over the experts placed there of T_C and T_Sync; the
      All-to-All term (Eq. 8) is left out (no bandwidth table on one GPU), so
      without a `sync_cost` table the cost is the largest GPU load times
      `token_cost`.
  S4  Migrate (Alg. 1, last step) exchanges the owners of two slots so that an
      expert leaves a GPU where it holds a single vExpert for a GPU where it
      already has one; one exchange per call of the scheduler, the one with the
      smallest estimated cost, and only if that is below the current cost.
  S5  The balance ratio of a cluster without tokens is 1.
  S6  Ties of argmax / argmin capacity go to the lowest expert id.

Pins (tests/test_oracle_scheduler.py): the worked example of Figure 1(b), closed
forms of Eq. 6, a hand-computed Alg. 2 step, token-by-token dealing for the
shares, exhaustive search over every (release, target) pair and over every
placement of a tiny cluster, and the invariants of Alg. 1.
"""
from __future__ import annotations

from fractions import Fraction

FREE = -1
EXPAND, SHRINK, MIGRATE = 0, 1, 2


# ---------------------------------------------------------------------------
# Section 3.2: placement at vExpert level
# ---------------------------------------------------------------------------
def slots_of(slot_owner, e: int):
    """Slot ids of the vExperts of expert e, ascending (replica order)."""
    return [s for s, o in enumerate(slot_owner) if o == e]


def vexpert_shares(I, slot_owner):
    """Tokens each slot computes: even partition of I_e over the vExperts of e."""
    share = [0] * len(slot_owner)
    for e, I_e in enumerate(I):
        slots = slots_of(slot_owner, e)
        if not slots:
            if I_e:
                raise ValueError(f"expert {e} has tokens but no vExpert")
            continue
        q, m = divmod(int(I_e), len(slots))
        for r, s in enumerate(slots):
            share[s] = q + (1 if r < m else 0)
    return share


def expert_gpu_loads(I, slot_owner, G: int):
    """I_{e,g} of Eq. 5 / Eq. 6: tokens of expert e computed on GPU g, as a list of rows."""
    S = len(slot_owner) // G
    share = vexpert_shares(I, slot_owner)
    J = [[0] * G for _ in I]
    for s, o in enumerate(slot_owner):
        if o != FREE:
            J[o][s // S] += share[s]
    return J


def gpu_loads(I, slot_owner, G: int):
    J = expert_gpu_loads(I, slot_owner, G)
    return [sum(J[e][g] for e in range(len(I))) for g in range(G)]


def replica_spread(slot_owner, G: int, e: int) -> int:
    """Number of GPUs that hold a vExpert of e (size of its synchronisation group, Eq. 9)."""
    S = len(slot_owner) // G
    return len({s // S for s in slots_of(slot_owner, e)})


# ---------------------------------------------------------------------------
# Eq. 6
# ---------------------------------------------------------------------------
def balance_ratio_exact(J) -> Fraction:
    """Eq. 6 on a matrix J[e][g]: largest GPU load over the mean GPU load."""
    G = len(J[0])
    per_gpu = [sum(row[g] for row in J) for g in range(G)]
    total = sum(per_gpu)
    if total == 0:
        return Fraction(1)
    return Fraction(max(per_gpu) * G, total)


def balance_ratio(J) -> float:
    r = balance_ratio_exact(J)
    return r.numerator / r.denominator      # one correctly rounded division


# ---------------------------------------------------------------------------
# Eq. 5 with Eq. 7 (and Eq. 9 when a table is given)
# ---------------------------------------------------------------------------
def step_cost(I, slot_owner, G: int, token_cost: int, sync_cost=None) -> int:
    """max over GPUs of sum over resident experts of T_C(I_{e,g}) + T_Sync(P, e)."""
    J = expert_gpu_loads(I, slot_owner, G)
    S = len(slot_owner) // G
    worst = 0
    for g in range(G):
        resident = sorted({o for o in slot_owner[g * S:(g + 1) * S] if o != FREE})
        t = 0
        for e in resident:
            t += J[e][g] * token_cost
            if sync_cost is not None:
                t += sync_cost[replica_spread(slot_owner, G, e)]
        worst = max(worst, t)
    return worst


# ---------------------------------------------------------------------------
# Alg. 2
# ---------------------------------------------------------------------------
def capacities(I, slot_owner):
    """cap_e = I_e / n_e as exact fractions (None for an expert without vExperts)."""
    caps = []
    for e, I_e in enumerate(I):
        n_e = len(slots_of(slot_owner, e))
        caps.append(Fraction(int(I_e), n_e) if n_e else None)
    return caps


def make_scheduling_plan(I, slot_owner, G: int, token_cost: int, sync_cost=None):
    """Alg. 2.  Returns None (empty plan) or a dict describing (Expand e0, Shrink e1)."""
    S = len(slot_owner) // G
    t0 = step_cost(I, slot_owner, G, token_cost, sync_cost)
    caps = capacities(I, slot_owner)
    placed = [e for e in range(len(I)) if caps[e] is not None]
    if not placed:
        return None
    e0 = max(placed, key=lambda e: (caps[e], -e))
    shrinkable = [e for e in placed if len(slots_of(slot_owner, e)) >= 2]
    if not shrinkable:
        return None
    e1 = min(shrinkable, key=lambda e: (caps[e], e))
    if e1 == e0:
        return None
    best = None
    for released in slots_of(slot_owner, e1):
        trial = list(slot_owner)
        trial[released] = FREE
        targets = {released}
        for g in range(G):
            free = [s for s in range(g * S, (g + 1) * S) if trial[s] == FREE]
            if free:
                targets.add(free[0])
        for target in sorted(targets):
            placed_trial = list(trial)
            placed_trial[target] = e0
            t1 = step_cost(I, placed_trial, G, token_cost, sync_cost)
            if best is None or t1 < best["t1"]:
                best = {"t1": t1, "released": released, "target": target}
    if best["t1"] >= t0:
        return None
    # the copy source of Expand: a vExpert of e0 on the target's GPU if there is one
    # (parameter sharing inside a GPU), else its lowest slot
    src_slots = slots_of(slot_owner, e0)
    same_gpu = [s for s in src_slots if s // S == best["target"] // S]
    return {"e0": e0, "e1": e1, "t0": t0, "t1": best["t1"], "released": best["released"],
            "target": best["target"], "source": (same_gpu or src_slots)[0]}


def apply_plan(slot_owner, plan):
    out = list(slot_owner)
    out[plan["released"]] = FREE
    out[plan["target"]] = plan["e0"]
    return out


# ---------------------------------------------------------------------------
# Migrate
# ---------------------------------------------------------------------------
def make_migrate_plan(I, slot_owner, G: int, token_cost: int, sync_cost=None):
    """Best single exchange that takes an expert off a GPU where it has one vExpert (reading S4)."""
    S = len(slot_owner) // G
    t0 = step_cost(I, slot_owner, G, token_cost, sync_cost)
    best = None
    for a, e in enumerate(slot_owner):
        if e == FREE:
            continue
        ga = a // S
        on_ga = [s for s in slots_of(slot_owner, e) if s // S == ga]
        if len(on_ga) != 1:
            continue
        hosts = sorted({s // S for s in slots_of(slot_owner, e)} - {ga})
        for gb in hosts:
            for b in range(gb * S, (gb + 1) * S):
                if slot_owner[b] == e:
                    continue
                trial = list(slot_owner)
                trial[a], trial[b] = trial[b], trial[a]
                t1 = step_cost(I, trial, G, token_cost, sync_cost)
                if best is None or t1 < best["t1"]:
                    best = {"t1": t1, "a": a, "b": b}
    if best is None or best["t1"] >= t0:
        return None
    best["t0"] = t0
    return best


# ---------------------------------------------------------------------------
# Alg. 1 (one pass of its outer loop)
# ---------------------------------------------------------------------------
def schedule(I, slot_owner, G: int, token_cost: int, threshold: float, max_ops: int, sync_cost=None):
    """One iteration of Alg. 1's outer loop for the token assignment I.

    Returns (ops, new_slot_owner, ratio_before, ratio_after); an op is a tuple
    (kind, expert, slot_a, slot_b): (EXPAND, e0, source slot, target slot),
    (SHRINK, e1, released slot, -1), (MIGRATE, owner of slot_a before, slot_a, slot_b).
    """
    P = list(slot_owner)
    ops = []
    before = ratio = balance_ratio(expert_gpu_loads(I, P, G))
    while ratio > threshold and len(ops) + 2 <= max_ops:
        plan = make_scheduling_plan(I, P, G, token_cost, sync_cost)
        if plan is None:
            break
        # the slot is released before it can be taken again
        ops.append((SHRINK, plan["e1"], plan["released"], -1))
        ops.append((EXPAND, plan["e0"], plan["source"], plan["target"]))
        P = apply_plan(P, plan)
        ratio = balance_ratio(expert_gpu_loads(I, P, G))
    if len(ops) + 1 <= max_ops:
        mig = make_migrate_plan(I, P, G, token_cost, sync_cost)
        if mig is not None:
            ops.append((MIGRATE, P[mig["a"]], mig["a"], mig["b"]))
            P[mig["a"]], P[mig["b"]] = P[mig["b"]], P[mig["a"]]
            ratio = balance_ratio(expert_gpu_loads(I, P, G))
    return ops, P, before, ratio


# ---------------------------------------------------------------------------
# the table the router consumes
# ---------------------------------------------------------------------------
def placement_table(slot_owner, E: int):
    """CSR expert -> vExpert ids; occupied slots are numbered in ascending slot id."""
    vid, nxt = {}, 0
    for s, o in enumerate(slot_owner):
        if o != FREE:
            vid[s] = nxt
            nxt += 1
    rep_off, rep_ids = [0], []
    for e in range(E):
        ids = [vid[s] for s in slots_of(slot_owner, e)]
        if not ids:
            raise ValueError(f"expert {e} has no vExpert")
        rep_ids += ids
        rep_off.append(len(rep_ids))
    return rep_off, rep_ids
