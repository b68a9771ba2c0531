"""ctypes binding of the host-side scheduler entry points (include/flexmoe_scheduler.h).

Argument marshalling only: numpy arrays in host memory go in and come out; the balance ratio
(Eq. 6), the cost of a step (Eq. 5), the Policy Maker (Alg. 2) and the Scheduler pass (Alg. 1)
run in the library.  Function names and argument order follow the C entry points.
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import binding

FREE = -1
EXPAND, SHRINK, MIGRATE = 0, 1, 2


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(status: int, where: str):
    if status != binding.OK:
        raise binding.FlexMoEError(status, where)


def _cluster(tokens, slot_owner, G):
    tokens, slot_owner = _i64(tokens), _i32(slot_owner)
    if G < 1 or slot_owner.size % G:
        raise ValueError("slot_owner must hold G * S entries")
    return tokens, slot_owner, int(tokens.size), int(G), int(slot_owner.size // G)


def _sync(sync_cost, G):
    if sync_cost is None:
        return None
    sync_cost = _i64(sync_cost)
    if sync_cost.size != G + 1:
        raise ValueError("sync_cost must hold G + 1 entries")
    return sync_cost


def flexmoe_balance_ratio(tokens, slot_owner, G: int):
    """-> (ratio, gpu_load[G])"""
    tokens, slot_owner, E, G, S = _cluster(tokens, slot_owner, G)
    ratio = ctypes.c_double()
    load = np.zeros(G, dtype=np.int64)
    _check(binding.load_library().flexmoe_balance_ratio(_p(tokens), _p(slot_owner), E, G, S, ctypes.byref(ratio),
                                                        _p(load)), "flexmoe_balance_ratio")
    return ratio.value, load


def flexmoe_step_cost(tokens, slot_owner, G: int, token_cost: int, sync_cost=None) -> int:
    tokens, slot_owner, E, G, S = _cluster(tokens, slot_owner, G)
    sync_cost = _sync(sync_cost, G)
    cost = ctypes.c_int64()
    _check(binding.load_library().flexmoe_step_cost(_p(tokens), _p(slot_owner), E, G, S, int(token_cost),
                                                    _p(sync_cost), ctypes.byref(cost)), "flexmoe_step_cost")
    return cost.value


def flexmoe_make_scheduling_plan(tokens, slot_owner, G: int, token_cost: int, sync_cost=None):
    """-> None (empty plan) or dict(e0, source, target, e1, released, t0, t1)"""
    tokens, slot_owner, E, G, S = _cluster(tokens, slot_owner, G)
    sync_cost = _sync(sync_cost, G)
    plan = np.zeros(5, dtype=np.int32)
    t = np.zeros(2, dtype=np.int64)
    has = ctypes.c_int()
    _check(binding.load_library().flexmoe_make_scheduling_plan(_p(tokens), _p(slot_owner), E, G, S, int(token_cost),
                                                               _p(sync_cost), _p(plan), _p(t), ctypes.byref(has)),
           "flexmoe_make_scheduling_plan")
    if not has.value:
        return None
    return {"e0": int(plan[0]), "source": int(plan[1]), "target": int(plan[2]), "e1": int(plan[3]),
            "released": int(plan[4]), "t0": int(t[0]), "t1": int(t[1])}


def flexmoe_schedule(tokens, slot_owner, G: int, token_cost: int, threshold: float, max_ops: int, sync_cost=None):
    """-> (ops [n,4] int32, new slot_owner, ratio_before, ratio_after); slot_owner is not modified"""
    tokens, slot_owner, E, G, S = _cluster(tokens, slot_owner, G)
    sync_cost = _sync(sync_cost, G)
    owner = slot_owner.copy()
    ops = np.zeros((max(int(max_ops), 1), 4), dtype=np.int32)
    n_ops = ctypes.c_int()
    before, after = ctypes.c_double(), ctypes.c_double()
    _check(binding.load_library().flexmoe_schedule(_p(tokens), _p(owner), E, G, S, int(token_cost), _p(sync_cost),
                                                   float(threshold), int(max_ops), _p(ops), ctypes.byref(n_ops),
                                                   ctypes.byref(before), ctypes.byref(after)), "flexmoe_schedule")
    return ops[:n_ops.value].copy(), owner, before.value, after.value


def flexmoe_placement_table(slot_owner, E: int):
    """-> (rep_off [E+1], rep_ids [V]) int32, the table flexmoe_route takes"""
    slot_owner = _i32(slot_owner)
    rep_off = np.zeros(E + 1, dtype=np.int32)
    rep_ids = np.zeros(slot_owner.size, dtype=np.int32)
    V = ctypes.c_int()
    _check(binding.load_library().flexmoe_placement_table(_p(slot_owner), int(E), int(slot_owner.size), _p(rep_off),
                                                          _p(rep_ids), ctypes.byref(V)), "flexmoe_placement_table")
    return rep_off, rep_ids[:V.value].copy()
