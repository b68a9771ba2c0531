"""Pins for the oracle's gate (Eq. 3) and router (Section 3.2, Alg. 3 on one GPU).

Every expected value here comes from the mathematics, a library routine, a hand
computation spelled out in the test, or the paper's own worked example -- never
from the HIP path and never from the oracle itself.
"""
import os

import numpy as np
import pytest
import torch

from oracle import flexmoe_oracle as O
from paper_2304_03946_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ gate (Eq. 3)
def test_gate_logits_hand_example():
    # x = [1 2], W_g = [[1 0 2],[0 1 3]]  ->  x.W_g = [1, 2, 8]; a transposed operand
    # or a swapped index cannot give this.
    x = np.array([[1.0, 2.0]])
    wg = np.array([[1.0, 0.0, 2.0], [0.0, 1.0, 3.0]])
    assert O.gate_logits(x, wg).tolist() == [[1.0, 2.0, 8.0]]


def test_topk_closed_form_weights():
    # logits (0, ln 3, -5): top-2 keeps ln 3 then 0 -> softmax = (3/4, 1/4), in that order
    idx, w = O.topk_from_logits(np.array([[0.0, np.log(3.0), -5.0]]), 2)
    assert idx.tolist() == [[1, 0]]
    np.testing.assert_allclose(w, [[0.75, 0.25]], rtol=0, atol=1e-15)


def test_topk_tie_break_lower_index_first():
    idx, w = O.topk_from_logits(np.array([[1.0, 3.0, 3.0, 0.0], [2.0, 2.0, 2.0, 2.0]]), 3)
    assert idx.tolist() == [[1, 2, 0], [0, 1, 2]]
    np.testing.assert_allclose(w[1], [1 / 3, 1 / 3, 1 / 3], atol=1e-15)


def test_topk_k1_weight_is_exactly_one():
    rng = np.random.default_rng(0)
    idx, w = O.topk_from_logits(rng.standard_normal((50, 7)), 1)
    assert np.all(w == 1.0)


@pytest.mark.parametrize("E,k", [(4, 1), (5, 2), (16, 2), (8, 8), (64, 3)])
def test_topk_matches_library_topk_and_softmax(E, k):
    rng = np.random.default_rng(E * 100 + k)
    logits = rng.standard_normal((200, E))
    idx, w = O.topk_from_logits(logits, k)
    tv, ti = torch.topk(torch.from_numpy(logits), k, dim=1)      # no ties in random doubles
    assert np.array_equal(idx, ti.numpy().astype(np.int32))
    np.testing.assert_allclose(w, torch.softmax(tv, dim=1).numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-14)
    # every token lands in k distinct experts
    assert all(len(set(r)) == k for r in idx.tolist())


def test_topk_k_equals_E_is_full_softmax():
    rng = np.random.default_rng(3)
    logits = rng.standard_normal((20, 6))
    idx, w = O.topk_from_logits(logits, 6)
    full = torch.softmax(torch.from_numpy(logits), dim=1).numpy()
    np.testing.assert_allclose(w, np.take_along_axis(full, idx.astype(np.int64), axis=1), rtol=1e-13)


def test_topk_rejects_bad_k():
    with pytest.raises(ValueError):
        O.topk_from_logits(np.zeros((2, 3)), 4)
    with pytest.raises(ValueError):
        O.topk_from_logits(np.zeros((2, 3)), 0)


def test_topk_margin_hand_example():
    m = O.topk_margin(np.array([[5.0, 1.0, 4.5, 4.0], [0.0, 0.0, 9.0, 1.0]]), 2)
    assert m.tolist() == [0.5, 0.0 + 1.0]      # (5-4.5, 4.5-4) ; (9-1, 1-0)


# ------------------------------------------------------------------ replica split
def test_replica_shares_hand_examples():
    assert O.replica_shares(10, 4) == [3, 3, 2, 2]
    assert O.replica_shares(2, 4) == [1, 1, 0, 0]
    assert O.replica_shares(0, 3) == [0, 0, 0]
    assert O.replica_shares(7, 1) == [7]


def test_replica_shares_even_partition_properties():
    for I in range(0, 70):
        for n in range(1, 9):
            s = O.replica_shares(I, n)
            assert sum(s) == I and max(s) - min(s) <= 1
            assert all(x in (I // n, -(-I // n)) for x in s)        # floor or ceil of cap_e
            assert s == sorted(s, reverse=True)                      # extras go first


# ------------------------------------------------------------------ route
def test_route_hand_worked_example():
    # 5 tokens, k=1, experts (0,1,0,0,1).  Expert 0 owns vExperts [2, 0] (in that
    # replica order), expert 1 owns [1].  I_0 = 3 -> shares (2,1): vExpert 2 takes
    # ranks 0,1 (a=0,2), vExpert 0 takes rank 2 (a=3).  Buckets ascend by vExpert id:
    # v0=[a3] at 0, v1=[a1,a4] at 1, v2=[a0,a2] at 3.
    r = O.route(np.array([[0], [1], [0], [0], [1]]), 2, [0, 2, 3], [2, 0, 1])
    assert r["expert_count"].tolist() == [3, 2]
    assert r["vexpert_count"].tolist() == [1, 2, 2]
    assert r["vexpert_off"].tolist() == [0, 1, 3, 5]
    assert r["vexpert_owner"].tolist() == [0, 1, 0]
    assert r["dest"].tolist() == [3, 1, 4, 0, 2]
    assert r["src"].tolist() == [3, 1, 4, 0, 2]


def test_route_reproduces_paper_fig1b_loads():
    with open(os.path.join(GOLDEN, "fig1b_expert_loads.txt")) as fh:
        row = [l for l in fh if l.strip() and not l.startswith("#")][0].split()
    a0, a1, b0, b1, load0, load1 = map(int, row)
    idx = np.array([0] * a0 + [1] * a1 + [0] * b0 + [1] * b1, dtype=np.int32)[:, None]
    r = O.route(idx, 2, *W.identity_placement(2))
    assert r["expert_count"].tolist() == [load0, load1]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_route_identity_placement_is_histogram_and_stable_sort(seed):
    rng = np.random.default_rng(seed)
    E, N, k = 6, 97, 2
    idx = np.stack([rng.permutation(E)[:k] for _ in range(N)]).astype(np.int32)
    r = O.route(idx, E, *W.identity_placement(E))
    flat = idx.reshape(-1)
    assert np.array_equal(r["expert_count"], np.bincount(flat, minlength=E))
    assert np.array_equal(r["vexpert_count"], r["expert_count"])
    assert np.array_equal(r["src"], np.argsort(flat, kind="stable"))
    assert np.array_equal(r["vexpert_off"], np.concatenate([[0], np.cumsum(np.bincount(flat, minlength=E))]))


def _random_table(rng, E, V):
    n = np.ones(E, dtype=int)
    for _ in range(V - E):
        n[rng.integers(E)] += 1
    rep_off = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    rep_ids = rng.permutation(V).astype(np.int32)
    return rep_off, rep_ids


@pytest.mark.parametrize("seed", range(6))
def test_route_invariants_random_tables(seed):
    rng = np.random.default_rng(100 + seed)
    E = int(rng.integers(2, 9))
    V = E + int(rng.integers(0, 7))
    k = int(rng.integers(1, min(E, 3) + 1))
    N = int(rng.integers(1, 120))
    p = rng.dirichlet(np.full(E, 0.3))
    idx = np.stack([rng.choice(E, size=k, replace=False, p=p * 0.9 + 0.1 / E) for _ in range(N)]).astype(np.int32)
    rep_off, rep_ids = _random_table(rng, E, V)
    r = O.route(idx, E, rep_off, rep_ids)
    A = N * k
    flat = idx.reshape(-1)
    # no token dropped: loads and buckets both sum to N*k
    assert r["expert_count"].sum() == A and r["vexpert_count"].sum() == A
    assert np.array_equal(r["expert_count"], np.bincount(flat, minlength=E))
    assert r["vexpert_off"][0] == 0 and r["vexpert_off"][V] == A
    assert np.array_equal(np.diff(r["vexpert_off"]), r["vexpert_count"])
    # dest is a permutation and src is its inverse
    assert sorted(r["dest"].tolist()) == list(range(A))
    assert np.array_equal(r["src"][r["dest"]], np.arange(A))
    for e in range(E):
        ids = rep_ids[rep_off[e]:rep_off[e + 1]]
        shares = r["vexpert_count"][ids]
        assert shares.tolist() == O.replica_shares(int(r["expert_count"][e]), len(ids))
        assert np.all(r["vexpert_owner"][ids] == e)
        # replicas in list order hold contiguous chunks of the expert's assignments in
        # ascending assignment id
        chain = np.concatenate([r["src"][r["vexpert_off"][v]:r["vexpert_off"][v + 1]] for v in ids])
        assert np.array_equal(chain, np.nonzero(flat == e)[0])


def test_route_degenerate_cases():
    # all tokens to one expert with more replicas than tokens; other experts empty
    r = O.route(np.array([[1], [1]]), 3, [0, 1, 5, 6], [0, 1, 2, 3, 4, 5])
    assert r["expert_count"].tolist() == [0, 2, 0]
    assert r["vexpert_count"].tolist() == [0, 1, 1, 0, 0, 0]
    assert r["dest"].tolist() == [0, 1]
    # empty batch
    r = O.route(np.zeros((0, 2), dtype=np.int32), 2, [0, 1, 2], [0, 1])
    assert r["vexpert_off"].tolist() == [0, 0, 0] and r["dest"].size == 0


@pytest.mark.parametrize("off,ids", [([0, 1, 1], [0]), ([0, 1, 3], [0, 1, 1]), ([1, 2, 3], [0, 1, 2]),
                                     ([0, 2, 3], [0, 1, 3])])
def test_route_rejects_bad_tables(off, ids):
    with pytest.raises(ValueError):
        O.route(np.array([[0]]), 2, off, ids)


def test_route_rejects_bad_expert_id():
    with pytest.raises(ValueError):
        O.route(np.array([[2]]), 2, [0, 1, 2], [0, 1])


# ------------------------------------------------------------------ permute / combine
def test_permute_combine_hand_example():
    x = np.array([[1.0, 10.0], [2.0, 20.0], [3.0, 30.0]])
    # k = 2: assignments a=0..5 belong to tokens 0,0,1,1,2,2
    src = np.array([4, 0, 3, 1, 5, 2])
    xp = O.permute(x, src, 2)
    assert xp[:, 0].tolist() == [3.0, 1.0, 2.0, 1.0, 3.0, 2.0]
    scaled = O.permute(x, src, 2, row_scale=np.array([0.5, 1, 1, 1, 2, 1.0]))
    assert scaled[:2].tolist() == [[6.0, 60.0], [0.5, 5.0]]
    dest = np.empty(6, dtype=int)
    dest[src] = np.arange(6)
    w = np.array([[0.25, 0.75], [1.0, 0.0], [0.5, 0.5]])
    # gate weights sum to one, so combining the permuted copies returns x
    np.testing.assert_allclose(O.combine(xp, dest, w, 2), x, atol=1e-15)
    # without weights the k copies add up
    np.testing.assert_allclose(O.combine(xp, dest, None, 2), 2 * x, atol=1e-15)
