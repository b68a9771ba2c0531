"""Pins for the oracle's float results: Eq. 2 (expert FFN), Eq. 4 (weighted sum)
and the gradients of the expert path.  Expected values come from library
routines (torch CPU fp64: gelu, softmax, topk, autograd), closed forms, special
cases and finite differences.
"""
import math

import numpy as np
import pytest
import torch

from oracle import flexmoe_oracle as O
from paper_2304_03946_amd import workloads as W

torch.set_default_dtype(torch.float64)


def _small_problem(seed, N=37, d=12, f=20, E=5, k=2, bias=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, d))
    wg = rng.standard_normal((d, E))
    w1 = rng.standard_normal((E, d, f)) * 0.3
    w2 = rng.standard_normal((E, f, d)) * 0.3
    b1 = rng.standard_normal((E, f)) * 0.1 if bias else None
    b2 = rng.standard_normal((E, d)) * 0.1 if bias else None
    return x, wg, w1, b1, w2, b2


def _torch_act(z, act):
    if act == O.ACT_RELU:
        return torch.relu(z)
    if act == O.ACT_GELU_ERF:
        return torch.nn.functional.gelu(z)
    return torch.nn.functional.gelu(z, approximate="tanh")


def _dense_layer_torch(x, wg, w1, b1, w2, b2, k, act):
    """All experts evaluated on every token; Eq. 4 with the dense gate vector
    (zero outside the top-k).  Library ops only; shares nothing with routing."""
    logits = x @ wg
    tv, ti = torch.topk(logits, k, dim=1)
    g = torch.zeros_like(logits).scatter(1, ti, torch.softmax(tv, dim=1)).detach()
    y = torch.zeros_like(x)
    for e in range(w1.shape[0]):
        h = x @ w1[e] + (b1[e] if b1 is not None else 0.0)
        o = _torch_act(h, act) @ w2[e] + (b2[e] if b2 is not None else 0.0)
        y = y + g[:, e:e + 1] * o
    return y


# ------------------------------------------------------------------ activations
@pytest.mark.parametrize("act", [O.ACT_RELU, O.ACT_GELU_ERF, O.ACT_GELU_TANH])
def test_activation_matches_library(act):
    z = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(O.act_fn(z, act), _torch_act(torch.from_numpy(z), act).numpy(), rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("act", [O.ACT_GELU_ERF, O.ACT_GELU_TANH])
def test_activation_gradient_finite_difference(act):
    z = np.linspace(-5, 5, 101)
    h = 1e-6
    fd = (O.act_fn(z + h, act) - O.act_fn(z - h, act)) / (2 * h)
    np.testing.assert_allclose(O.act_grad(z, act), fd, rtol=0, atol=1e-8)


def test_relu_gradient_is_step():
    assert O.act_grad(np.array([-1.0, 0.0, 2.0]), O.ACT_RELU).tolist() == [0.0, 0.0, 1.0]


def test_gelu_closed_form_points():
    # GELU(0) = 0, GELU'(0) = 1/2, GELU(z) -> z for large z, Phi(1) = 0.841344746...
    assert O.act_fn(np.array([0.0]), O.ACT_GELU_ERF)[0] == 0.0
    assert O.act_grad(np.array([0.0]), O.ACT_GELU_ERF)[0] == 0.5
    np.testing.assert_allclose(O.act_fn(np.array([1.0]), O.ACT_GELU_ERF), [0.8413447460685429], rtol=1e-14)
    np.testing.assert_allclose(O.act_fn(np.array([12.0]), O.ACT_GELU_ERF), [12.0], rtol=1e-15)


# ------------------------------------------------------------------ forward
@pytest.mark.parametrize("act", [O.ACT_RELU, O.ACT_GELU_ERF, O.ACT_GELU_TANH])
@pytest.mark.parametrize("k", [1, 2, 5])
def test_definition_matches_dense_library_evaluation(act, k):
    x, wg, w1, b1, w2, b2 = _small_problem(10 + k)
    y = O.moe_layer_forward(x, wg, w1, b1, w2, b2, k, act)
    t = lambda a: None if a is None else torch.from_numpy(a)
    yd = _dense_layer_torch(t(x), t(wg), t(w1), t(b1), t(w2), t(b2), k, act).numpy()
    np.testing.assert_allclose(y, yd, rtol=1e-11, atol=1e-12)


def test_ffn_hand_example():
    # one expert, d=1, f=2, ReLU: W1 = [2, -1], b1 = [0, 0.5], W2 = [[3],[4]], b2 = [1]
    # x = 1  -> h = (2, -0.5) -> relu (2, 0) -> y = 6 + 1 = 7;  x = -1 -> h = (-2, 1.5) -> (0,1.5) -> 7
    w1 = np.array([[[2.0, -1.0]]])
    w2 = np.array([[[3.0], [4.0]]])
    hpre, yp = O.expert_ffn_fwd(np.array([[1.0], [-1.0]]), [0, 2], [0], w1, np.array([[0.0, 0.5]]),
                                w2, np.array([[1.0]]), O.ACT_RELU)
    assert hpre.tolist() == [[2.0, -0.5], [-2.0, 1.5]]
    assert yp.tolist() == [[7.0], [7.0]]


def _random_table(rng, E, V):
    n = np.ones(E, dtype=int)
    for _ in range(V - E):
        n[rng.integers(E)] += 1
    return np.concatenate([[0], np.cumsum(n)]).astype(np.int32), rng.permutation(V).astype(np.int32)


@pytest.mark.parametrize("seed", range(4))
def test_staged_path_is_independent_of_placement(seed):
    rng = np.random.default_rng(seed)
    x, wg, w1, b1, w2, b2 = _small_problem(seed, N=53, E=6, k=2)
    ref = O.moe_layer_forward(x, wg, w1, b1, w2, b2, 2, O.ACT_GELU_ERF)
    for V in (6, 9, 17):
        rep_off, rep_ids = _random_table(rng, 6, V)
        st = O.staged_forward(x, wg, w1, b1, w2, b2, 2, O.ACT_GELU_ERF, rep_off, rep_ids)
        np.testing.assert_allclose(st["y"], ref, rtol=1e-12, atol=1e-13)


def test_identity_experts_reproduce_input():
    # ReLU, f = 2d, W1 = [I, -I], W2 = [I; -I]  =>  e(x) = relu(x) - relu(-x) = x for every
    # expert, and the gate weights sum to one, so y = x whatever the routing.
    rng = np.random.default_rng(5)
    N, d, E, k = 40, 6, 4, 2
    x = rng.standard_normal((N, d))
    wg = rng.standard_normal((d, E))
    I = np.eye(d)
    w1 = np.tile(np.concatenate([I, -I], axis=1)[None], (E, 1, 1))
    w2 = np.tile(np.concatenate([I, -I], axis=0)[None], (E, 1, 1))
    np.testing.assert_allclose(O.moe_layer_forward(x, wg, w1, None, w2, None, k, O.ACT_RELU), x, atol=1e-14)
    st = O.staged_forward(x, wg, w1, None, w2, None, k, O.ACT_RELU, [0, 2, 3, 4, 7], [6, 0, 1, 2, 3, 4, 5])
    np.testing.assert_allclose(st["y"], x, atol=1e-14)
    np.testing.assert_allclose(st["topk_w"].sum(axis=1), 1.0, atol=1e-14)


def test_top1_output_is_selected_expert_unweighted():
    x, wg, w1, b1, w2, b2 = _small_problem(8, E=3)
    y = O.moe_layer_forward(x, wg, w1, b1, w2, b2, 1, O.ACT_RELU)
    sel = np.argmax(x @ wg, axis=1)
    for t in range(x.shape[0]):
        e = sel[t]
        ref = np.maximum(x[t] @ w1[e] + b1[e], 0) @ w2[e] + b2[e]
        np.testing.assert_allclose(y[t], ref, rtol=1e-12, atol=1e-13)


def test_oracle_accepts_bf16_storage():
    cfg = W.scaled(W.CONFIGS["bert"], N=32, d=16, f=32, E=4, V=6)
    inp = W.make_layer_inputs(cfg)
    y1 = O.moe_layer_forward(inp.x, inp.wg, inp.w1, None, inp.w2, None, 2, cfg.act)
    y2 = O.moe_layer_forward(W.decode(inp.x), W.decode(inp.wg), W.decode(inp.w1), None, W.decode(inp.w2), None, 2, cfg.act)
    assert np.array_equal(y1, y2)


# ------------------------------------------------------------------ backward
@pytest.mark.parametrize("act", [O.ACT_RELU, O.ACT_GELU_ERF, O.ACT_GELU_TANH])
def test_gradients_match_autograd_on_dense_formulation(act):
    x, wg, w1, b1, w2, b2 = _small_problem(21, N=29, bias=False)
    rng = np.random.default_rng(1)
    dy = rng.standard_normal(x.shape)
    dx, dw1, dw2 = O.moe_layer_backward(x, wg, w1, None, w2, 2, act, dy)
    tx = torch.from_numpy(x).requires_grad_(True)
    tw1 = torch.from_numpy(w1).requires_grad_(True)
    tw2 = torch.from_numpy(w2).requires_grad_(True)
    twg = torch.from_numpy(wg)
    # gate evaluated on a detached copy: gradient flows through the experts only
    logits = tx.detach() @ twg
    tv, ti = torch.topk(logits, 2, dim=1)
    g = torch.zeros_like(logits).scatter(1, ti, torch.softmax(tv, dim=1))
    y = torch.zeros_like(tx)
    for e in range(w1.shape[0]):
        y = y + g[:, e:e + 1] * (_torch_act(tx @ tw1[e], act) @ tw2[e])
    (y * torch.from_numpy(dy)).sum().backward()
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dw1, tw1.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dw2, tw2.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_gradients_finite_differences():
    x, wg, w1, b1, w2, b2 = _small_problem(33, N=9, d=4, f=6, E=3, k=2)
    rng = np.random.default_rng(2)
    dy = rng.standard_normal(x.shape)
    topk = O.gate_topk(x, wg, 2)[:2]
    act = O.ACT_GELU_ERF
    L = lambda x_, w1_, w2_: float((dy * O.moe_layer_forward(x_, wg, w1_, b1, w2_, b2, 2, act, topk=topk)).sum())
    dx, dw1, dw2 = O.moe_layer_backward(x, wg, w1, b1, w2, 2, act, dy, topk=topk)
    h = 1e-6
    for arr, grad, pos in ((x, dx, 0), (w1, dw1, 1), (w2, dw2, 2)):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            args = [x.copy(), w1.copy(), w2.copy()]
            args[pos][i] += h
            up = L(*args)
            args[pos][i] -= 2 * h
            dn = L(*args)
            assert abs((up - dn) / (2 * h) - grad[i]) <= 1e-6 * max(1.0, abs(grad[i])), (pos, i)


@pytest.mark.parametrize("seed", range(3))
def test_staged_backward_matches_definition_for_any_placement(seed):
    rng = np.random.default_rng(seed + 50)
    x, wg, w1, b1, w2, b2 = _small_problem(seed + 40, N=45, E=5, k=2, bias=False)
    dy = rng.standard_normal(x.shape)
    dx, dw1, dw2 = O.moe_layer_backward(x, wg, w1, None, w2, 2, O.ACT_GELU_ERF, dy)
    for V in (5, 11):
        rep_off, rep_ids = _random_table(rng, 5, V)
        fwd = O.staged_forward(x, wg, w1, None, w2, None, 2, O.ACT_GELU_ERF, rep_off, rep_ids)
        bwd = O.staged_backward(fwd, dy, w1, w2, 2, O.ACT_GELU_ERF)
        np.testing.assert_allclose(bwd["dx"], dx, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(bwd["dw1"], dw1, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(bwd["dw2"], dw2, rtol=1e-11, atol=1e-12)


def test_empty_expert_gets_zero_weight_gradient():
    x, wg, w1, b1, w2, b2 = _small_problem(60, N=10, E=4, k=1, bias=False)
    wg = wg.copy()
    wg[:, 3] = 0.0
    x = np.abs(x)
    wg[:, 0] = 5.0            # expert 0 always wins
    dy = np.ones_like(x)
    dx, dw1, dw2 = O.moe_layer_backward(x, wg, w1, None, w2, 1, O.ACT_RELU, dy)
    assert np.all(dw1[1:] == 0) and np.all(dw2[1:] == 0) and np.any(dw1[0] != 0)


def test_gradient_columns_match_full_gradient():
    x, wg, w1, b1, w2, b2 = _small_problem(70, N=31, E=4, k=2, bias=False)
    dy = np.random.default_rng(7).standard_normal(x.shape)
    idx, w, _ = O.gate_topk(x, wg, 2)
    _, dw1, dw2 = O.moe_layer_backward(x, wg, w1, None, w2, 2, O.ACT_GELU_ERF, dy)
    cols = np.array([0, 7, 19])
    for e in range(4):
        c1, r2 = O.expert_grad_columns(x, dy, idx, w, e, w1[e], w2[e], cols, O.ACT_GELU_ERF)
        np.testing.assert_allclose(c1, dw1[e][:, cols], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(r2, dw2[e][cols, :], rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ gate path and biases
def _staged_full(x, wg, w1, b1, w2, b2, k, act, dy, rep=None):
    E = w1.shape[0]
    rep_off, rep_ids = rep if rep is not None else W.identity_placement(E)
    fwd = O.staged_forward(x, wg, w1, b1, w2, b2, k, act, rep_off, rep_ids)
    return fwd, O.staged_backward(fwd, dy, w1, w2, k, act, x=x, wg=wg)


@pytest.mark.parametrize("act", [O.ACT_RELU, O.ACT_GELU_ERF, O.ACT_GELU_TANH])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_full_layer_gradients_match_autograd(act, k):
    """Everything trainable at once: autograd through topk -> softmax -> dense experts with the
    gate left attached gives dX (both paths), dW_g, dW1, dW2, db1, db2."""
    x, wg, w1, b1, w2, b2 = _small_problem(60 + k, N=31, E=5, k=k)
    dy = np.random.default_rng(3).standard_normal(x.shape)
    rng = np.random.default_rng(4)
    rep = _random_table(rng, 5, 8)
    _, g = _staged_full(x, wg, w1, b1, w2, b2, k, act, dy, rep)
    t = {n: torch.from_numpy(a).requires_grad_(True) for n, a in dict(x=x, wg=wg, w1=w1, b1=b1, w2=w2, b2=b2).items()}
    logits = t["x"] @ t["wg"]
    tv, ti = torch.topk(logits, k, dim=1)
    gate = torch.zeros_like(logits).scatter(1, ti, torch.softmax(tv, dim=1))
    y = torch.zeros_like(t["x"])
    for e in range(5):
        y = y + gate[:, e:e + 1] * (_torch_act(t["x"] @ t["w1"][e] + t["b1"][e], act) @ t["w2"][e] + t["b2"][e])
    (y * torch.from_numpy(dy)).sum().backward()
    for name, got in (("x", g["dx_total"]), ("wg", g["dwg"]), ("w1", g["dw1"]), ("w2", g["dw2"]),
                      ("b1", g["db1"]), ("b2", g["db2"])):
        np.testing.assert_allclose(got, t[name].grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=name)
    if k == 1:        # a single kept logit has gate value 1 whatever the logit: no gradient through the gate
        assert np.abs(g["dwg"]).max() == 0.0 and np.abs(g["dx_gate"]).max() == 0.0


def test_gate_weight_gradient_finite_differences():
    """Central differences in W_g with the selection left to the gate itself (steps far smaller
    than any logit margin of this problem, so the kept set does not change)."""
    x, wg, w1, b1, w2, b2 = _small_problem(71, N=11, d=5, f=7, E=4, k=2)
    dy = np.random.default_rng(5).standard_normal(x.shape)
    act = O.ACT_GELU_ERF
    assert O.topk_margin(O.gate_logits(x, wg), 2).min() > 1e-3
    _, g = _staged_full(x, wg, w1, b1, w2, b2, 2, act, dy)
    L = lambda wg_: float((dy * O.moe_layer_forward(x, wg_, w1, b1, w2, b2, 2, act)).sum())
    h = 1e-6
    for i in range(wg.shape[0]):
        for e in range(wg.shape[1]):
            up, dn = wg.copy(), wg.copy()
            up[i, e] += h
            dn[i, e] -= h
            fd = (L(up) - L(dn)) / (2 * h)
            assert abs(fd - g["dwg"][i, e]) <= 1e-6 * max(1.0, abs(g["dwg"][i, e])), (i, e)


def test_softmax_jacobian_properties():
    """The kept gate values sum to one, so their logit gradients sum to zero per token; a
    gradient that is the same for all kept experts moves nothing; two experts: closed form."""
    rng = np.random.default_rng(6)
    g = rng.random((50, 3))
    g /= g.sum(axis=1, keepdims=True)
    dg = rng.standard_normal((50, 3))
    dl = O.topk_softmax_bwd(g, dg)
    np.testing.assert_allclose(dl.sum(axis=1), 0.0, atol=1e-15)
    np.testing.assert_allclose(O.topk_softmax_bwd(g, np.ones_like(dg) * 2.5), 0.0, atol=1e-15)
    g2, dg2 = g[:, :2] / g[:, :2].sum(axis=1, keepdims=True), dg[:, :2]
    want0 = g2[:, 0] * g2[:, 1] * (dg2[:, 0] - dg2[:, 1])        # d sigmoid(l0 - l1) chain rule
    np.testing.assert_allclose(O.topk_softmax_bwd(g2, dg2)[:, 0], want0, rtol=1e-12, atol=1e-15)


def test_bias_gradients_are_bucket_column_sums_for_linear_experts():
    """Hand case: W2 = 0 makes dHpre vanish (db1 = 0) and db2_e the gate-weighted sum of dY over
    the tokens routed to e, whatever the placement."""
    x, wg, w1, b1, w2, b2 = _small_problem(81, N=23, E=4, k=2)
    dy = np.random.default_rng(7).standard_normal(x.shape)
    fwd, g = _staged_full(x, wg, w1, b1, np.zeros_like(w2), b2, 2, O.ACT_GELU_ERF, dy,
                          _random_table(np.random.default_rng(8), 4, 7))
    assert np.abs(g["db1"]).max() == 0.0
    want = np.zeros_like(b2)
    for t in range(x.shape[0]):
        for j in range(2):
            want[fwd["topk_idx"][t, j]] += fwd["topk_w"][t, j] * dy[t]
    np.testing.assert_allclose(g["db2"], want, rtol=1e-12, atol=1e-14)


def test_bias_gradient_columns_match_full_gradient():
    x, wg, w1, b1, w2, b2 = _small_problem(91, N=33, E=4, k=2, bias=False)
    dy = np.random.default_rng(9).standard_normal(x.shape)
    _, g = _staged_full(x, wg, w1, None, w2, None, 2, O.ACT_GELU_ERF, dy)
    idx, w, _ = O.gate_topk(x, wg, 2)
    cols = np.array([1, 8, 17])
    for e in range(4):
        c1, c2 = O.expert_bias_grad_columns(x, dy, idx, w, e, w1[e], w2[e], cols, O.ACT_GELU_ERF)
        np.testing.assert_allclose(c1, g["db1"][e][cols], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(c2, g["db2"][e], rtol=1e-12, atol=1e-13)
