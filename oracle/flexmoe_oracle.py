"""CPU oracle for the single-GPU FlexMoE MoE-layer hot path.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, fp64 numpy statement of
what the path computes, written from the paper (arXiv 2304.03946).  It shares no
code with the HIP library and must never be imported by the product path; only
the tests, the smoke check and the benchmark's `cpu_baseline` leg use it.

Two faces:

* the *definition* of the layer (Section 2.1, Eq. 2 expert FFN, Eq. 3 top-k gate,
  Eq. 4 gate-weighted sum) with no routing machinery at all -- `moe_layer_forward`
  and `moe_layer_backward`.  The paper's placement mechanism never changes this
  result (Section 3: replicating experts and re-partitioning their tokens leaves
  the model's definition untouched), so it is what every placement must reproduce;
* the *method's steps* in the paper's order (Section 3.1 workflow: gate ->
  router splits each expert's tokens over its replicas -> replicas compute ->
  results delivered back), with the vExpert rules of Section 3.2 (a vExpert
  replicates exactly one expert; an expert's tokens are partitioned evenly over
  its vExperts), Alg. 3 reduced to one GPU, and the expert-wise layout
  transformation of Section 4 -- `gate_topk`, `route`, `permute`,
  `expert_ffn_fwd`, `expert_ffn_bwd`, `combine`.

Readings of points the paper leaves open are stated where they are taken.
All functions take numpy arrays (any float dtype; tensors may also be objects
whose indexing yields arrays) and compute in float64.

Pins (tests/test_oracle_*.py): brute-force top-k and softmax against library
routines, closed-form replica shares, numpy bincount/stable argsort for the
identity placement, identity experts, independence of the placement table,
a dense all-experts evaluation, finite differences and torch.autograd (CPU,
fp64) for the gradients (expert path, gate path and biases).  No function here is
"parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf   # library routine: the error function

ACT_RELU, ACT_GELU_ERF, ACT_GELU_TANH = 0, 1, 2

def _f64(a):
    return np.asarray(a, dtype=np.float64)


# ---------------------------------------------------------------------------
# activation (Eq. 2 uses ReLU; the GELU variants are the benchmark configs')
# ---------------------------------------------------------------------------
def act_fn(z: np.ndarray, act: int) -> np.ndarray:
    if act == ACT_RELU:
        return np.where(z > 0.0, z, 0.0)
    if act == ACT_GELU_ERF:                    # z * Phi(z)
        return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))
    if act == ACT_GELU_TANH:
        return 0.5 * z * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)))
    raise ValueError("unknown activation")


def act_grad(z: np.ndarray, act: int) -> np.ndarray:
    if act == ACT_RELU:
        return np.where(z > 0.0, 1.0, 0.0)
    if act == ACT_GELU_ERF:                    # Phi(z) + z * phi(z)
        return 0.5 * (1.0 + _erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
    if act == ACT_GELU_TANH:
        c = math.sqrt(2.0 / math.pi)
        u = c * (z + 0.044715 * z ** 3)
        th = np.tanh(u)
        return 0.5 * (1.0 + th) + 0.5 * z * (1.0 - th * th) * c * (1.0 + 3.0 * 0.044715 * z * z)
    raise ValueError("unknown activation")


# ---------------------------------------------------------------------------
# Eq. 3: top-k gate
# ---------------------------------------------------------------------------
def gate_logits(x, wg) -> np.ndarray:
    """l = x . W_g  (Eq. 3's argument), [N, E] float64."""
    return _f64(x) @ _f64(wg)


def topk_from_logits(logits: np.ndarray, k: int):
    """Eq. 3: keep the k largest logits of each token, then softmax over the kept ones.

    Reading (the paper fixes no tie rule): larger logit first; equal logits ->
    lower expert index first; slot j of the output is the j-th in that order.
    Returns (idx int32 [N,k], weights float64 [N,k]).
    """
    logits = _f64(logits)
    N, E = logits.shape
    if not 1 <= k <= E:
        raise ValueError("need 1 <= k <= E")
    idx = np.empty((N, k), dtype=np.int32)
    w = np.empty((N, k), dtype=np.float64)
    for t in range(N):
        order = sorted(range(E), key=lambda e: (-logits[t, e], e))[:k]
        kept = logits[t, order]
        ex = np.exp(kept - kept.max())
        idx[t] = order
        w[t] = ex / ex.sum()
    return idx, w


def gate_topk(x, wg, k: int):
    """Eq. 3 end to end.  Returns (idx [N,k] int32, weights [N,k] f64, logits [N,E] f64)."""
    logits = gate_logits(x, wg)
    idx, w = topk_from_logits(logits, k)
    return idx, w, logits


def topk_margin(logits: np.ndarray, k: int) -> np.ndarray:
    """Smallest gap between neighbours among each token's k+1 largest logits.

    A token whose margin is below the accumulation error of a lower-precision
    gate may legitimately come out with another order or another k-th expert;
    tests use this to decide where index equality must hold bit for bit.
    """
    logits = _f64(logits)
    N, E = logits.shape
    s = -np.sort(-logits, axis=1)[:, :min(k + 1, E)]
    if s.shape[1] < 2:
        return np.full(N, np.inf)
    return np.min(s[:, :-1] - s[:, 1:], axis=1)


# ---------------------------------------------------------------------------
# Section 3.2 + Alg. 3 on one GPU: route
# ---------------------------------------------------------------------------
def check_placement(E: int, rep_off, rep_ids) -> int:
    """Validate the expert->vExpert table; return V.

    Section 3.2: every vExpert replicates exactly one expert, so the lists
    rep_ids[rep_off[e]:rep_off[e+1]] partition the slot ids 0..V-1; an expert
    without a vExpert could not take tokens, so each list is non-empty.
    """
    rep_off = np.asarray(rep_off)
    rep_ids = np.asarray(rep_ids)
    if rep_off.shape != (E + 1,) or rep_off[0] != 0:
        raise ValueError("bad rep_off")
    V = int(rep_off[E])
    if np.any(np.diff(rep_off) < 1):
        raise ValueError("an expert has no vExpert")
    if rep_ids.shape != (V,) or sorted(rep_ids.tolist()) != list(range(V)):
        raise ValueError("rep_ids is not a permutation of 0..V-1")
    return V


def replica_shares(I_e: int, n_e: int):
    """Even partition of I_e tokens over n_e vExperts (Section 3.2, cap_e = I_e/n_e of Alg. 3).

    Reading: cap_e is real-valued in the paper; shares are its floor or ceiling,
    the first (I_e mod n_e) replicas taking the extra token.
    """
    q, m = divmod(I_e, n_e)
    return [q + (1 if r < m else 0) for r in range(n_e)]


def route(topk_idx, E: int, rep_off, rep_ids):
    """Router on one GPU.

    With a single GPU Alg. 3's locality-first branch keeps every token
    (r_{e,g} = I_e, nothing is sent away); what remains is the split of each
    expert's tokens over its own vExperts and the layout of the contiguous
    per-vExpert buckets (Section 4, expert-wise layout transformation).

    Assignment id a = t*k + j.  Readings: an expert's assignments are taken in
    ascending a and cut into contiguous chunks, one per replica in list order;
    buckets are laid out in ascending vExpert id; inside a bucket assignments
    keep ascending a.

    Returns dict with int32 arrays: expert_count[E], vexpert_count[V],
    vexpert_off[V+1], vexpert_owner[V], dest[A], src[A].
    """
    topk_idx = np.asarray(topk_idx)
    N, k = topk_idx.shape
    A = N * k
    V = check_placement(E, rep_off, rep_ids)
    flat = topk_idx.reshape(A)
    if A and (flat.min() < 0 or flat.max() >= E):
        raise ValueError("expert id out of range")

    # step 1-2: loads I_e and the stable rank of each assignment inside its expert
    expert_count = [0] * E
    rank = [0] * A
    for a in range(A):
        e = int(flat[a])
        rank[a] = expert_count[e]
        expert_count[e] += 1

    # step 3: shares per replica, owner of every vExpert
    vexpert_count = [0] * V
    vexpert_owner = [0] * V
    start_in_expert = [0] * V
    for e in range(E):
        ids = [int(v) for v in rep_ids[rep_off[e]:rep_off[e + 1]]]
        shares = replica_shares(expert_count[e], len(ids))
        run = 0
        for v, s in zip(ids, shares):
            vexpert_owner[v] = e
            vexpert_count[v] = s
            start_in_expert[v] = run
            run += s

    # step 5: bucket offsets in ascending vExpert id
    vexpert_off = [0] * (V + 1)
    for v in range(V):
        vexpert_off[v + 1] = vexpert_off[v] + vexpert_count[v]

    # step 4 + 6: the replica whose chunk holds rank(a), and the slot inside its bucket
    dest = [0] * A
    src = [0] * A
    for a in range(A):
        e = int(flat[a])
        for v in (int(u) for u in rep_ids[rep_off[e]:rep_off[e + 1]]):
            if start_in_expert[v] <= rank[a] < start_in_expert[v] + vexpert_count[v]:
                p = vexpert_off[v] + rank[a] - start_in_expert[v]
                dest[a] = p
                src[p] = a
                break
        else:  # pragma: no cover - unreachable when shares sum to I_e
            raise AssertionError("assignment not covered by any replica")

    i32 = lambda l: np.asarray(l, dtype=np.int32)
    return dict(expert_count=i32(expert_count), vexpert_count=i32(vexpert_count),
                vexpert_off=i32(vexpert_off), vexpert_owner=i32(vexpert_owner),
                dest=i32(dest), src=i32(src))


# ---------------------------------------------------------------------------
# Section 4: expert-wise layout transformation, and its reverse with Eq. 4
# ---------------------------------------------------------------------------
def permute(x, src, k: int, row_scale=None) -> np.ndarray:
    """Xp[p,:] = x[src[p] // k, :] (times row_scale[src[p]] when given)."""
    x = _f64(x)
    src = np.asarray(src)
    xp = np.empty((src.shape[0], x.shape[1]), dtype=np.float64)
    for p in range(src.shape[0]):
        a = int(src[p])
        xp[p] = x[a // k]
        if row_scale is not None:
            xp[p] = xp[p] * float(row_scale[a])
    return xp


def combine(yp, dest, topk_w, k: int) -> np.ndarray:
    """Eq. 4 through the reverse routing: y[t,:] = sum_j w[t,j] * Yp[dest[t*k+j],:]
    (weights None -> 1, which is the gradient of `permute` w.r.t. x)."""
    yp = _f64(yp)
    dest = np.asarray(dest)
    N = dest.shape[0] // k
    y = np.zeros((N, yp.shape[1]), dtype=np.float64)
    wflat = None if topk_w is None else _f64(topk_w).reshape(-1)
    for t in range(N):
        for j in range(k):
            a = t * k + j
            g = 1.0 if wflat is None else wflat[a]
            y[t] += g * yp[int(dest[a])]
    return y


# ---------------------------------------------------------------------------
# Eq. 2 per vExpert bucket (what each replica computes, Section 3.1 step 3)
# ---------------------------------------------------------------------------
def expert_ffn_fwd(xp, vexpert_off, vexpert_owner, w1, b1, w2, b2, act: int):
    """For bucket v owned by e: Hpre = Xp_v.W1_e + b1_e, Yp_v = act(Hpre).W2_e + b2_e.
    Row-vector form of Eq. 2 (W1 is [d,f], W2 is [f,d]).  Returns (hpre [A,f], yp [A,d])."""
    xp = _f64(xp)
    A, d = xp.shape
    V = len(vexpert_owner)
    f = np.asarray(w1[0]).shape[1]
    hpre = np.zeros((A, f), dtype=np.float64)
    yp = np.zeros((A, d), dtype=np.float64)
    for v in range(V):
        lo, hi = int(vexpert_off[v]), int(vexpert_off[v + 1])
        if hi == lo:
            continue
        e = int(vexpert_owner[v])
        h = xp[lo:hi] @ _f64(w1[e])
        if b1 is not None:
            h = h + _f64(b1[e])[None, :]
        hpre[lo:hi] = h
        o = act_fn(h, act) @ _f64(w2[e])
        if b2 is not None:
            o = o + _f64(b2[e])[None, :]
        yp[lo:hi] = o
    return hpre, yp


def expert_ffn_bwd(dyp, xp, hpre, w1, w2, vexpert_off, vexpert_owner, E: int, act: int):
    """Gradients of Eq. 2 per bucket; an expert's weight gradient is the sum over
    its vExperts (the paper's replicas synchronise gradients, Section 2.3 T_Sync;
    vExperts of one expert on one GPU share weights, Section 3.2).

    dH = dYp.W2^T, dHpre = dH * act'(Hpre), dW2_e += act(Hpre_v)^T.dYp_v,
    dW1_e += Xp_v^T.dHpre_v, dXp = dHpre.W1^T.
    Returns (dxp [A,d], dw1 [E,d,f], dw2 [E,f,d]); experts without tokens get zeros.
    """
    dyp, xp, hpre = _f64(dyp), _f64(xp), _f64(hpre)
    A, d = xp.shape
    f = hpre.shape[1]
    dxp = np.zeros((A, d), dtype=np.float64)
    dw1 = np.zeros((E, d, f), dtype=np.float64)
    dw2 = np.zeros((E, f, d), dtype=np.float64)
    for v in range(len(vexpert_owner)):
        lo, hi = int(vexpert_off[v]), int(vexpert_off[v + 1])
        if hi == lo:
            continue
        e = int(vexpert_owner[v])
        W1, W2 = _f64(w1[e]), _f64(w2[e])
        dh = dyp[lo:hi] @ W2.T
        dhpre = dh * act_grad(hpre[lo:hi], act)
        dw2[e] += act_fn(hpre[lo:hi], act).T @ dyp[lo:hi]
        dw1[e] += xp[lo:hi].T @ dhpre
        dxp[lo:hi] = dhpre @ W1.T
    return dxp, dw1, dw2


# ---------------------------------------------------------------------------
# the rest of a trainable layer: gradient through the gate (Eq. 3-4), bias gradients (Eq. 2)
# ---------------------------------------------------------------------------
def gate_value_grad(dy, yp, dest, k: int) -> np.ndarray:
    """Eq. 4 is linear in the gate values: dL/dg[t,j] = <dY_t, Yp[dest[t*k+j]]>, where
    Yp holds the experts' outputs (bias b2 included) in bucket order.  Returns [N,k]."""
    dy, yp = _f64(dy), _f64(yp)
    dest = np.asarray(dest)
    N = dest.shape[0] // k
    dg = np.zeros((N, k), dtype=np.float64)
    for t in range(N):
        for j in range(k):
            dg[t, j] = float(np.dot(dy[t], yp[int(dest[t * k + j])]))
    return dg


def topk_softmax_bwd(topk_w, dg) -> np.ndarray:
    """Gradient w.r.t. the k kept logits of Eq. 3 (the discarded logits get none: their gate
    value is identically zero).  Softmax Jacobian: dl_j = g_j * (dg_j - sum_i g_i dg_i)."""
    g, dg = _f64(topk_w), _f64(dg)
    inner = (g * dg).sum(axis=1, keepdims=True)
    return g * (dg - inner)


def gate_bwd(x, wg, topk_idx, topk_w, dy, yp, dest):
    """Backward of the gate path for an upstream dY.  The logits are l = x.W_g, so with dl
    scattered to the selected experts' columns: dW_g = X^T.dl and dX_gate = dl.W_g^T.
    Returns (dl [N,k], dwg [d,E], dx_gate [N,d]); dx_gate adds to the expert-path dX."""
    x, wg = _f64(x), _f64(wg)
    idx = np.asarray(topk_idx)
    N, k = idx.shape
    dl = topk_softmax_bwd(topk_w, gate_value_grad(dy, yp, dest, k))
    dwg = np.zeros_like(wg)
    dxg = np.zeros_like(x)
    for t in range(N):
        for j in range(k):
            e = int(idx[t, j])
            dwg[:, e] += dl[t, j] * x[t]
            dxg[t] += dl[t, j] * wg[:, e]
    return dl, dwg, dxg


def expert_bias_grads(dyp, hpre, w2, vexpert_off, vexpert_owner, E: int, act: int):
    """db2_e = sum of the rows of dYp in e's buckets; db1_e = sum of the rows of
    dHpre = (dYp.W2_e^T) * act'(Hpre) there (b1 enters Hpre, b2 enters Yp, both with unit
    coefficient).  Returns (db1 [E,f], db2 [E,d])."""
    dyp, hpre = _f64(dyp), _f64(hpre)
    db1 = np.zeros((E, hpre.shape[1]), dtype=np.float64)
    db2 = np.zeros((E, dyp.shape[1]), dtype=np.float64)
    for v in range(len(vexpert_owner)):
        lo, hi = int(vexpert_off[v]), int(vexpert_off[v + 1])
        if hi == lo:
            continue
        e = int(vexpert_owner[v])
        dhpre = (dyp[lo:hi] @ _f64(w2[e]).T) * act_grad(hpre[lo:hi], act)
        db1[e] += dhpre.sum(axis=0)
        db2[e] += dyp[lo:hi].sum(axis=0)
    return db1, db2


# ---------------------------------------------------------------------------
# the method end to end, step by step
# ---------------------------------------------------------------------------
def staged_forward(x, wg, w1, b1, w2, b2, k: int, act: int, rep_off, rep_ids, topk=None):
    """gate -> route -> permute -> per-vExpert FFN -> combine.  `topk` = (idx, w)
    replaces the gate (used to follow a lower-precision gate's own decisions)."""
    E = len(rep_off) - 1
    if topk is None:
        idx, w, _ = gate_topk(x, wg, k)
    else:
        idx, w = topk
    r = route(idx, E, rep_off, rep_ids)
    xp = permute(x, r["src"], k)
    hpre, yp = expert_ffn_fwd(xp, r["vexpert_off"], r["vexpert_owner"], w1, b1, w2, b2, act)
    y = combine(yp, r["dest"], w, k)
    return dict(topk_idx=idx, topk_w=w, route=r, xp=xp, hpre=hpre, yp=yp, y=y)


def staged_backward(fwd: dict, dy, w1, w2, k: int, act: int, x=None, wg=None):
    """Backward of the expert path for an upstream gradient dY (gate weights held
    constant): dYp = permute(dY, scale = gate weights); FFN backward per bucket;
    dX = combine(dXp, weights = 1).  With x and W_g given, also the gate path and the bias
    gradients: dl, dwg, dx_gate (dx_total = dx + dx_gate), db1, db2."""
    r = fwd["route"]
    E = r["expert_count"].shape[0]
    dyp = permute(dy, r["src"], k, row_scale=_f64(fwd["topk_w"]).reshape(-1))
    dxp, dw1, dw2 = expert_ffn_bwd(dyp, fwd["xp"], fwd["hpre"], w1, w2,
                                   r["vexpert_off"], r["vexpert_owner"], E, act)
    dx = combine(dxp, r["dest"], None, k)
    out = dict(dyp=dyp, dxp=dxp, dw1=dw1, dw2=dw2, dx=dx)
    if x is not None:
        dl, dwg, dxg = gate_bwd(x, wg, fwd["topk_idx"], fwd["topk_w"], dy, fwd["yp"], r["dest"])
        db1, db2 = expert_bias_grads(dyp, fwd["hpre"], w2, r["vexpert_off"], r["vexpert_owner"], E, act)
        out.update(dl=dl, dwg=dwg, dx_gate=dxg, dx_total=dx + dxg, db1=db1, db2=db2)
    return out


# ---------------------------------------------------------------------------
# the definition (Eq. 2-4), no routing machinery
# ---------------------------------------------------------------------------
def moe_layer_forward(x, wg, w1, b1, w2, b2, k: int, act: int, topk=None) -> np.ndarray:
    """y_t = sum_{e in S_t} g_{t,e} * (act(x_t.W1_e + b1_e).W2_e + b2_e)  (Eq. 4 with
    the gate of Eq. 3 and the expert of Eq. 2; experts outside the top-k have g = 0
    and are skipped).  Summed expert by expert over the tokens that selected it."""
    x = _f64(x)
    N, d = x.shape
    if topk is None:
        idx, w, _ = gate_topk(x, wg, k)
    else:
        idx, w = np.asarray(topk[0]), _f64(topk[1])
    E = len(w1)
    y = np.zeros((N, d), dtype=np.float64)
    for e in range(E):
        tok, slot = np.nonzero(idx == e)
        if tok.size == 0:
            continue
        h = x[tok] @ _f64(w1[e])
        if b1 is not None:
            h = h + _f64(b1[e])[None, :]
        o = act_fn(h, act) @ _f64(w2[e])
        if b2 is not None:
            o = o + _f64(b2[e])[None, :]
        np.add.at(y, tok, w[tok, slot][:, None] * o)
    return y


def moe_layer_backward(x, wg, w1, b1, w2, k: int, act: int, dy, topk=None):
    """Gradients of L = sum(dY * y) w.r.t. x (through the experts only), W1, W2,
    with the gate's output held constant.  Returns (dx [N,d], dw1 [E,d,f], dw2 [E,f,d])."""
    x, dy = _f64(x), _f64(dy)
    N, d = x.shape
    if topk is None:
        idx, w, _ = gate_topk(x, wg, k)
    else:
        idx, w = np.asarray(topk[0]), _f64(topk[1])
    E = len(w1)
    f = np.asarray(w1[0]).shape[1]
    dx = np.zeros((N, d), dtype=np.float64)
    dw1 = np.zeros((E, d, f), dtype=np.float64)
    dw2 = np.zeros((E, f, d), dtype=np.float64)
    for e in range(E):
        tok, slot = np.nonzero(idx == e)
        if tok.size == 0:
            continue
        W1, W2 = _f64(w1[e]), _f64(w2[e])
        h = x[tok] @ W1
        if b1 is not None:
            h = h + _f64(b1[e])[None, :]
        do = w[tok, slot][:, None] * dy[tok]          # d L / d e(x_t)
        dh = (do @ W2.T) * act_grad(h, act)
        dw2[e] = act_fn(h, act).T @ do
        dw1[e] = x[tok].T @ dh
        np.add.at(dx, tok, dh @ W1.T)
    return dx, dw1, dw2


def expert_grad_columns(x, dy, idx, w, e: int, w1_e, w2_e, cols, act: int):
    """Columns `cols` of dW1_e ([d,|cols|]) and the matching rows of dW2_e ([|cols|,d])
    from the definition: each hidden unit j of Eq. 2 depends only on column j of W1_e
    and row j of W2_e, so the sums over the expert's tokens can be taken for a few
    hidden units alone (full-size parity samples)."""
    x, dy = _f64(x), _f64(dy)
    idx, w = np.asarray(idx), _f64(w)
    cols = np.asarray(cols)
    tok, slot = np.nonzero(idx == e)
    d = x.shape[1]
    if tok.size == 0:
        return np.zeros((d, cols.size)), np.zeros((cols.size, d))
    W1c = _f64(w1_e)[:, cols]
    W2r = _f64(w2_e)[cols, :]
    h = x[tok] @ W1c
    do = w[tok, slot][:, None] * dy[tok]
    dh = (do @ W2r.T) * act_grad(h, act)
    return x[tok].T @ dh, act_fn(h, act).T @ do


def expert_bias_grad_columns(x, dy, idx, w, e: int, w1_e, w2_e, cols, act: int):
    """Entries `cols` of db1_e and the whole of db2_e from the definition (no biases in the
    forward pass): db2_e is the gate-weighted sum of dY over the tokens that selected e, and
    hidden unit j of db1_e needs only column j of W1_e and row j of W2_e (full-size samples)."""
    x, dy = _f64(x), _f64(dy)
    idx, w = np.asarray(idx), _f64(w)
    cols = np.asarray(cols)
    tok, slot = np.nonzero(idx == e)
    if tok.size == 0:
        return np.zeros(cols.size), np.zeros(x.shape[1])
    h = x[tok] @ _f64(w1_e)[:, cols]
    do = w[tok, slot][:, None] * dy[tok]
    dh = (do @ _f64(w2_e)[cols, :].T) * act_grad(h, act)
    return dh.sum(axis=0), do.sum(axis=0)
