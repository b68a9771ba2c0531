"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot evaluate a whole 65536-token GPT-XL-like layer in seconds, so outputs
are checked on samples it can compute one by one: tokens are independent of each other
(Eq. 2-4), and every hidden unit of an expert's weight gradient is a sum over that
expert's tokens that can be evaluated alone.  Routing artefacts are compared in full,
bit for bit.
"""
import numpy as np
import pytest
import torch

from oracle import flexmoe_oracle as O
from paper_2304_03946_amd import workloads as W
from test_gpu_parity import TOL, api, check_gate, host, rel_err, upload  # noqa: F401

pytestmark = pytest.mark.gpu


def _rows_by_bucket(r, rng, per_bucket=3, max_buckets=24):
    V = r["vexpert_count"].shape[0]
    nonempty = [v for v in range(V) if r["vexpert_count"][v] > 0]
    pick = sorted(set(nonempty[:2] + nonempty[-2:] + list(rng.choice(nonempty, size=min(max_buckets, len(nonempty)), replace=False))))
    rows = []
    for v in pick:
        lo, hi = int(r["vexpert_off"][v]), int(r["vexpert_off"][v + 1])
        rows += [lo, hi - 1] + list(rng.integers(lo, hi, size=per_bucket))
    return np.array(sorted(set(rows)))


@pytest.mark.parametrize("name", ["bert", "gpt_m", "swin", "gpt_xl"])
def test_full_config_sampled(api, name):
    binding, layer_mod = api
    cfg = W.CONFIGS[name]
    tol = TOL[cfg.dtype]
    print(f"[fullsize] {name}: generating inputs", flush=True)
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    L = layer_mod.MoELayer.for_config(cfg)
    k, E = cfg.k, cfg.E
    # the table comes from the loads observed on a first pass, as the paper's scheduler would see them
    rep_off, rep_ids = W.config_placement(cfg)
    L.gate(dev["x"], dev["wg"])
    L.route(rep_off, rep_ids)
    torch.cuda.synchronize()
    if name != "bert":
        rep_off, rep_ids = W.placement_from_loads(host(L.expert_count), cfg.V, cfg.max_rep)
    print(f"[fullsize] {name}: forward", flush=True)
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], rep_off, rep_ids)
    torch.cuda.synchronize()
    rng = np.random.default_rng(cfg.cfg_id)
    idx_gpu, w_gpu = host(L.topk_idx), host(L.topk_w)

    tok = np.unique(np.concatenate([[0, cfg.N - 1], rng.integers(0, cfg.N, size=2048)]))
    same = check_gate(idx_gpu[tok], w_gpu[tok], inp.x, inp.wg, k, cfg.dtype, tokens=tok)

    print(f"[fullsize] {name}: route", flush=True)
    r = O.route(idx_gpu, E, rep_off, rep_ids)
    for nm in ("expert_count", "vexpert_count", "vexpert_off", "vexpert_owner", "dest", "src"):
        assert np.array_equal(host(getattr(L, nm)), r[nm]), nm
    assert r["vexpert_count"].sum() == cfg.A

    xd = W.decode(inp.x)
    rows = _rows_by_bucket(r, rng)
    rows_t = torch.from_numpy(rows).cuda()
    xp_rows = host(L.xp[rows_t])
    assert np.array_equal(xp_rows, xd[r["src"][rows] // k]), "permute is not an exact copy"
    more = rng.integers(0, cfg.A, size=4096)
    assert np.array_equal(host(L.xp[torch.from_numpy(more).cuda()]), xd[r["src"][more] // k])

    print(f"[fullsize] {name}: ffn rows", flush=True)
    bucket_of = np.searchsorted(r["vexpert_off"], rows, side="right") - 1
    owner = r["vexpert_owner"][bucket_of]
    hpre_rows, yp_rows = host(L.hpre[rows_t]), host(L.yp[rows_t])
    hpre_ref = np.zeros_like(hpre_rows, dtype=np.float64)
    yp_ref = np.zeros_like(yp_rows, dtype=np.float64)
    for e in np.unique(owner):
        m = owner == e
        h, y_ = O.expert_ffn_fwd(xp_rows[m], [0, int(m.sum())], [0], [inp.w1[int(e)]], None, [inp.w2[int(e)]], None, cfg.act)
        hpre_ref[m], yp_ref[m] = h, y_
    assert rel_err(hpre_rows, hpre_ref) <= tol, "hpre"
    assert rel_err(yp_rows, yp_ref) <= tol, "yp"

    print(f"[fullsize] {name}: layer output on sampled tokens", flush=True)
    st = tok[same][:384]
    y_ref = O.moe_layer_forward(xd[st], None, inp.w1, None, inp.w2, None, k, cfg.act, topk=(idx_gpu[st], w_gpu[st]))
    assert rel_err(host(L.y[torch.from_numpy(st).cuda()]), y_ref) <= tol, "layer output"

    if not cfg.backward:
        return
    print(f"[fullsize] {name}: backward", flush=True)
    L.backward(dev["dy"], dev["w1"], dev["w2"])
    torch.cuda.synchronize()
    dyd = W.decode(inp.dy)
    a_rows = r["src"][rows]
    dyp_ref = dyd[a_rows // k] * w_gpu.reshape(-1)[a_rows][:, None].astype(np.float64)
    assert rel_err(host(L.dyp[rows_t]), dyp_ref) <= 2.0 ** -8, "dyp"
    dyp_rows = host(L.dyp[rows_t])
    dxp_ref = np.zeros_like(dyp_rows, dtype=np.float64)
    for e in np.unique(owner):
        m = owner == e
        dxp, _, _ = O.expert_ffn_bwd(dyp_rows[m], xp_rows[m], hpre_rows[m], [inp.w1[int(e)]], [inp.w2[int(e)]],
                                     [0, int(m.sum())], [0], 1, cfg.act)
        dxp_ref[m] = dxp
    assert rel_err(host(L.dxp[rows_t]), dxp_ref) <= tol, "dxp"
    dx_ref, _, _ = O.moe_layer_backward(xd[st], None, inp.w1, None, inp.w2, k, cfg.act, dyd[st], topk=(idx_gpu[st], w_gpu[st]))
    assert rel_err(host(L.dx[torch.from_numpy(st).cuda()]), dx_ref) <= tol, "dx"

    print(f"[fullsize] {name}: weight gradients on sampled hidden units", flush=True)
    order = np.argsort(-r["expert_count"], kind="stable")
    experts = sorted({int(order[0]), int(order[1]), int(order[E // 2]), int(order[-1])})
    cols = np.sort(rng.choice(cfg.f, size=6, replace=False))
    for e in experts:
        c1, r2 = O.expert_grad_columns(xd, dyd, idx_gpu, w_gpu, e, inp.w1[e], inp.w2[e], cols, cfg.act)
        g1 = host(L.dw1[e][:, torch.from_numpy(cols).cuda()])
        g2 = host(L.dw2[e][torch.from_numpy(cols).cuda(), :])
        if r["expert_count"][e] == 0:
            assert not g1.any() and not g2.any()
        else:
            assert rel_err(g1, c1) <= tol, f"dw1 expert {e}"
            assert rel_err(g2, r2) <= tol, f"dw2 expert {e}"
