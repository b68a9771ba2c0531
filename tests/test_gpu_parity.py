"""GPU parity: every stage of the HIP path (called through the C ABI) against the CPU oracle.

Integer artefacts (routing counts, offsets, permutation) must match bit for bit; the
permuted copy must match bit for bit; floating-point outputs must satisfy
    max|gpu - ref| / max|ref| <= 2e-2   (bf16 operands, fp32 accumulation)
                              <= 1e-5   (fp32)
per output tensor.  Top-k indices must be identical on every token whose logit
margin exceeds the worst-case fp32 accumulation error of the gate; on the few
tokens below it the GPU's choice must be a valid top-k within that error.
"""
import numpy as np
import pytest
import torch

from oracle import flexmoe_oracle as O
from paper_2304_03946_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {W.DT_BF16: 2e-2, W.DT_F32: 1e-5}


@pytest.fixture(scope="module")
def api():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X")
    from paper_2304_03946_amd import binding, layer
    binding.load_library()          # fails loudly when the HIP library is not built
    return binding, layer


def rel_err(gpu, ref):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = np.abs(ref).max()
    if scale == 0:
        return float(np.abs(gpu).max())
    return float(np.abs(gpu - ref).max() / scale)


def group_err(gpu, ref, groups):
    """Worst max|gpu - ref| / max|ref| over `groups`, each an index (slice, array or tuple) into both
    arrays, normalised by the GROUP's own largest reference value: an expert's slice of a weight
    gradient, a vExpert's bucket of rows, a column of dW_g.  A tensor-wide norm would let the hottest
    expert's scale hide an error in a cold expert's few-token contraction."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    worst = 0.0
    for g in groups:
        a, b = gpu[g], ref[g]
        if b.size == 0:
            continue
        scale = np.abs(b).max()
        err = np.abs(a - b).max()
        worst = max(worst, float(err if scale == 0 else err / scale))
    return worst


def bucket_groups(r):
    off = r["vexpert_off"]
    return [slice(int(off[v]), int(off[v + 1])) for v in range(len(off) - 1) if off[v + 1] > off[v]]


def expert_groups(r):
    return [int(e) for e in np.nonzero(r["expert_count"] > 0)[0]]


def host(t):
    return t.detach().float().cpu().numpy() if t.dtype != torch.int32 else t.cpu().numpy()


def gate_error_bound(x, wg, dtype):
    """Worst-case |fp32 accumulated logit - exact logit| per token: (d+1) u sum_i |x_i w_i|
    maximised over experts (u = 2^-24; bf16 products are exact in fp32, fp32 products add one
    more rounding, covered by the +1 and the factor 2)."""
    ax = np.abs(np.asarray(x, dtype=np.float64))
    aw = np.abs(np.asarray(wg, dtype=np.float64))
    s = (ax @ aw).max(axis=1)
    return 2.0 * (x.shape[1] + 1) * 2.0 ** -24 * s


def check_gate(idx_gpu, w_gpu, x, wg, k, dtype, tokens=None):
    """Returns the boolean mask of tokens whose selection is pinned (margin above the bound)."""
    xs = W.decode(x) if tokens is None else W.decode(x)[tokens]
    wgd = W.decode(wg)
    idx_ref, w_ref, logits = O.gate_topk(xs, wgd, k)
    bound = gate_error_bound(xs, wgd, dtype)
    pinned = O.topk_margin(logits, k) > 2.0 * bound
    # The bound is the worst case over all rounding patterns (linear in d), so at d = 1024..2048 a few
    # per cent of the tokens fall under it although their fp32 logits order as the exact ones do; the
    # selection must still be the oracle's on at least 99.5 % of ALL tokens (checked below).
    assert pinned.mean() >= 0.95, f"too many near-tie tokens: {1 - pinned.mean():.4f}"
    assert np.array_equal(idx_gpu[pinned], idx_ref[pinned]), "top-k indices differ on pinned tokens"
    # near-tie tokens: the selection must be a set of distinct experts whose exact logits are
    # within the error bound of the exact top-k values, slot by slot
    for t in np.nonzero(~pinned)[0]:
        sel = idx_gpu[t]
        assert len(set(sel.tolist())) == k and sel.min() >= 0 and sel.max() < logits.shape[1]
        ref_sorted = np.sort(logits[t])[::-1][:k]
        assert np.all(np.abs(logits[t, sel] - ref_sorted) <= 2.0 * bound[t] + 1e-30)
    # gate weights: softmax of the kept logits; an error e in each logit moves a weight by < 2e
    same = np.all(idx_gpu == idx_ref, axis=1)
    assert same.mean() >= 0.995, f"selection differs from the oracle's on {1 - same.mean():.4f} of the tokens"
    assert np.all(np.abs(w_gpu[same] - w_ref[same]) <= 4.0 * bound[same, None] + 2e-6)
    np.testing.assert_allclose(w_gpu.sum(axis=1), 1.0, atol=1e-5)
    return same


def upload(layer_mod, inp):
    up = layer_mod.to_device
    return dict(x=up(inp.x), wg=up(inp.wg), w1=up(inp.w1), w2=up(inp.w2), dy=up(inp.dy))


def run_stagewise(api, cfg, inp, rep_off, rep_ids, b1=None, b2=None):
    """Run the layer on the GPU and compare stage by stage, each oracle stage fed with the
    GPU's own upstream results (so only that stage's arithmetic is under test), then end to end."""
    binding, layer_mod = api
    tol = TOL[cfg.dtype]
    dev = upload(layer_mod, inp)
    L = layer_mod.MoELayer.for_config(cfg)
    db1 = layer_mod.to_device(b1)
    db2 = layer_mod.to_device(b2)
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], rep_off, rep_ids, db1, db2)
    torch.cuda.synchronize()
    k, E = cfg.k, cfg.E
    x, wg, w1, w2 = inp.x, inp.wg, inp.w1, inp.w2

    # a1 gate
    idx_gpu, w_gpu = host(L.topk_idx), host(L.topk_w)
    same = check_gate(idx_gpu, w_gpu, x, wg, k, cfg.dtype)

    # a2 route, on the GPU's own top-k: bit exact
    r = O.route(idx_gpu, E, rep_off, rep_ids)
    for name in ("expert_count", "vexpert_count", "vexpert_off", "vexpert_owner", "dest", "src"):
        assert np.array_equal(host(getattr(L, name)), r[name]), name

    # a3 permute: exact copy
    xd = W.decode(x)
    xp_ref = O.permute(xd, r["src"], k)
    xp_gpu = host(L.xp)
    assert np.array_equal(xp_gpu.astype(np.float64), xp_ref), "permute is not an exact copy"

    # a4 expert FFN forward
    b1d = None if b1 is None else W.decode(b1)
    b2d = None if b2 is None else W.decode(b2)
    hpre_ref, yp_ref = O.expert_ffn_fwd(xp_ref, r["vexpert_off"], r["vexpert_owner"], w1, b1d, w2, b2d, cfg.act)
    assert rel_err(host(L.hpre), hpre_ref) <= tol, "hpre"
    assert rel_err(host(L.yp), yp_ref) <= tol, "yp"
    buckets, live = bucket_groups(r), expert_groups(r)
    assert group_err(host(L.hpre), hpre_ref, buckets) <= tol, "hpre, bucket by bucket"
    assert group_err(host(L.yp), yp_ref, buckets) <= tol, "yp, bucket by bucket"

    # a6 combine, fed with the GPU's yp and gate weights
    y_stage = O.combine(host(L.yp), r["dest"], w_gpu, k)
    assert rel_err(host(L.y), y_stage) <= (tol if cfg.dtype == W.DT_F32 else 2.0 ** -8), "combine"

    # end to end against the definition (Eq. 2-4), on the tokens whose selection is pinned
    y_def = O.moe_layer_forward(xd, W.decode(wg), w1, b1d, w2, b2d, k, cfg.act)
    assert rel_err(host(L.y)[same], y_def[same]) <= tol, "layer output"

    out = dict(layer=L, route=r, idx=idx_gpu, w=w_gpu, same=same)
    if not cfg.backward:
        return out

    L.backward(dev["dy"], dev["w1"], dev["w2"])
    torch.cuda.synchronize()
    dyd = W.decode(inp.dy)
    # backward permute with the gate weights as row scale
    dyp_ref = O.permute(dyd, r["src"], k, row_scale=w_gpu.reshape(-1))
    assert rel_err(host(L.dyp), dyp_ref) <= (tol if cfg.dtype == W.DT_F32 else 2.0 ** -8), "dyp"
    # a5 FFN backward, fed with the GPU's dyp and hpre
    dxp_ref, dw1_ref, dw2_ref = O.expert_ffn_bwd(host(L.dyp), xp_ref, host(L.hpre), w1, w2, r["vexpert_off"],
                                                 r["vexpert_owner"], E, cfg.act)
    assert rel_err(host(L.dxp), dxp_ref) <= tol, "dxp"
    assert rel_err(host(L.dw1), dw1_ref) <= tol, "dw1"
    assert rel_err(host(L.dw2), dw2_ref) <= tol, "dw2"
    # the same on every group's own scale: each vExpert's rows, each expert's weight gradient
    assert group_err(host(L.dyp), dyp_ref, buckets) <= (tol if cfg.dtype == W.DT_F32 else 2.0 ** -8), "dyp, bucket by bucket"
    assert group_err(host(L.dxp), dxp_ref, buckets) <= tol, "dxp, bucket by bucket"
    assert group_err(host(L.dw1), dw1_ref, live) <= tol, "dw1, expert by expert"
    assert group_err(host(L.dw2), dw2_ref, live) <= tol, "dw2, expert by expert"
    dx_stage = O.combine(host(L.dxp), r["dest"], None, k)
    assert rel_err(host(L.dx), dx_stage) <= (tol if cfg.dtype == W.DT_F32 else 2.0 ** -8), "dx combine"
    # end to end gradients against the definition with the GPU's selection and the exact gate weights
    # (exact softmax over the kept logits, in the order the GPU reported them)
    kept = np.take_along_axis(O.gate_logits(xd, W.decode(wg)), idx_gpu.astype(np.int64), axis=1)
    ex = np.exp(kept - kept.max(axis=1, keepdims=True))
    w_sel = ex / ex.sum(axis=1, keepdims=True)
    dx_def, dw1_def, dw2_def = O.moe_layer_backward(xd, W.decode(wg), w1, None, w2, k, cfg.act, dyd,
                                                    topk=(idx_gpu, w_sel))
    assert rel_err(host(L.dx), dx_def) <= tol, "dx"
    assert rel_err(host(L.dw1), dw1_def) <= tol, "dw1 end to end"
    assert rel_err(host(L.dw2), dw2_def) <= tol, "dw2 end to end"
    assert group_err(host(L.dw1), dw1_def, live) <= tol, "dw1 end to end, expert by expert"
    assert group_err(host(L.dw2), dw2_def, live) <= tol, "dw2 end to end, expert by expert"
    empty = np.nonzero(r["expert_count"] == 0)[0]
    for e in empty:
        assert not host(L.dw1[e]).any() and not host(L.dw2[e]).any(), "empty expert must get zero gradient"
    return out


# ---------------------------------------------------------------------------------- cases
def test_tiny_fp32_full_config(api):
    cfg = W.CONFIGS["tiny"]
    inp = W.make_layer_inputs(cfg)
    run_stagewise(api, cfg, inp, *W.config_placement(cfg))


def test_tiny_fp32_backward_and_bias(api):
    cfg = W.scaled(W.CONFIGS["tiny"], N=301, E=5, V=8, k=2, backward=True, max_rep=3)
    inp = W.make_layer_inputs(cfg, seed=77)
    rng = np.random.default_rng(0)
    b1 = (rng.standard_normal((cfg.E, cfg.f)) * 0.05).astype(np.float32)
    b2 = (rng.standard_normal((cfg.E, cfg.d)) * 0.05).astype(np.float32)
    binding, layer_mod = api
    # biases only enter the forward pass (bias gradients are not part of the path)
    cfg_f = W.scaled(cfg, backward=False)
    run_stagewise(api, cfg_f, inp, *W.placement_from_loads([5, 4, 3, 2, 1], cfg.V, 3, shuffle_seed=3), b1=b1, b2=b2)
    run_stagewise(api, cfg, inp, *W.placement_from_loads([5, 4, 3, 2, 1], cfg.V, 3, shuffle_seed=3))


SMALL = {
    # several 256-row tiles per bucket, ragged bucket tails, K and column tails (d, f multiples of 8 only)
    "bert_small": W.scaled(W.CONFIGS["bert"], N=1500, d=328, f=776, E=6, V=9, max_rep=2),
    "gpt_small": W.scaled(W.CONFIGS["gpt_m"], N=2100, d=264, f=520, E=8, V=14, max_rep=4),
    "swin_small": W.scaled(W.CONFIGS["swin"], N=3000, d=256, f=512, E=8, V=11, max_rep=4),
    "xl_small": W.scaled(W.CONFIGS["gpt_xl"], N=2600, d=192, f=384, E=64, V=96, max_rep=8),
    # d and f multiples of 128 with ragged column tiles: the backward GEMMs take the direct-to-LDS path
    "gpt_dma": W.scaled(W.CONFIGS["gpt_m"], N=1900, d=384, f=640, E=8, V=13, max_rep=4),
    # the same with enough tokens (A/32 >= 128 K tiles) that the hot experts' weight-gradient contraction is
    # cut into segments (fp32 partial tiles + reduce kernel) inside the shared dXp/dW2/dW1 launch
    "gpt_dma_seg": W.scaled(W.CONFIGS["gpt_m"], N=2300, d=384, f=640, E=8, V=13, max_rep=4),
    # more than one round of workgroups in the second forward product (66000 rows, one column tile -> about 265
    # tiles for 256 compute units) and a long contraction: the tiles left for the last round are cut along K
    # into four segments (fp32 partial tiles + reduce kernel)
    "split_tail": W.scaled(W.CONFIGS["swin"], N=66000, d=128, f=1024, E=8, V=12, max_rep=4, backward=False),
    # three and six column tiles: patches of the tile grid that start and end inside a row of their column strip
    # (32 is no multiple of the strip's width), in all four rows products and both weight gradients
    "strip_patches": W.scaled(W.CONFIGS["bert"], N=2600, d=768, f=1536, E=6, V=9, max_rep=2, backward=True),
    # whole 256 x 256 weight-gradient tiles with two patches per job (d = 512, f = 1024) and skewed loads: the
    # work lists are dealt out over the XCD groups by load, with holes the persistent kernel skips
    "wgrad_balance": W.scaled(W.CONFIGS["gpt_m"], N=2500, d=512, f=1024, E=8, V=13, max_rep=4),
    # the library's limits: 256 experts, 512 vExperts, 8 experts per token -- hundreds of buckets of a few dozen rows
    # (every one a ragged tile, many experts with a handful of tokens, the bucket lookups at their widest)
    "max_experts": W.scaled(W.CONFIGS["gpt_xl"], N=2500, d=128, f=256, E=256, V=512, k=8, max_rep=8, skew_s=1.0),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_reduced_configs_elementwise(api, name):
    cfg = SMALL[name]
    inp = W.make_layer_inputs(cfg)
    rep_off, rep_ids = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=11)
    out = run_stagewise(api, cfg, inp, rep_off, rep_ids)
    r = out["route"]
    # replica shares differ by at most one token
    for e in range(cfg.E):
        shares = r["vexpert_count"][rep_ids[rep_off[e]:rep_off[e + 1]]]
        assert shares.max() - shares.min() <= 1 and shares.sum() == r["expert_count"][e]


def test_bf16_bias_forward(api):
    cfg = W.scaled(SMALL["bert_small"], N=700)
    inp = W.make_layer_inputs(cfg, seed=5)
    rng = np.random.default_rng(1)
    b1 = W.Bf16Tensor.from_f32((rng.standard_normal((cfg.E, cfg.f)) * 0.3).astype(np.float32))
    b2 = W.Bf16Tensor.from_f32((rng.standard_normal((cfg.E, cfg.d)) * 0.3).astype(np.float32))
    run_stagewise(api, cfg, inp, *W.placement_from_loads(W.prior_loads(cfg), cfg.V, 2), b1=b1, b2=b2)


@pytest.mark.parametrize("act", [W.ACT_RELU, W.ACT_GELU_TANH])
def test_other_activations(api, act):
    cfg = W.scaled(SMALL["gpt_small"], N=900, act=act)
    inp = W.make_layer_inputs(cfg, seed=9)
    run_stagewise(api, cfg, inp, *W.placement_from_loads(W.prior_loads(cfg), cfg.V, 4))


def run_full_backward(api, cfg, inp, rep_off, rep_ids, b1=None, b2=None):
    """Gate path and bias gradients: each stage against the oracle fed with the GPU's own
    upstream tensors, then every gradient of the layer against the staged oracle run on the
    GPU's selection."""
    binding, layer_mod = api
    tol = TOL[cfg.dtype]
    dev = upload(layer_mod, inp)
    L = layer_mod.MoELayer.for_config(cfg)
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], rep_off, rep_ids, layer_mod.to_device(b1),
              layer_mod.to_device(b2))
    g = L.backward_full(dev["dy"], dev["wg"], dev["w1"], dev["w2"])
    torch.cuda.synchronize()
    k, E = cfg.k, cfg.E
    xd, wgd, dyd = W.decode(inp.x), W.decode(inp.wg), W.decode(inp.dy)
    b1d = None if b1 is None else W.decode(b1)
    b2d = None if b2 is None else W.decode(b2)
    idx_gpu, w_gpu = host(L.topk_idx), host(L.topk_w)
    r = O.route(idx_gpu, E, rep_off, rep_ids)

    # stage: dl from the GPU's yp and gate weights
    dl_ref = O.topk_softmax_bwd(w_gpu, O.gate_value_grad(dyd, host(L.yp), r["dest"], k))
    if k == 1:
        assert not host(g["dl"]).any() and not host(g["dwg"]).any(), "a single kept logit carries no gradient"
    else:
        assert rel_err(host(g["dl"]), dl_ref) <= tol, "dl"
    # stage: bias gradients from the GPU's dyp and hpre
    db1_ref, db2_ref = O.expert_bias_grads(host(L.dyp), host(L.hpre), inp.w2, r["vexpert_off"], r["vexpert_owner"],
                                           E, cfg.act)
    assert rel_err(host(g["db1"]), db1_ref) <= tol, "db1"
    assert rel_err(host(g["db2"]), db2_ref) <= tol, "db2"
    live = expert_groups(r)
    assert group_err(host(g["db1"]), db1_ref, live) <= tol, "db1, expert by expert"
    assert group_err(host(g["db2"]), db2_ref, live) <= tol, "db2, expert by expert"
    # stage: dW_g from the GPU's dl
    dwg_stage = np.zeros_like(wgd, dtype=np.float64)
    dl_gpu = host(g["dl"]).astype(np.float64)
    for j in range(k):
        np.add.at(dwg_stage.T, idx_gpu[:, j], dl_gpu[:, j:j + 1] * xd)
    if k > 1:
        assert rel_err(host(g["dwg"]), dwg_stage) <= (tol if cfg.dtype == W.DT_F32 else 2.0 ** -8), "dwg stage"
        cols = [(slice(None), e) for e in live]
        assert group_err(host(g["dwg"]), dwg_stage, cols) <= (tol if cfg.dtype == W.DT_F32 else 2.0 ** -8), "dwg stage, column by column"

    # end to end on the GPU's selection with the exact gate weights
    kept = np.take_along_axis(O.gate_logits(xd, wgd), idx_gpu.astype(np.int64), axis=1)
    ex = np.exp(kept - kept.max(axis=1, keepdims=True))
    w_sel = ex / ex.sum(axis=1, keepdims=True)
    fwd = O.staged_forward(xd, wgd, inp.w1, b1d, inp.w2, b2d, k, cfg.act, rep_off, rep_ids, topk=(idx_gpu, w_sel))
    ref = O.staged_backward(fwd, dyd, inp.w1, inp.w2, k, cfg.act, x=xd, wg=wgd)
    assert rel_err(host(g["dx"]), ref["dx_total"]) <= tol, "dx (both paths)"
    for name in ("dw1", "dw2", "db1", "db2"):
        assert rel_err(host(g[name]), ref[name]) <= tol, name
        assert group_err(host(g[name]), ref[name], live) <= tol, name + ", expert by expert"
    if k > 1:
        assert rel_err(host(g["dwg"]), ref["dwg"]) <= tol, "dwg"
        # column by column for the experts with enough tokens that the logit gradients' own rounding
        # noise (dl is a difference of dot products over bf16 rows) averages out
        busy = [(slice(None), e) for e in live if r["expert_count"][e] >= 64]
        assert group_err(host(g["dwg"]), ref["dwg"], busy) <= tol, "dwg, column by column"
        assert np.abs(ref["dx_gate"]).max() > 1e-3 * np.abs(ref["dx"]).max(), "the case must exercise the gate path"
    empty = np.nonzero(r["expert_count"] == 0)[0]
    for e in empty:
        assert not host(g["db1"][e]).any() and not host(g["db2"][e]).any() and not host(g["dwg"][:, e]).any()
    return L, g


def test_full_backward_fp32(api):
    cfg = W.scaled(W.CONFIGS["tiny"], N=301, E=5, V=8, k=2, backward=True, max_rep=3)
    inp = W.make_layer_inputs(cfg, seed=78)
    rng = np.random.default_rng(0)
    b1 = (rng.standard_normal((cfg.E, cfg.f)) * 0.05).astype(np.float32)
    b2 = (rng.standard_normal((cfg.E, cfg.d)) * 0.05).astype(np.float32)
    run_full_backward(api, cfg, inp, *W.placement_from_loads([5, 4, 3, 2, 1], cfg.V, 3, shuffle_seed=3), b1=b1, b2=b2)


@pytest.mark.parametrize("name", ["gpt_small", "swin_small", "xl_small", "gpt_dma", "gpt_dma_seg", "strip_patches", "wgrad_balance"])
def test_full_backward_reduced_configs(api, name):
    cfg = SMALL[name]
    inp = W.make_layer_inputs(cfg)
    rng = np.random.default_rng(2)
    b1 = W.Bf16Tensor.from_f32((rng.standard_normal((cfg.E, cfg.f)) * 0.3).astype(np.float32))
    b2 = W.Bf16Tensor.from_f32((rng.standard_normal((cfg.E, cfg.d)) * 0.3).astype(np.float32))
    rep_off, rep_ids = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=11)
    run_full_backward(api, cfg, inp, rep_off, rep_ids, b1=b1, b2=b2)


def test_full_backward_is_reproducible(api):
    cfg = SMALL["gpt_small"]
    inp = W.make_layer_inputs(cfg)
    rep = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=11)
    runs = []
    for _ in range(2):
        _, g = run_full_backward(api, cfg, inp, *rep)
        runs.append({n: host(t).copy() for n, t in g.items()})
    for n in runs[0]:
        assert np.array_equal(runs[0][n], runs[1][n]), n


@pytest.mark.parametrize("name,bias", [("gpt_dma", False), ("gpt_dma", True)])
def test_gathered_forward_equals_permute_then_ffn(api, name, bias):
    """flexmoe_expert_ffn_fwd_gather must reproduce flexmoe_permute + flexmoe_expert_ffn_fwd bit for
    bit (same tiles, same arithmetic, only the row addresses differ)."""
    binding, layer_mod = api
    cfg = SMALL[name]
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    rng = np.random.default_rng(4)
    b1 = layer_mod.to_device(W.Bf16Tensor.from_f32((rng.standard_normal((cfg.E, cfg.f)) * 0.3).astype(np.float32))) if bias else None
    b2 = layer_mod.to_device(W.Bf16Tensor.from_f32((rng.standard_normal((cfg.E, cfg.d)) * 0.3).astype(np.float32))) if bias else None
    rep = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=11)
    L = layer_mod.MoELayer.for_config(cfg)
    assert L.gather_supported()
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep, b1, b2)
    torch.cuda.synchronize()
    want = {n: host(getattr(L, n)).copy() for n in ("hpre", "yp", "y")}
    for t in (L.hpre, L.yp, L.y, L.xp):
        t.zero_()
    L.forward_fused(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep, b1, b2)
    torch.cuda.synchronize()
    for n in want:
        assert np.array_equal(host(getattr(L, n)), want[n]), n
    assert not host(L.xp).any(), "the fused path must not touch xp"


@pytest.mark.parametrize("name", ["tiny_f32", "bert_small", "gpt_dma"])
def test_forward_without_stored_preactivations(api, name):
    """hpre = NULL (inference): yp and y are the same bits, the hpre buffer is not touched.
    Covers the fp32 kernels, the register-staged bf16 kernels and the direct-to-LDS ones (both entry points)."""
    binding, layer_mod = api
    cfg = W.CONFIGS["tiny"] if name == "tiny_f32" else SMALL[name]
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    rep = W.config_placement(cfg) if name == "tiny_f32" else W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep)
    L = layer_mod.MoELayer.for_config(cfg)
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep)
    torch.cuda.synchronize()
    want = {n: host(getattr(L, n)).copy() for n in ("yp", "y")}
    variants = [L.forward] + ([L.forward_fused] if L.gather_supported() else [])
    for fwd in variants:
        for t in (L.yp, L.y):
            t.zero_()
        L.hpre.fill_(7.0)
        fwd(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep, keep_hpre=False)
        torch.cuda.synchronize()
        for n in want:
            assert np.array_equal(host(getattr(L, n)), want[n]), n
        assert bool((L.hpre == 7.0).all()), "hpre must stay untouched"


@pytest.mark.parametrize("bias", [False, True])
def test_top1_forward_equals_the_staged_forward(api, bias):
    """flexmoe_expert_ffn_fwd_top1 (rows gathered on load, results scattered on store) must give the y
    of permute + FFN + combine bit for bit, and must not touch xp or yp."""
    binding, layer_mod = api
    cfg = SMALL["swin_small"]                       # k = 1, d = 256, f = 512
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    rng = np.random.default_rng(5)
    b1 = layer_mod.to_device(W.Bf16Tensor.from_f32((rng.standard_normal((cfg.E, cfg.f)) * 0.3).astype(np.float32))) if bias else None
    b2 = layer_mod.to_device(W.Bf16Tensor.from_f32((rng.standard_normal((cfg.E, cfg.d)) * 0.3).astype(np.float32))) if bias else None
    rep = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=7)
    L = layer_mod.MoELayer.for_config(cfg)
    assert L.top1_supported()
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep, b1, b2)
    torch.cuda.synchronize()
    want = {n: host(getattr(L, n)).copy() for n in ("hpre", "y")}
    for t in (L.hpre, L.y, L.xp, L.yp):
        t.zero_()
    L.forward_top1(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep, b1, b2)
    torch.cuda.synchronize()
    for n in want:
        assert np.array_equal(host(getattr(L, n)), want[n]), n
    assert not host(L.xp).any() and not host(L.yp).any(), "the fused path must not touch xp or yp"
    # inference form: no pre-activations either
    L.y.zero_()
    L.hpre.fill_(3.0)
    L.forward_top1(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep, b1, b2, keep_hpre=False)
    torch.cuda.synchronize()
    assert np.array_equal(host(L.y), want["y"]) and bool((L.hpre == 3.0).all())


@pytest.mark.parametrize("N,d,f,E,V,k,bias", [(70000, 128, 1024, 4, 7, 1, False), (40000, 256, 1024, 6, 9, 1, True),
                                               (36000, 384, 1024, 5, 9, 2, False), (33000, 256, 2048, 8, 16, 2, True),
                                               (66100, 128, 1152, 3, 5, 1, True)])
def test_forward_variants_agree_bit_for_bit(api, N, d, f, E, V, k, bias):
    """The staged forward, the gathered forward, the top-1 call and their hpre = NULL forms run the same
    tiles with the same arithmetic: identical bits on shapes that reach one or several rounds of workgroups,
    with and without a split last round (no oracle needed: the staged forward is checked against it elsewhere)."""
    binding, layer_mod = api
    cfg = W.scaled(W.CONFIGS["gpt_m"], N=N, d=d, f=f, E=E, V=V, k=k, max_rep=4, backward=False)
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    rng = np.random.default_rng(N)
    b1 = layer_mod.to_device(W.Bf16Tensor.from_f32((rng.standard_normal((E, f)) * 0.3).astype(np.float32))) if bias else None
    b2 = layer_mod.to_device(W.Bf16Tensor.from_f32((rng.standard_normal((E, d)) * 0.3).astype(np.float32))) if bias else None
    rep = W.placement_from_loads(W.prior_loads(cfg), V, cfg.max_rep, shuffle_seed=N)
    L = layer_mod.MoELayer.for_config(cfg)
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep, b1, b2)
    torch.cuda.synchronize()
    want = {n: getattr(L, n).clone() for n in ("hpre", "yp", "y")}
    variants = [("gathered", L.forward_fused, True, ("hpre", "yp", "y")), ("gathered, no hpre", L.forward_fused, False, ("yp", "y")),
                ("staged, no hpre", L.forward, False, ("yp", "y"))]
    if L.top1_supported():
        variants += [("top-1", L.forward_top1, True, ("hpre", "y")), ("top-1, no hpre", L.forward_top1, False, ("y",))]
    for tag, fn, keep, outs in variants:
        for n in ("hpre", "yp", "y"):
            getattr(L, n).zero_()
        fn(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep, b1, b2, keep_hpre=keep)
        torch.cuda.synchronize()
        for n in outs:
            assert torch.equal(getattr(L, n), want[n]), f"{tag}: {n}"


@pytest.mark.parametrize("name", ["swin_small", "many_rounds"])
def test_top1_backward_equals_the_staged_backward(api, name):
    """flexmoe_expert_ffn_bwd_top1 stores dXp's rows through src: the same dX as the staged backward's
    combine, and the same weight gradients, bit for bit (shared launch and, at the larger size, the
    separate dXp launch)."""
    binding, layer_mod = api
    if name == "swin_small":
        cfg = SMALL[name]
    else:   # dXp alone: more than eight rounds of workgroups are needed for the separate launch
        cfg = W.scaled(W.CONFIGS["swin"], N=70000, d=2048, f=128, E=4, V=6, max_rep=2)
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    rep = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=9)
    L = layer_mod.MoELayer.for_config(cfg)
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep)
    L.backward(dev["dy"], dev["w1"], dev["w2"])
    torch.cuda.synchronize()
    want = {n: getattr(L, n).clone() for n in ("dx", "dw1", "dw2")}
    for n in ("dx", "dw1", "dw2", "dxp"):
        getattr(L, n).zero_()
    L.backward_top1(dev["dy"], dev["w1"], dev["w2"])
    torch.cuda.synchronize()
    for n in want:
        assert torch.equal(getattr(L, n), want[n]), n
    assert not bool(L.dxp.any()), "the fused backward must not touch dxp"


@pytest.mark.parametrize("name", ["gpt_small", "gpt_dma", "gpt_dma_seg", "swin_small", "tiny_f32", "gelu_tanh"])
def test_backward_with_kept_activations_equals_the_recomputing_backward(api, name):
    """The forward pass may leave act(Hpre) in a buffer of the caller's, and the backward pass then skips
    computing and storing it: the kept tensor is what the recomputing backward derives from hpre, and dX, dW1,
    dW2 are the same bits (direct-to-LDS and register-staged paths, shared and separate backward launches,
    the top-1 calls, fp32)."""
    binding, layer_mod = api
    if name == "tiny_f32":
        cfg = W.scaled(W.CONFIGS["tiny"], N=301, E=5, V=8, k=2, backward=True, max_rep=3)
    elif name == "gelu_tanh":
        cfg = W.scaled(SMALL["gpt_dma"], act=W.ACT_GELU_TANH)
    else:
        cfg = SMALL[name]
    cfg = W.scaled(cfg, backward=True)
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    rep = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=4)
    grads = {}
    for keep in (False, True):
        L = layer_mod.MoELayer(cfg.N, cfg.d, cfg.f, cfg.E, cfg.k, cfg.V, cfg.dtype, cfg.act, backward=True, keep_h=keep)
        assert (L.h is not None) == keep
        L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep)
        top1 = keep and L.k == 1 and L.dtype_code == binding.BF16 and L.f % 128 == 0
        (L.backward_top1 if top1 else L.backward)(dev["dy"], dev["w1"], dev["w2"])
        torch.cuda.synchronize()
        grads[keep] = {n: getattr(L, n).clone() for n in ("y", "dx", "dw1", "dw2")}
        if keep:
            kept = L.h.clone()
        else:
            # the recomputing backward leaves act(Hpre) behind dHpre in its workspace
            esz = L.hpre.element_size()
            off = (L.A * L.f * esz + 255) // 256 * 256 if L.dtype_code == binding.BF16 else L.A * L.f * esz
            recomputed = L.ws[off:off + L.A * L.f * esz].view(L.hpre.dtype).view(L.A, L.f).clone()
    assert torch.equal(kept, recomputed), "act(Hpre): kept by the forward pass vs computed again by the backward pass"
    for n in grads[True]:
        assert torch.equal(grads[True][n], grads[False][n]), n


def test_gathered_forward_refuses_what_it_cannot_do(api):
    binding, layer_mod = api
    cfg = SMALL["bert_small"]                       # d = 328: not a multiple of 128
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    L = layer_mod.MoELayer.for_config(cfg)
    assert not L.gather_supported()
    rep = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep)
    with pytest.raises(binding.FlexMoEError) as ei:
        L.forward_fused(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep)
    assert ei.value.status == binding.UNSUPPORTED


def _bf16_ulp(v):
    """Spacing of bf16 numbers at |v| (8 significand bits; subnormals below 2^-126)."""
    a = np.maximum(np.abs(np.asarray(v, dtype=np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


@pytest.mark.parametrize("act", [W.ACT_GELU_ERF, W.ACT_GELU_TANH])
def test_activation_on_every_bf16_value(api, act):
    """Every finite bf16 pre-activation once: with identity weights (one expert, d = f = 128, exact
    sums) Hpre is Xp itself, Yp is act(Xp) and, for dY = 1, dXp is act'(Xp), each rounded once to
    bf16.  Covers the tiny and huge magnitudes the random workloads never produce."""
    B, layer = api
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    bits[(bits & 0x7F80) == 0x7F80] = 0                      # NaN/Inf patterns -> +0
    bits[(bits & 0x7F80) == 0] &= 0x8000                     # subnormals -> +-0 (matrix cores may flush them)
    A, d = 512, 128
    xp = W.Bf16Tensor(bits.reshape(A, d))
    z = W.decode(xp).astype(np.float64)
    eye = W.Bf16Tensor.from_f32(np.eye(d, dtype=np.float32)[None])
    ones = W.Bf16Tensor.from_f32(np.ones((A, d), dtype=np.float32))
    up = layer.to_device
    i32 = lambda a: torch.tensor(a, dtype=torch.int32, device="cuda")
    voff, owner = i32([0, A]), i32([0])
    hpre = torch.empty(A, d, dtype=torch.bfloat16, device="cuda")
    yp, dxp = torch.empty_like(hpre), torch.empty_like(hpre)
    dw1 = torch.empty(1, d, d, dtype=torch.bfloat16, device="cuda")
    dw2 = torch.empty_like(dw1)
    ws = torch.empty(B.flexmoe_workspace_bytes(A, d, d, 1, 1, 1, W.DT_BF16), dtype=torch.uint8, device="cuda")
    xp_d, eye_d = up(xp), up(eye)
    B.flexmoe_expert_ffn_fwd(xp_d, voff, owner, eye_d, None, eye_d, None, act, hpre, yp, ws)
    B.flexmoe_expert_ffn_bwd(up(ones), xp_d, hpre, eye_d, eye_d, voff, owner, act, dxp, dw1, dw2, ws)
    torch.cuda.synchronize()
    assert np.array_equal(host(hpre).astype(np.float64), z)
    # magnitudes below 2^-24 are evaluated at 2^-24: an absolute error below 2^-25
    for got, ref in ((host(yp), O.act_fn(z, act)), (host(dxp), O.act_grad(z, act))):
        err = np.abs(got.astype(np.float64) - ref)
        allowed = np.maximum(_bf16_ulp(ref), 2.0 ** -24)
        worst = int(np.argmax(err / allowed))
        assert (err <= allowed).all(), (z.flat[worst], got.flat[worst], ref.flat[worst])
        assert (err <= 0.5 * _bf16_ulp(ref) + 2.0 ** -24).mean() > 0.999        # correctly rounded almost everywhere


@pytest.mark.parametrize("N,d,E,k", [(333, 136, 5, 1), (333, 136, 33, 2), (1000, 72, 64, 8), (97, 520, 100, 3),
                                     (515, 264, 256, 8), (40000, 64, 16, 2), (33000, 136, 64, 2), (70001, 72, 48, 1)])
def test_gate_alone_shapes(api, N, d, E, k):
    """The gate on its own over expert counts on both sides of the 64-expert kernel switch, ragged
    token tiles, K tails that are not a multiple of the 64-wide tile, and every launch shape."""
    binding, layer_mod = api
    rng = np.random.default_rng(N + d + E)
    x = W.Bf16Tensor.from_f32(rng.standard_normal((N, d)).astype(np.float32))
    wg = W.Bf16Tensor.from_f32((rng.standard_normal((d, E)) / np.sqrt(d) * 3.0).astype(np.float32))
    xd, wgd = layer_mod.to_device(x), layer_mod.to_device(wg)
    idx = torch.full((N, k), -1, dtype=torch.int32, device="cuda")
    w = torch.zeros((N, k), dtype=torch.float32, device="cuda")
    ws = torch.empty(binding.flexmoe_workspace_bytes(N, d, 64, E, k, E, W.DT_BF16), dtype=torch.uint8, device="cuda")
    binding.flexmoe_gate_topk(xd, wgd, k, idx, w, ws)
    torch.cuda.synchronize()
    check_gate(host(idx), host(w), x, wg, k, W.DT_BF16)


def test_exact_ties_pick_lower_expert(api):
    """Small-integer inputs make every fp32 sum exact, so ties are real ties on both sides."""
    binding, layer_mod = api
    rng = np.random.default_rng(4)
    N, d, E, k = 257, 64, 12, 3
    x = rng.integers(-2, 3, size=(N, d)).astype(np.float32)
    wg = rng.integers(-1, 2, size=(d, E)).astype(np.float32)
    wg[:, 5] = wg[:, 2]                       # two identical experts: always tied
    idx_ref, w_ref, logits = O.gate_topk(x, wg, k)
    for dtype, store in ((binding.F32, lambda a: a), (binding.BF16, W.Bf16Tensor.from_f32)):
        xd, wd = layer_mod.to_device(store(x)), layer_mod.to_device(store(wg))
        idx = torch.empty((N, k), dtype=torch.int32, device="cuda")
        w = torch.empty((N, k), dtype=torch.float32, device="cuda")
        ws = torch.empty(binding.flexmoe_workspace_bytes(N, d, 64, E, k, E, dtype), dtype=torch.uint8, device="cuda")
        binding.flexmoe_gate_topk(xd, wd, k, idx, w, ws)
        torch.cuda.synchronize()
        assert np.array_equal(idx.cpu().numpy(), idx_ref)
        np.testing.assert_allclose(w.cpu().numpy(), w_ref, atol=2e-6)


def _route_only(api, idx_np, E, rep_off, rep_ids):
    binding, layer_mod = api
    N, k = idx_np.shape
    V = len(rep_ids)
    i32 = dict(dtype=torch.int32, device="cuda")
    idx = torch.from_numpy(np.ascontiguousarray(idx_np, dtype=np.int32)).cuda()
    out = dict(expert_count=torch.full((E,), -7, **i32), vexpert_count=torch.full((V,), -7, **i32),
               vexpert_off=torch.full((V + 1,), -7, **i32), vexpert_owner=torch.full((V,), -7, **i32),
               dest=torch.full((max(N * k, 1),), -7, **i32), src=torch.full((max(N * k, 1),), -7, **i32))
    ws = torch.empty(binding.flexmoe_workspace_bytes(max(N, 1), 8, 8, E, k, V, binding.F32), dtype=torch.uint8, device="cuda")
    binding.flexmoe_route(idx, E, rep_off, rep_ids, out["expert_count"], out["vexpert_count"], out["vexpert_off"],
                          out["vexpert_owner"], out["dest"], out["src"], ws)
    torch.cuda.synchronize()
    return {n: t.cpu().numpy() for n, t in out.items()}


@pytest.mark.parametrize("case", ["one_expert", "fewer_tokens_than_replicas", "k_equals_E", "ragged_unit", "max_sizes"])
def test_route_adversarial(api, case):
    rng = np.random.default_rng(12)
    if case == "one_expert":                # every token to expert 3, which has 5 replicas
        E, V, N, k = 8, 12, 4099, 1
        idx = np.full((N, 1), 3, dtype=np.int32)
        rep_off, rep_ids = W.placement_from_loads([0, 0, 0, 100, 0, 0, 0, 0], V, 5, shuffle_seed=2)
    elif case == "fewer_tokens_than_replicas":
        E, V, N, k = 4, 16, 3, 2
        idx = np.array([[0, 1], [0, 2], [1, 0]], dtype=np.int32)
        rep_off, rep_ids = W.placement_from_loads([9, 1, 1, 1], V, 13)
    elif case == "k_equals_E":
        E, V, N, k = 4, 6, 777, 4
        idx = np.stack([rng.permutation(E) for _ in range(N)]).astype(np.int32)
        rep_off, rep_ids = W.placement_from_loads([1, 1, 1, 1], V, 3, shuffle_seed=1)
    elif case == "ragged_unit":             # A not a multiple of the 64-lane rounds nor of the unit length
        E, V, N, k = 37, 53, 12345, 2
        cfg = W.scaled(W.CONFIGS["gpt_xl"], N=N, E=E, V=V, k=k)
        idx = W.sample_topk_idx(cfg, 3, log_p=1.5 * np.log(1.0 / (np.arange(E) + 1.0)))
        rep_off, rep_ids = W.placement_from_loads(np.bincount(idx.reshape(-1), minlength=E), V, 8, shuffle_seed=5)
    else:                                    # the library's limits: E = 256, V = 512, k = 8
        E, V, N, k = 256, 512, 20000, 8
        cfg = W.scaled(W.CONFIGS["gpt_xl"], N=N, E=E, V=V, k=k)
        idx = W.sample_topk_idx(cfg, 4, log_p=1.2 * np.log(1.0 / (np.arange(E) + 1.0)))
        rep_off, rep_ids = W.placement_from_loads(np.bincount(idx.reshape(-1), minlength=E), V, 8, shuffle_seed=6)
    got = _route_only(api, idx, E, rep_off, rep_ids)
    ref = O.route(idx, E, rep_off, rep_ids)
    for name, arr in ref.items():
        assert np.array_equal(got[name][:arr.shape[0]], arr), (case, name)


def test_route_empty_batch(api):
    got = _route_only(api, np.zeros((0, 2), dtype=np.int32), 3, [0, 1, 2, 4], [0, 1, 2, 3])
    assert got["expert_count"].tolist() == [0, 0, 0] and got["vexpert_off"].tolist() == [0, 0, 0, 0, 0]
    assert got["vexpert_owner"].tolist() == [0, 1, 2, 2]


def test_errors_are_reported_before_any_launch(api):
    binding, layer_mod = api
    idx = np.zeros((4, 1), dtype=np.int32)
    for off, ids in (([0, 1, 1], [0]), ([0, 1, 3], [0, 1, 1]), ([0, 2, 3], [0, 1, 3])):
        with pytest.raises(binding.FlexMoEError) as ei:
            _route_only(api, idx, 2, off, ids + [0] * 0)
        assert ei.value.status in (binding.BAD_PLACEMENT, binding.INVALID_ARG)
    x = torch.zeros((4, 12), dtype=torch.bfloat16, device="cuda")     # d not a multiple of 8
    with pytest.raises(binding.FlexMoEError) as ei:
        binding.flexmoe_permute(x, torch.zeros(4, dtype=torch.int32, device="cuda"), None, 1, torch.empty_like(x))
    assert ei.value.status == binding.INVALID_ARG
    # workspace too small
    L = layer_mod.MoELayer(64, 64, 64, 4, 1, 4, binding.BF16, binding.RELU)
    xp = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((4, 64, 64), dtype=torch.bfloat16, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.FlexMoEError) as ei:
        binding.flexmoe_expert_ffn_fwd(xp, L.vexpert_off, L.vexpert_owner, w, None, w, None, binding.RELU, L.hpre, L.yp, small)
    assert ei.value.status == binding.WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()


def test_two_runs_are_bit_identical(api):
    binding, layer_mod = api
    cfg = SMALL["gpt_small"]
    inp = W.make_layer_inputs(cfg)
    rep = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=11)
    dev = upload(layer_mod, inp)
    outs = []
    for _ in range(2):
        L = layer_mod.MoELayer.for_config(cfg)
        L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep)
        L.backward(dev["dy"], dev["w1"], dev["w2"])
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (L.dest, L.src, L.vexpert_off, L.y, L.dx, L.dw1, L.dw2)])
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b)


def test_hot_set_drift_with_a_new_table_each_time(api):
    """Routing fluctuation (Observation 2): three drifts of the hot set, each with a new bias row in
    W_g and a new placement table built from the loads of the step before, on one set of layer
    buffers.  After every drift routing is bit-exact and every float output within tolerance, group
    by group."""
    binding, layer_mod = api
    cfg = W.scaled(W.CONFIGS["gpt_xl"], N=2400, d=256, f=512, E=16, V=24, max_rep=4)
    inp = W.make_layer_inputs(cfg)
    tol = TOL[cfg.dtype]
    dev = upload(layer_mod, inp)
    L = layer_mod.MoELayer.for_config(cfg)
    xd, dyd = W.decode(inp.x), W.decode(inp.dy)
    loads = W.prior_loads(cfg)
    hottest = []
    for drift in range(4):
        wg, _ = W.make_gate_weights(cfg, inp.seed, drift=drift)
        wg_dev = layer_mod.to_device(wg)
        rep_off, rep_ids = W.placement_from_loads(loads, cfg.V, cfg.max_rep, shuffle_seed=drift)
        L.forward(dev["x"], wg_dev, dev["w1"], dev["w2"], rep_off, rep_ids)
        L.backward(dev["dy"], dev["w1"], dev["w2"])
        torch.cuda.synchronize()
        idx_gpu, w_gpu = host(L.topk_idx), host(L.topk_w)
        check_gate(idx_gpu, w_gpu, inp.x, wg, cfg.k, cfg.dtype)
        r = O.route(idx_gpu, cfg.E, rep_off, rep_ids)
        for name in ("expert_count", "vexpert_count", "vexpert_off", "vexpert_owner", "dest", "src"):
            assert np.array_equal(host(getattr(L, name)), r[name]), (drift, name)
        fwd = O.staged_forward(xd, W.decode(wg), inp.w1, None, inp.w2, None, cfg.k, cfg.act, rep_off, rep_ids,
                               topk=(idx_gpu, w_gpu))
        ref = O.staged_backward(fwd, dyd, inp.w1, inp.w2, cfg.k, cfg.act)
        live, buckets = expert_groups(r), bucket_groups(r)
        assert rel_err(host(L.y), fwd["y"]) <= tol and rel_err(host(L.dx), ref["dx"]) <= tol, drift
        assert group_err(host(L.yp), fwd["yp"], buckets) <= tol, drift
        assert group_err(host(L.dw1), ref["dw1"], live) <= tol and group_err(host(L.dw2), ref["dw2"], live) <= tol, drift
        for e in np.nonzero(r["expert_count"] == 0)[0]:
            assert not host(L.dw1[e]).any() and not host(L.dw2[e]).any()
        loads = r["expert_count"]
        hottest.append(int(np.argmax(loads)))
    assert len(set(hottest)) > 1, "the hot set must have moved"


def test_scheduler_in_the_loop_keeps_the_layer_output(api):
    """Alg. 1 next to the training loop: the router's expert counts reach the host without a stream
    wait, one scheduler pass turns them into a new placement, and the router takes the new table on
    the next step.  Replicating experts and re-partitioning their tokens leaves the model untouched
    (Section 3), so the layer output must not change by a single bit, while the balance ratio of
    the emulated cluster (4 GPUs x 4 vExpert slots, computed here on the one GPU) drops."""
    from oracle import scheduler_oracle as SO
    from paper_2304_03946_amd import scheduler as sch
    binding, layer_mod = api
    G, S = 4, 4
    cfg = W.scaled(W.CONFIGS["gpt_m"], N=1900, d=384, f=640, E=8, V=G * S, max_rep=8)
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    L = layer_mod.MoELayer.for_config(cfg)
    # GPU g hosts experts g and g + 4, two slots each (the hottest and the coldest expert of this
    # workload do not share a GPU: Alg. 2 as printed finds no plan when the slot the coldest expert
    # releases sits on the very GPU it is meant to relieve)
    owner = np.array([e for g in range(G) for e in (g, g, g + 4, g + 4)], dtype=np.int32)
    rep = sch.flexmoe_placement_table(owner, cfg.E)
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep)
    loads, ev = L.post_loads()
    y_before = L.y.clone()
    ev.synchronize()
    I = loads.numpy().astype(np.int64)
    assert np.array_equal(I, np.bincount(host(L.topk_idx).ravel(), minlength=cfg.E))

    ops, new_owner, before, after = sch.flexmoe_schedule(I, owner, G, 1, 1.0, 32)
    r_ops, r_owner, r_before, r_after = SO.schedule(I.tolist(), owner.tolist(), G, 1, 1.0, 32)
    assert [tuple(o) for o in ops.tolist()] == r_ops and new_owner.tolist() == r_owner
    assert (before, after) == (r_before, r_after)
    assert len(ops) > 0 and after < before

    # Eq. 7: the cost per token comes from profiling the expert computation; with a synchronisation table in
    # the same unit the plan made with the measured cost is the oracle's plan for that cost
    L.backward(dev["dy"], dev["w1"], dev["w2"])
    cost = L.profile_token_cost(dev["w1"], dev["w2"])
    assert isinstance(cost, int) and 1 <= cost < 10 ** 7
    sync = [0, 0] + [40 * cost * g for g in range(2, G + 1)]
    m_ops, m_owner, _, _ = sch.flexmoe_schedule(I, owner, G, cost, 1.0, 32, sync_cost=sync)
    o_ops, o_owner, _, _ = SO.schedule(I.tolist(), owner.tolist(), G, cost, 1.0, 32, sync)
    assert [tuple(o) for o in m_ops.tolist()] == o_ops and m_owner.tolist() == o_owner

    rep2 = sch.flexmoe_placement_table(new_owner, cfg.E)
    L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep2)
    torch.cuda.synchronize()
    assert torch.equal(L.y.view(torch.int16), y_before.view(torch.int16))
    # the shares the router handed out are the ones the scheduler planned with
    assert host(L.vexpert_count).tolist() == SO.vexpert_shares(I.tolist(), r_owner)
    ratio, gpu_load = sch.flexmoe_balance_ratio(I, new_owner, G)
    assert host(L.vexpert_count).reshape(G, S).sum(1).tolist() == gpu_load.tolist() and ratio == after


def test_step_replays_from_a_hip_graph(api):
    """The calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
    memset nodes), so a forward + backward step can be captured once and replayed.  Every replay is
    compared bit for bit with the eager step on the same buffers, with eager work and
    synchronisations between the replays and the inputs changed in place."""
    binding, layer_mod = api
    cfg = SMALL["gpt_dma"]
    inp = W.make_layer_inputs(cfg)
    dev = upload(layer_mod, inp)
    rep = W.placement_from_loads(W.prior_loads(cfg), cfg.V, cfg.max_rep, shuffle_seed=3)
    L = layer_mod.MoELayer.for_config(cfg)
    names = ("topk_idx", "dest", "src", "vexpert_off", "hpre", "yp", "y", "dx", "dw1", "dw2")

    def step():
        L.forward(dev["x"], dev["wg"], dev["w1"], dev["w2"], *rep)
        L.backward(dev["dy"], dev["w1"], dev["w2"])

    def snapshot():
        torch.cuda.synchronize()
        return [getattr(L, n).clone() for n in names]

    def same(a, b):
        return all(torch.equal(x.view(torch.int16) if x.dtype == torch.bfloat16 else x,
                               y.view(torch.int16) if y.dtype == torch.bfloat16 else y) for x, y in zip(a, b))

    step()                                  # eager first: one-time set-up (activation table, kernel attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    x0 = dev["x"].clone()
    for trial in range(4):
        if trial:                           # new inputs in the same buffers
            dev["x"].copy_(torch.roll(x0, shifts=trial * 17, dims=0))
        step()
        want = snapshot()
        for n in names:
            getattr(L, n).zero_()
        graph.replay()
        got = snapshot()
        assert same(got, want), f"replay {trial} differs from the eager step"
