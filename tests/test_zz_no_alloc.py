"""Collected last (file name): flexmoe_route_static (the router for callers that cannot allocate: its scratch is a fixed array inside the
library) against flexmoe_route, through the C ABI: all six outputs bit for bit, on two calls in a row, the second
with a smaller input (the shared array then still holds the first call's histograms)."""
import numpy as np
import pytest
import torch

from paper_2304_03946_amd import workloads as W

pytestmark = pytest.mark.gpu

NAMES = ("expert_count", "vexpert_count", "vexpert_off", "vexpert_owner", "dest", "src")


def _buffers(A, E, V):
    i32 = dict(dtype=torch.int32, device="cuda")
    return dict(expert_count=torch.full((E,), -7, **i32), vexpert_count=torch.full((V,), -7, **i32),
                vexpert_off=torch.full((V + 1,), -7, **i32), vexpert_owner=torch.full((V,), -7, **i32),
                dest=torch.full((max(A, 1),), -7, **i32), src=torch.full((max(A, 1),), -7, **i32))


def _both(B, idx_np, E, rep_off, rep_ids):
    N, k = idx_np.shape
    V = len(rep_ids)
    idx = torch.from_numpy(np.ascontiguousarray(idx_np, dtype=np.int32)).cuda()
    ref, got = _buffers(N * k, E, V), _buffers(N * k, E, V)
    ws = torch.empty(B.flexmoe_workspace_bytes(max(N, 1), 8, 8, E, k, V, B.F32), dtype=torch.uint8, device="cuda")
    B.flexmoe_route(idx, E, rep_off, rep_ids, *[ref[n] for n in NAMES], ws)
    B.flexmoe_route_static(idx, E, rep_off, rep_ids, *[got[n] for n in NAMES])
    torch.cuda.synchronize()
    for n in NAMES:
        assert torch.equal(got[n], ref[n]), n
    assert int(ref["vexpert_off"][-1]) == N * k


def test_static_scratch_router_matches_the_workspace_router():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X")
    from paper_2304_03946_amd import binding as B
    B.load_library()
    # first call: the GPT-XL-like layer's routing problem (131072 assignments, two-kernel path, 256 units)
    cfg = W.scaled(W.CONFIGS["gpt_xl"], N=65536)
    idx = W.sample_topk_idx(cfg, 21)
    rep = W.placement_from_loads(np.bincount(idx.reshape(-1), minlength=cfg.E), cfg.V, cfg.max_rep, shuffle_seed=2)
    _both(B, idx, cfg.E, *rep)
    # second call, smaller and with other experts hot: stale histograms of the first call are still in the array
    small = W.scaled(W.CONFIGS["gpt_xl"], N=9001, E=37, V=53, k=2)
    idx2 = W.sample_topk_idx(small, 22, log_p=1.5 * np.log(1.0 / (np.arange(37)[::-1] + 1.0)))
    rep2 = W.placement_from_loads(np.bincount(idx2.reshape(-1), minlength=37), 53, 8, shuffle_seed=3)
    _both(B, idx2, 37, *rep2)
    # third: small enough for the single-workgroup router (no scratch at all), then the large one again
    tiny = W.scaled(W.CONFIGS["gpt_m"], N=700, E=8, V=12, k=2)
    idx3 = W.sample_topk_idx(tiny, 23)
    _both(B, idx3, 8, *W.placement_from_loads(np.bincount(idx3.reshape(-1), minlength=8), 12, 4))
    _both(B, idx, cfg.E, *rep)


def test_static_scratch_router_rejects_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X")
    from paper_2304_03946_amd import binding as B
    B.load_library()
    # units * E * 4 bytes must stay within FLEXMOE_ROUTE_STATIC_SCRATCH_BYTES (256 KiB): the 274 units of
    # 140000 assignments x 256 experts do not
    E, V, N, k = 256, 256, 140000, 1
    idx = torch.zeros((N, k), dtype=torch.int32, device="cuda")
    out = _buffers(N * k, E, V)
    before = {n: t.clone() for n, t in out.items()}
    with pytest.raises(B.FlexMoEError) as ei:
        B.flexmoe_route_static(idx, E, np.arange(E + 1), np.arange(V), *[out[n] for n in NAMES])
    assert ei.value.status == B.SCRATCH_LIMIT
    torch.cuda.synchronize()
    for n in NAMES:
        assert torch.equal(out[n], before[n]), "a rejected call must not write anything"
