"""One MoE layer on one GPU: buffers owned here, every step done by libflexmoe.

Forward (paper Section 3.1 workflow on a single GPU):
    gate_topk -> route(placement table) -> permute -> expert_ffn_fwd -> combine
Backward of the expert path for an upstream gradient dY (gate output held constant):
    permute(dY, row_scale = gate weights) -> expert_ffn_bwd -> combine(weights = None)

This class only allocates device memory once and sequences the C-ABI calls; it
does no arithmetic of its own.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import workloads as W


def to_device(t, device="cuda"):
    """Upload a stored tensor (Bf16Tensor bit patterns or float32 ndarray) unchanged."""
    if t is None:
        return None
    if isinstance(t, W.Bf16Tensor):
        return torch.from_numpy(t.bits.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(t, dtype=np.float32)).to(device)


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


class MoELayer:
    def __init__(self, N, d, f, E, k, V, dtype, act, backward=False, device="cuda", keep_h=None):
        """keep_h (training layers; default on): the forward pass leaves act(Hpre) in a buffer of the layer's
        and the backward pass reads it there instead of computing and storing it again -- A*f more elements
        of saved activations for a shorter backward pass."""
        self.N, self.d, self.f, self.E, self.k, self.V = N, d, f, E, k, V
        self.A = N * k
        self.act = act
        self.dtype_code = dtype
        tdt = torch.bfloat16 if dtype == B.BF16 else torch.float32
        dev = device
        i32 = dict(dtype=torch.int32, device=dev)
        A = self.A
        self.topk_idx = torch.empty((N, k), **i32)
        self.topk_w = torch.empty((N, k), dtype=torch.float32, device=dev)
        self.expert_count = torch.empty(E, **i32)
        self.vexpert_count = torch.empty(V, **i32)
        self.vexpert_off = torch.empty(V + 1, **i32)
        self.vexpert_owner = torch.empty(V, **i32)
        self.dest = torch.empty(A, **i32)
        self.src = torch.empty(A, **i32)
        self.xp = torch.empty((A, d), dtype=tdt, device=dev)
        self.hpre = torch.empty((A, f), dtype=tdt, device=dev)
        self.yp = torch.empty((A, d), dtype=tdt, device=dev)
        self.y = torch.empty((N, d), dtype=tdt, device=dev)
        ws_bytes = B.flexmoe_workspace_bytes(N, d, f, E, k, V, dtype)
        if ws_bytes == 0:
            raise ValueError("unsupported layer shape")
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.has_backward = backward
        self.h = None
        if backward and (keep_h is None or keep_h):
            self.h = torch.empty((A, f), dtype=tdt, device=dev)
        if backward:
            self.dyp = torch.empty((A, d), dtype=tdt, device=dev)
            self.dxp = torch.empty((A, d), dtype=tdt, device=dev)
            self.dx = torch.empty((N, d), dtype=tdt, device=dev)
            self.dw1 = torch.empty((E, d, f), dtype=tdt, device=dev)
            self.dw2 = torch.empty((E, f, d), dtype=tdt, device=dev)

    @classmethod
    def for_config(cls, cfg: W.LayerConfig, device="cuda"):
        return cls(cfg.N, cfg.d, cfg.f, cfg.E, cfg.k, cfg.V, cfg.dtype, cfg.act, cfg.backward, device)

    # -- individual stages ------------------------------------------------
    def gate(self, x, wg):
        B.flexmoe_gate_topk(x, wg, self.k, self.topk_idx, self.topk_w, self.ws)

    def route(self, rep_off, rep_ids):
        B.flexmoe_route(self.topk_idx, self.E, rep_off, rep_ids, self.expert_count, self.vexpert_count,
                        self.vexpert_off, self.vexpert_owner, self.dest, self.src, self.ws)

    def post_loads(self):
        """Start copying this step's expert loads I_e (expert_count, as the router wrote it) into
        pinned host memory on the current stream.  Returns (host int32 tensor, event): the host-side
        scheduler reads the tensor once the event has completed -- normally while later steps run --
        so the stream never waits for the host (Section 3.3: the Scheduler monitors the workloads
        next to the training loop)."""
        if not hasattr(self, "_loads_host"):
            self._loads_host = torch.empty(self.E, dtype=torch.int32, pin_memory=True)
        self._loads_host.copy_(self.expert_count, non_blocking=True)
        ev = torch.cuda.Event()
        ev.record()
        return self._loads_host, ev

    def profile_token_cost(self, w1, w2, reps: int = 3) -> int:
        """T_C of Eq. 7 from profiling: nanoseconds of expert computation (forward, plus backward for a
        training layer) per routed token, measured with HIP events around flexmoe_expert_ffn_fwd / _bwd on
        the buckets the layer currently holds (call after `forward`, and after `backward` for a training
        layer: xp, hpre, dyp must be filled).  The integer it returns is the `token_cost` (1 / TPS) the
        scheduler entry points take; a sync_cost table in the same unit (ns) then weighs T_Sync against it."""
        if self.A == 0:
            return 1
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

        def once():
            B.flexmoe_expert_ffn_fwd(self.xp, self.vexpert_off, self.vexpert_owner, w1, None, w2, None, self.act,
                                     self.hpre, self.yp, self.ws, h=self.h)
            if self.has_backward:
                B.flexmoe_expert_ffn_bwd(self.dyp, self.xp, self.hpre, w1, w2, self.vexpert_off, self.vexpert_owner,
                                         self.act, self.dxp, self.dw1, self.dw2, self.ws, h=self.h)
        once()
        ev[0].record()
        for _ in range(reps):
            once()
        ev[1].record()
        ev[1].synchronize()
        ns = ev[0].elapsed_time(ev[1]) * 1e6 / reps
        return max(1, int(round(ns / self.A)))

    def forward(self, x, wg, w1, w2, rep_off, rep_ids, b1=None, b2=None, keep_hpre=True):
        """keep_hpre=False (inference): the pre-activations are not stored; `backward` cannot follow."""
        self.gate(x, wg)
        self.route(rep_off, rep_ids)
        B.flexmoe_permute(x, self.src, None, self.k, self.xp)
        B.flexmoe_expert_ffn_fwd(self.xp, self.vexpert_off, self.vexpert_owner, w1, b1, w2, b2, self.act,
                                 self.hpre if keep_hpre else None, self.yp, self.ws, h=self.h)
        B.flexmoe_combine(self.yp, self.dest, self.topk_w, self.k, self.y)
        return self.y

    def gather_supported(self) -> bool:
        return self.dtype_code == B.BF16 and self.d % 128 == 0 and self.N * self.d < 2 ** 32

    def forward_fused(self, x, wg, w1, w2, rep_off, rep_ids, b1=None, b2=None, keep_hpre=True):
        """Forward-only variant: the permutation is folded into the first expert GEMM (xp is not
        written, so `backward` cannot follow); keep_hpre=False also drops the pre-activations."""
        self.gate(x, wg)
        self.route(rep_off, rep_ids)
        B.flexmoe_expert_ffn_fwd_gather(x, self.src, self.k, self.vexpert_off, self.vexpert_owner, w1, b1, w2, b2,
                                        self.act, self.hpre if keep_hpre else None, self.yp, self.ws)
        B.flexmoe_combine(self.yp, self.dest, self.topk_w, self.k, self.y)
        return self.y

    def top1_supported(self) -> bool:
        return self.k == 1 and self.gather_supported() and self.f % 128 == 0

    def forward_top1(self, x, wg, w1, w2, rep_off, rep_ids, b1=None, b2=None, keep_hpre=True):
        """Forward-only top-1 layer: gate, route and one expert call that reads x through src and
        stores y through src (neither xp nor yp is written)."""
        self.gate(x, wg)
        self.route(rep_off, rep_ids)
        B.flexmoe_expert_ffn_fwd_top1(x, self.src, self.vexpert_off, self.vexpert_owner, w1, b1, w2, b2, self.act,
                                      self.hpre if keep_hpre else None, self.y, self.ws)
        return self.y

    def backward(self, dy, w1, w2):
        """After `forward` (the one pass that fills xp, hpre and, with keep_h, h)."""
        B.flexmoe_permute(dy, self.src, self.topk_w, self.k, self.dyp)
        B.flexmoe_expert_ffn_bwd(self.dyp, self.xp, self.hpre, w1, w2, self.vexpert_off, self.vexpert_owner,
                                 self.act, self.dxp, self.dw1, self.dw2, self.ws, h=self.h)
        B.flexmoe_combine(self.dxp, self.dest, None, self.k, self.dx)
        return self.dx, self.dw1, self.dw2

    def backward_top1(self, dy, w1, w2):
        """`backward` for a top-1 layer: dX comes straight out of the expert backward (no dXp, no combine)."""
        B.flexmoe_permute(dy, self.src, self.topk_w, self.k, self.dyp)
        B.flexmoe_expert_ffn_bwd_top1(self.dyp, self.xp, self.hpre, w1, w2, self.vexpert_off, self.vexpert_owner,
                                      self.src, self.act, self.dx, self.dw1, self.dw2, self.ws, h=self.h)
        return self.dx, self.dw1, self.dw2

    def backward_full(self, dy, wg, w1, w2):
        """Backward of everything trainable: the expert path as in `backward`, plus the bias
        gradients and the gate path (dW_g, and the gate's share of dX added to self.dx)."""
        dev, tdt = self.dx.device, self.dx.dtype
        if not hasattr(self, "dwg"):
            self.db1 = torch.empty((self.E, self.f), dtype=tdt, device=dev)
            self.db2 = torch.empty((self.E, self.d), dtype=tdt, device=dev)
            self.dl = torch.empty((self.N, self.k), dtype=torch.float32, device=dev)
            self.dwg = torch.empty((self.d, self.E), dtype=tdt, device=dev)
        B.flexmoe_permute(dy, self.src, self.topk_w, self.k, self.dyp)
        B.flexmoe_expert_ffn_bwd(self.dyp, self.xp, self.hpre, w1, w2, self.vexpert_off, self.vexpert_owner,
                                 self.act, self.dxp, self.dw1, self.dw2, self.ws, h=self.h)
        B.flexmoe_expert_bias_grads(self.dyp, self.vexpert_off, self.vexpert_owner, self.f, self.E, self.db1,
                                    self.db2, self.ws)
        B.flexmoe_combine(self.dxp, self.dest, None, self.k, self.dx)
        B.flexmoe_gate_bwd(wg, self.topk_idx, self.topk_w, dy, self.yp, self.xp, self.dest, self.src,
                           self.vexpert_off, self.vexpert_owner, self.dl, self.dx, self.dwg, self.ws)
        return dict(dx=self.dx, dw1=self.dw1, dw2=self.dw2, db1=self.db1, db2=self.db2, dwg=self.dwg, dl=self.dl)
