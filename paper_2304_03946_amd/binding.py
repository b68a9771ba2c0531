"""ctypes binding of libflexmoe.so: argument marshalling only.

Every function has the name and argument order of its C entry point
(include/flexmoe.h).  Tensors are torch CUDA tensors (PyTorch supplies device
memory and the stream, nothing else); all arithmetic happens in the library's
HIP kernels.  The library is required: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflexmoe.so")

F32, BF16 = 0, 1
RELU, GELU_ERF, GELU_TANH = 0, 1, 2
OK, INVALID_ARG, BAD_PLACEMENT, WORKSPACE_TOO_SMALL, UNSUPPORTED, DEVICE_ERROR, SCRATCH_LIMIT = range(7)

EXPORTS = ["flexmoe_status_str", "flexmoe_workspace_bytes", "flexmoe_gate_topk", "flexmoe_route",
           "flexmoe_permute", "flexmoe_expert_ffn_fwd", "flexmoe_expert_ffn_bwd", "flexmoe_combine",
           "flexmoe_gate_bwd", "flexmoe_expert_bias_grads", "flexmoe_expert_ffn_fwd_gather",
           "flexmoe_expert_ffn_fwd_top1", "flexmoe_expert_ffn_bwd_top1", "flexmoe_route_static",
           # host-side scheduler (include/flexmoe_scheduler.h; Python face in scheduler.py)
           "flexmoe_balance_ratio", "flexmoe_step_cost", "flexmoe_make_scheduling_plan", "flexmoe_schedule",
           "flexmoe_placement_table"]

_lib = None


class FlexMoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_str(status)} (status {status})")


def load_library(path: str | None = None) -> ctypes.CDLL:
    """dlopen libflexmoe.so and declare the signatures; raises if it is not built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(path)
    c_int, c_vp, c_sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.flexmoe_status_str.restype = ctypes.c_char_p
    lib.flexmoe_status_str.argtypes = [c_int]
    lib.flexmoe_workspace_bytes.restype = c_sz
    lib.flexmoe_workspace_bytes.argtypes = [c_int] * 7
    lib.flexmoe_gate_topk.restype = c_int
    lib.flexmoe_gate_topk.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.flexmoe_route.restype = c_int
    lib.flexmoe_route.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp,
                                  c_vp, c_sz, c_vp]
    lib.flexmoe_route_static.restype = c_int
    lib.flexmoe_route_static.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp,
                                         c_vp]
    lib.flexmoe_permute.restype = c_int
    lib.flexmoe_permute.argtypes = [c_vp, c_vp, c_vp, c_int, c_int, c_int, c_int, c_vp, c_vp]
    lib.flexmoe_combine.restype = c_int
    lib.flexmoe_combine.argtypes = [c_vp, c_vp, c_vp, c_int, c_int, c_int, c_int, c_vp, c_vp]
    lib.flexmoe_expert_ffn_fwd.restype = c_int
    lib.flexmoe_expert_ffn_fwd.argtypes = [c_vp] * 7 + [c_int] * 7 + [c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.flexmoe_expert_ffn_bwd.restype = c_int
    lib.flexmoe_expert_ffn_bwd.argtypes = [c_vp] * 8 + [c_int] * 7 + [c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.flexmoe_expert_ffn_fwd_gather.restype = c_int
    lib.flexmoe_expert_ffn_fwd_gather.argtypes = [c_vp] * 8 + [c_int] * 8 + [c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.flexmoe_expert_ffn_fwd_top1.restype = c_int
    lib.flexmoe_expert_ffn_fwd_top1.argtypes = [c_vp] * 8 + [c_int] * 7 + [c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.flexmoe_expert_ffn_bwd_top1.restype = c_int
    lib.flexmoe_expert_ffn_bwd_top1.argtypes = [c_vp] * 9 + [c_int] * 7 + [c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.flexmoe_gate_bwd.restype = c_int
    lib.flexmoe_gate_bwd.argtypes = [c_vp] * 10 + [c_int] * 6 + [c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    lib.flexmoe_expert_bias_grads.restype = c_int
    lib.flexmoe_expert_bias_grads.argtypes = [c_vp] * 3 + [c_int] * 6 + [c_vp, c_vp, c_vp, c_sz, c_vp]
    c_i64, c_dbl = ctypes.c_int64, ctypes.c_double
    lib.flexmoe_balance_ratio.restype = c_int
    lib.flexmoe_balance_ratio.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_vp, c_vp]
    lib.flexmoe_step_cost.restype = c_int
    lib.flexmoe_step_cost.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_i64, c_vp, c_vp]
    lib.flexmoe_make_scheduling_plan.restype = c_int
    lib.flexmoe_make_scheduling_plan.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_i64, c_vp, c_vp, c_vp, c_vp]
    lib.flexmoe_schedule.restype = c_int
    lib.flexmoe_schedule.argtypes = [c_vp, c_vp, c_int, c_int, c_int, c_i64, c_vp, c_dbl, c_int, c_vp, c_vp, c_vp,
                                     c_vp]
    lib.flexmoe_placement_table.restype = c_int
    lib.flexmoe_placement_table.argtypes = [c_vp, c_int, c_int, c_vp, c_vp, c_vp]
    if path == LIB_PATH:
        _lib = lib
    return lib


def status_str(status: int) -> str:
    return load_library().flexmoe_status_str(int(status)).decode()


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return ctypes.c_void_p(t.data_ptr())


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream():
    """Handle of torch's current stream on the current device (the stream every call is enqueued on)."""
    if _raw_stream is not None:
        return ctypes.c_void_p(_raw_stream(torch.cuda.current_device()))
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != OK:
        raise FlexMoEError(status, where)


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _host_i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def flexmoe_workspace_bytes(N, d, f, E, k, V, dtype) -> int:
    return int(load_library().flexmoe_workspace_bytes(N, d, f, E, k, V, dtype))


def flexmoe_gate_topk(x, wg, k, topk_idx, topk_w, ws):
    N, d = x.shape
    E = wg.shape[1]
    st = load_library().flexmoe_gate_topk(_ptr(x), _ptr(wg), N, d, E, k, dtype_code(x), _ptr(topk_idx), _ptr(topk_w),
                                          _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_gate_topk")


def flexmoe_route(topk_idx, E, rep_off_host, rep_ids_host, expert_count, vexpert_count, vexpert_off, vexpert_owner,
                  dest, src, ws):
    N, k = topk_idx.shape
    off, ids = _host_i32(rep_off_host), _host_i32(rep_ids_host)
    V = int(ids.shape[0])
    st = load_library().flexmoe_route(_ptr(topk_idx), N, k, E, V, off.ctypes.data_as(ctypes.c_void_p),
                                      ids.ctypes.data_as(ctypes.c_void_p), _ptr(expert_count), _ptr(vexpert_count),
                                      _ptr(vexpert_off), _ptr(vexpert_owner), _ptr(dest), _ptr(src), _ptr(ws),
                                      ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_route")


def flexmoe_route_static(topk_idx, E, rep_off_host, rep_ids_host, expert_count, vexpert_count, vexpert_off,
                         vexpert_owner, dest, src):
    N, k = topk_idx.shape
    off, ids = _host_i32(rep_off_host), _host_i32(rep_ids_host)
    V = int(ids.shape[0])
    st = load_library().flexmoe_route_static(_ptr(topk_idx), N, k, E, V, off.ctypes.data_as(ctypes.c_void_p),
                                             ids.ctypes.data_as(ctypes.c_void_p), _ptr(expert_count),
                                             _ptr(vexpert_count), _ptr(vexpert_off), _ptr(vexpert_owner), _ptr(dest),
                                             _ptr(src), _stream())
    _check(st, "flexmoe_route_static")


def flexmoe_permute(x, src, row_scale, k, xp):
    N, d = x.shape
    st = load_library().flexmoe_permute(_ptr(x), _ptr(src), _ptr(row_scale), N, k, d, dtype_code(x), _ptr(xp), _stream())
    _check(st, "flexmoe_permute")


def flexmoe_expert_ffn_bwd_top1(dyp, xp, hpre, w1, w2, vexpert_off, vexpert_owner, src, act, dx, dw1, dw2, ws, h=None):
    N, d = xp.shape
    E, _, f = w1.shape
    V = vexpert_owner.shape[0]
    st = load_library().flexmoe_expert_ffn_bwd_top1(_ptr(dyp), _ptr(xp), _ptr(hpre), _ptr(h), _ptr(w1), _ptr(w2),
                                                    _ptr(vexpert_off), _ptr(vexpert_owner), _ptr(src), N, d, f, E, V,
                                                    act, dtype_code(xp), _ptr(dx), _ptr(dw1), _ptr(dw2), _ptr(ws),
                                                    ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_expert_ffn_bwd_top1")


def flexmoe_combine(yp, dest, topk_w, k, y):
    N, d = y.shape
    st = load_library().flexmoe_combine(_ptr(yp), _ptr(dest), _ptr(topk_w), N, k, d, dtype_code(yp), _ptr(y), _stream())
    _check(st, "flexmoe_combine")


def flexmoe_expert_ffn_fwd(xp, vexpert_off, vexpert_owner, w1, b1, w2, b2, act, hpre, yp, ws, h=None):
    A, d = xp.shape
    E, _, f = w1.shape
    V = vexpert_owner.shape[0]
    st = load_library().flexmoe_expert_ffn_fwd(_ptr(xp), _ptr(vexpert_off), _ptr(vexpert_owner), _ptr(w1), _ptr(b1),
                                               _ptr(w2), _ptr(b2), A, d, f, E, V, act, dtype_code(xp), _ptr(hpre),
                                               _ptr(h), _ptr(yp), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_expert_ffn_fwd")


def flexmoe_expert_ffn_fwd_top1(x, src, vexpert_off, vexpert_owner, w1, b1, w2, b2, act, hpre, y, ws, h=None):
    N, d = x.shape
    E, _, f = w1.shape
    V = vexpert_owner.shape[0]
    st = load_library().flexmoe_expert_ffn_fwd_top1(_ptr(x), _ptr(src), _ptr(vexpert_off), _ptr(vexpert_owner),
                                                    _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2), N, d, f, E, V, act,
                                                    dtype_code(x), _ptr(hpre), _ptr(h), _ptr(y), _ptr(ws),
                                                    ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_expert_ffn_fwd_top1")


def flexmoe_expert_ffn_bwd(dyp, xp, hpre, w1, w2, vexpert_off, vexpert_owner, act, dxp, dw1, dw2, ws, h=None):
    A, d = xp.shape
    E, _, f = w1.shape
    V = vexpert_owner.shape[0]
    st = load_library().flexmoe_expert_ffn_bwd(_ptr(dyp), _ptr(xp), _ptr(hpre), _ptr(h), _ptr(w1), _ptr(w2), _ptr(vexpert_off),
                                               _ptr(vexpert_owner), A, d, f, E, V, act, dtype_code(xp), _ptr(dxp),
                                               _ptr(dw1), _ptr(dw2), _ptr(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_expert_ffn_bwd")


def flexmoe_gate_bwd(wg, topk_idx, topk_w, dy, yp, xp, dest, src, vexpert_off, vexpert_owner, dl, dx, dwg, ws):
    N, d = dy.shape
    E = wg.shape[1]
    k = topk_idx.shape[1]
    V = vexpert_owner.shape[0]
    st = load_library().flexmoe_gate_bwd(_ptr(wg), _ptr(topk_idx), _ptr(topk_w), _ptr(dy), _ptr(yp), _ptr(xp),
                                         _ptr(dest), _ptr(src), _ptr(vexpert_off), _ptr(vexpert_owner), N, d, E, k, V,
                                         dtype_code(dy), _ptr(dl), _ptr(dx), _ptr(dwg), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_gate_bwd")


def flexmoe_expert_bias_grads(dyp, vexpert_off, vexpert_owner, f, E, db1, db2, ws):
    A, d = dyp.shape
    V = vexpert_owner.shape[0]
    st = load_library().flexmoe_expert_bias_grads(_ptr(dyp), _ptr(vexpert_off), _ptr(vexpert_owner), A, d, f, E, V,
                                                  dtype_code(dyp), _ptr(db1), _ptr(db2), _ptr(ws),
                                                  ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_expert_bias_grads")


def flexmoe_expert_ffn_fwd_gather(x, src, k, vexpert_off, vexpert_owner, w1, b1, w2, b2, act, hpre, yp, ws, h=None):
    N, d = x.shape
    E, _, f = w1.shape
    V = vexpert_owner.shape[0]
    st = load_library().flexmoe_expert_ffn_fwd_gather(_ptr(x), _ptr(src), _ptr(vexpert_off), _ptr(vexpert_owner),
                                                      _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2), N, k, d, f, E, V, act,
                                                      dtype_code(x), _ptr(hpre), _ptr(h), _ptr(yp), _ptr(ws),
                                                      ws.numel() * ws.element_size(), _stream())
    _check(st, "flexmoe_expert_ffn_fwd_gather")
