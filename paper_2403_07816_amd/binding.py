"""ctypes binding of libbtx_moe.so: same names as the C ABI (include/btx_moe.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream; every step of the layer runs in the library's kernels.  There is no
fallback: if the shared library is missing, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

BTX_F32, BTX_BF16 = 0, 1
BTX_ROUTE_TOPK_RENORM, BTX_ROUTE_SWITCH_TOP1, BTX_ROUTE_SAMPLE_TOP1, BTX_ROUTE_GUMBEL_TOP1 = 0, 1, 2, 3
BTX_LB_TOKEN_FRAC, BTX_LB_GATE_MEAN = 0, 1
BTX_FLAG_LB_GRAD_THROUGH_U = 1
STAGE_NAMES = ["route", "gather_x", "up_swiglu", "down", "combine", "gather_dy", "bwd_act", "bwd_dx", "gather_x_bwd",
               "dw13", "dw2", "router_bwd", "norm_bwd"]

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libbtx_moe.so")
_lib = None

_vp, _i, _i64, _f, _sz, _u = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t,
                              ctypes.c_uint)
_SIGNATURES = {
    "btx_status_string": (ctypes.c_char_p, [_i]),
    "btx_version": (_i, []),
    "btx_profile_stages": (_i, [ctypes.POINTER(_vp), _i]),
    "btx_init": (_i, []),
    "btx_moe_route_workspace_bytes": (_sz, [_i, _i, _i, _i]),
    "btx_moe_route": (_i, [_vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _f, _f, _f] + [_vp] * 10 + [_vp, _sz, _vp]),
    "btx_moe_route_noalloc_max_workspace_bytes": (_sz, []),
    "btx_moe_route_noalloc": (_i, [_vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _f, _f, _f] + [_vp] * 10 + [_vp]),
    "btx_moe_norm_route": (_i, [_vp, _i, _vp, _f, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _f, _f, _f] + [_vp] * 10 +
                           [_vp, _sz, _vp]),
    "btx_rmsnorm_backward_workspace_bytes": (_sz, [_i, _i]),
    "btx_rmsnorm_backward": (_i, [_vp] * 5 + [_i, _i, _i, _vp, _vp, _vp, _sz, _vp]),
    "btx_moe_ff_forward_workspace_bytes": (_sz, [_i] * 6),
    "btx_moe_ff_forward": (_i, [_vp, _vp, _vp, _vp, _i, _i64, _i64, _i, _i, _i, _i, _i] + [_vp] * 4 + [_vp] * 4 +
                           [_vp, _sz, _vp]),
    "btx_moe_ff_backward_workspace_bytes": (_sz, [_i] * 6),
    "btx_moe_ff_backward": (_i, [_vp] * 6 + [_i, _i64, _i64] + [_i] * 7 + [_f, _f, _u, _vp, _f] + [_vp] * 11 + [_vp] * 6 +
                            [_i, _vp, _sz, _vp]),
    "btx_merge_average": (_i, [ctypes.POINTER(_vp), _i, _vp, _i64, _i, _vp]),
    "btx_merge_weighted": (_i, [ctypes.POINTER(_vp), ctypes.POINTER(ctypes.c_float), _i, _vp, _i64, _i, _vp]),
    "btx_adamw_step": (_i, [_vp, _vp, _vp, _vp, _i, _vp, _i64, _i, _f, _f, _f, _f, _f, _vp]),
    "btx_mix_experts": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp]),
}


def load_library() -> ctypes.CDLL:
    """Load the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2403_07816_amd.build` "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


class BtxError(RuntimeError):
    pass


def _check(status: int, what: str) -> None:
    if status != 0:
        raise BtxError(f"{what}: {load_library().btx_status_string(status).decode()} (status {status})")


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return BTX_F32
    if t.dtype == torch.bfloat16:
        return BTX_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor], stacked: bool = False):
    """Device address of a contiguous tensor (stacked: of expert matrices that _stacked() accepts)."""
    if t is None:
        return None
    assert t.is_cuda and (t.is_contiguous() or (stacked and _stacked(t))), "device-resident contiguous tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> torch.Tensor:
    if workspace is not None and workspace.numel() * workspace.element_size() >= nbytes:
        return workspace
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


@dataclass
class Routing:
    topk_idx: torch.Tensor   # [T,k] int32
    gates: torch.Tensor      # [T,k] fp32
    probs: torch.Tensor      # [T,E] fp32
    counts: torch.Tensor     # [E] int32
    offsets: torch.Tensor    # [E+1] int32
    perm: torch.Tensor       # [T*k] int32
    inv_pos: torch.Tensor    # [T,k] int32
    gate_sum: torch.Tensor   # [E] fp32
    prob_sum: torch.Tensor   # [E] fp32
    lb_loss: torch.Tensor    # [1] fp32


def alloc_routing(T: int, E: int, k: int, device) -> Routing:
    i32 = dict(dtype=torch.int32, device=device)
    f32 = dict(dtype=torch.float32, device=device)
    return Routing(torch.empty((T, k), **i32), torch.empty((T, k), **f32), torch.empty((T, E), **f32),
                   torch.zeros(E, **i32), torch.zeros(E + 1, **i32), torch.empty(T * k, **i32),
                   torch.empty((T, k), **i32), torch.zeros(E, **f32), torch.zeros(E, **f32), torch.zeros(1, **f32))


def btx_moe_route(x: torch.Tensor, W_router: torch.Tensor, b_router: Optional[torch.Tensor] = None,
                  U: Optional[torch.Tensor] = None, k: int = 2, route_mode: int = BTX_ROUTE_TOPK_RENORM,
                  lb_mode: int = BTX_LB_TOKEN_FRAC, lb_alpha: float = 0.0, out: Optional[Routing] = None,
                  workspace: Optional[torch.Tensor] = None, tau: float = 1.0,
                  capacity_factor: float = 0.0) -> Routing:
    """U: uniforms [T] for SAMPLE_TOP1, Gumbel noise [T,E] (with temperature tau) for GUMBEL_TOP1."""
    lib = load_library()
    T, d = x.shape
    E = W_router.shape[1]
    assert W_router.shape[0] == d and W_router.dtype == torch.float32
    r = out if out is not None else alloc_routing(T, E, k, x.device)
    ws = _workspace(lib.btx_moe_route_workspace_bytes(T, d, E, k), x.device, workspace)
    st = lib.btx_moe_route(_ptr(x), _dtype_code(x), _ptr(W_router), _ptr(b_router), _ptr(U), T, d, E, k, route_mode,
                           lb_mode, lb_alpha, tau, capacity_factor, _ptr(r.topk_idx), _ptr(r.gates), _ptr(r.probs), _ptr(r.counts),
                           _ptr(r.offsets), _ptr(r.perm), _ptr(r.inv_pos), _ptr(r.gate_sum), _ptr(r.prob_sum),
                           _ptr(r.lb_loss), _ptr(ws), ws.numel(), _stream())
    _check(st, "btx_moe_route")
    return r


def btx_moe_route_noalloc(x: torch.Tensor, W_router: torch.Tensor, out: Routing, b_router: Optional[torch.Tensor] = None,
                          U: Optional[torch.Tensor] = None, k: int = 2, route_mode: int = BTX_ROUTE_TOPK_RENORM,
                          lb_mode: int = BTX_LB_TOKEN_FRAC, lb_alpha: float = 0.0, tau: float = 1.0,
                          capacity_factor: float = 0.0) -> Routing:
    """btx_moe_route into caller-allocated outputs, with the library's fixed workspace: allocates nothing."""
    lib = load_library()
    T, d = x.shape
    E = W_router.shape[1]
    assert W_router.shape[0] == d and W_router.dtype == torch.float32
    r = out
    st = lib.btx_moe_route_noalloc(_ptr(x), _dtype_code(x), _ptr(W_router), _ptr(b_router), _ptr(U), T, d, E, k,
                                   route_mode, lb_mode, lb_alpha, tau, capacity_factor, _ptr(r.topk_idx), _ptr(r.gates),
                                   _ptr(r.probs), _ptr(r.counts), _ptr(r.offsets), _ptr(r.perm), _ptr(r.inv_pos),
                                   _ptr(r.gate_sum), _ptr(r.prob_sum), _ptr(r.lb_loss), _stream())
    _check(st, "btx_moe_route_noalloc")
    return r


def btx_moe_norm_route(h: torch.Tensor, gain: torch.Tensor, eps: float, W_router: torch.Tensor,
                       b_router: Optional[torch.Tensor] = None, U: Optional[torch.Tensor] = None, k: int = 2,
                       route_mode: int = BTX_ROUTE_TOPK_RENORM, lb_mode: int = BTX_LB_TOKEN_FRAC, lb_alpha: float = 0.0,
                       out: Optional[Routing] = None, workspace: Optional[torch.Tensor] = None, tau: float = 1.0,
                       capacity_factor: float = 0.0, xn: Optional[torch.Tensor] = None,
                       rstd: Optional[torch.Tensor] = None):
    """RMS-normalise the rows of h (gain [d] fp32) and route on the result.  Returns (routing, xn, rstd)."""
    lib = load_library()
    T, d = h.shape
    E = W_router.shape[1]
    assert W_router.shape[0] == d and W_router.dtype == torch.float32
    assert gain.shape == (d,) and gain.dtype == torch.float32 and h.is_contiguous()
    r = out if out is not None else alloc_routing(T, E, k, h.device)
    xn = xn if xn is not None else torch.empty_like(h)
    rstd = rstd if rstd is not None else torch.empty(T, dtype=torch.float32, device=h.device)
    ws = _workspace(lib.btx_moe_route_workspace_bytes(T, d, E, k), h.device, workspace)
    st = lib.btx_moe_norm_route(_ptr(h), _dtype_code(h), _ptr(gain), eps, _ptr(xn), _ptr(rstd), _ptr(W_router),
                                _ptr(b_router), _ptr(U), T, d, E, k, route_mode, lb_mode, lb_alpha, tau, capacity_factor,
                                _ptr(r.topk_idx), _ptr(r.gates), _ptr(r.probs), _ptr(r.counts), _ptr(r.offsets),
                                _ptr(r.perm), _ptr(r.inv_pos), _ptr(r.gate_sum), _ptr(r.prob_sum), _ptr(r.lb_loss),
                                _ptr(ws), ws.numel(), _stream())
    _check(st, "btx_moe_norm_route")
    return r, xn, rstd


def btx_rmsnorm_backward(dXn: torch.Tensor, h: torch.Tensor, gain: torch.Tensor, rstd: torch.Tensor,
                         dres: Optional[torch.Tensor] = None, dH: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, dgain: Optional[torch.Tensor] = None):
    """Returns (dH [T,d], dgain [d] fp32); dres (e.g. the layer's dY) is added to dH."""
    lib = load_library()
    T, d = h.shape
    assert dXn.shape == h.shape and dXn.dtype == h.dtype and dXn.is_contiguous() and h.is_contiguous()
    assert gain.dtype == torch.float32 and rstd.dtype == torch.float32 and rstd.numel() == T
    assert dres is None or (dres.shape == h.shape and dres.dtype == h.dtype and dres.is_contiguous())
    dH = dH if dH is not None else torch.empty_like(h)
    dgain = dgain if dgain is not None else torch.empty(d, dtype=torch.float32, device=h.device)
    ws = _workspace(lib.btx_rmsnorm_backward_workspace_bytes(T, d), h.device, workspace)
    st = lib.btx_rmsnorm_backward(_ptr(dXn), _ptr(h), _ptr(gain), _ptr(rstd), _ptr(dres), _dtype_code(h), T, d,
                                  _ptr(dH), _ptr(dgain), _ptr(ws), ws.numel(), _stream())
    _check(st, "btx_rmsnorm_backward")
    return dH, dgain


def _stacked(W: torch.Tensor) -> Tuple[int, int]:
    """(experts, expert stride in elements) of stacked expert matrices: each [rows, cols] matrix contiguous,
    the experts any multiple of 8 elements apart."""
    assert W.dim() == 3 and W.stride(2) == 1 and W.stride(1) == W.shape[2] and W.stride(0) >= W.shape[1] * W.shape[2]
    return W.shape[0], W.stride(0)


def btx_moe_ff_forward(x: torch.Tensor, W1: torch.Tensor, W3: torch.Tensor, W2: torch.Tensor, routing: Routing,
                       save: bool = True, out: Optional[torch.Tensor] = None,
                       saved: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
                       workspace: Optional[torch.Tensor] = None, residual: Optional[torch.Tensor] = None):
    """Returns (out[T,d], h1, h3); h1/h3 are None when save=False.  residual[T,d] is added to out."""
    lib = load_library()
    T, d = x.shape
    E, s13 = _stacked(W1)
    _, s2 = _stacked(W2)
    f = W1.shape[2]
    k = routing.topk_idx.shape[1]
    dt = _dtype_code(x)
    assert W1.dtype == x.dtype and W3.shape == W1.shape and W2.shape == (E, f, d)
    out = out if out is not None else torch.empty_like(x)
    h1 = h3 = None
    if save:
        h1, h3 = saved if saved is not None else (torch.empty((T * k, f), dtype=x.dtype, device=x.device),
                                                  torch.empty((T * k, f), dtype=x.dtype, device=x.device))
    ws = _workspace(lib.btx_moe_ff_forward_workspace_bytes(T, d, f, E, k, dt), x.device, workspace)
    st = lib.btx_moe_ff_forward(_ptr(x), _ptr(W1, True), _ptr(W3, True), _ptr(W2, True), dt, s13, s2, T, d, f, E, k,
                                _ptr(routing.gates), _ptr(routing.offsets), _ptr(routing.perm), _ptr(routing.inv_pos),
                                _ptr(residual), _ptr(out), _ptr(h1), _ptr(h3), _ptr(ws), ws.numel(), _stream())
    _check(st, "btx_moe_ff_forward")
    return out, h1, h3


@dataclass
class Grads:
    dX: torch.Tensor
    dW_router: torch.Tensor
    db_router: torch.Tensor
    dW1: Optional[torch.Tensor]
    dW3: Optional[torch.Tensor]
    dW2: Optional[torch.Tensor]


def btx_moe_ff_backward(dY: torch.Tensor, x: torch.Tensor, W_router: torch.Tensor, W1: torch.Tensor,
                        W3: torch.Tensor, W2: torch.Tensor, routing: Routing, h1: torch.Tensor, h3: torch.Tensor,
                        route_mode: int = BTX_ROUTE_TOPK_RENORM, lb_mode: int = BTX_LB_TOKEN_FRAC,
                        lb_alpha: float = 0.0, lb_grad_scale: float = 0.0, flags: int = 0,
                        dW_dtype: Optional[torch.dtype] = None, frozen_experts: bool = False,
                        out: Optional[Grads] = None, workspace: Optional[torch.Tensor] = None,
                        noise: Optional[torch.Tensor] = None, tau: float = 1.0) -> Grads:
    lib = load_library()
    T, d = x.shape
    E, s13 = _stacked(W1)
    _, s2 = _stacked(W2)
    f = W1.shape[2]
    k = routing.topk_idx.shape[1]
    dt = _dtype_code(x)
    dW_dtype = x.dtype if dW_dtype is None else dW_dtype
    if out is None:
        # weight gradients are stacked like the weights: same expert strides
        mk = (lambda W: None) if frozen_experts else (
            lambda W: torch.empty_strided(W.shape, W.stride(), dtype=dW_dtype, device=x.device))
        out = Grads(torch.empty_like(x), torch.empty((d, W_router.shape[1]), dtype=torch.float32, device=x.device),
                    torch.empty(W_router.shape[1], dtype=torch.float32, device=x.device), mk(W1), mk(W3), mk(W2))
    for dW, W in ((out.dW1, W1), (out.dW3, W3), (out.dW2, W2)):
        assert dW is None or (dW.shape == W.shape and _stacked(dW)[1] == _stacked(W)[1]), "dW is stacked like W"
    dwc = BTX_F32 if dW_dtype == torch.float32 else BTX_BF16
    ws = _workspace(lib.btx_moe_ff_backward_workspace_bytes(T, d, f, E, k, dt), x.device, workspace)
    st = lib.btx_moe_ff_backward(_ptr(dY), _ptr(x), _ptr(W_router), _ptr(W1, True), _ptr(W3, True), _ptr(W2, True), dt, s13, s2,
                                 T, d, f,
                                 E, k, route_mode, lb_mode, lb_alpha, lb_grad_scale, flags, _ptr(noise), tau,
                                 _ptr(routing.topk_idx),
                                 _ptr(routing.gates), _ptr(routing.probs), _ptr(routing.offsets), _ptr(routing.perm),
                                 _ptr(routing.inv_pos), _ptr(routing.gate_sum), _ptr(routing.prob_sum),
                                 _ptr(routing.counts), _ptr(h1), _ptr(h3), _ptr(out.dX), _ptr(out.dW_router),
                                 _ptr(out.db_router), _ptr(out.dW1, True), _ptr(out.dW3, True), _ptr(out.dW2, True), dwc, _ptr(ws),
                                 ws.numel(), _stream())
    _check(st, "btx_moe_ff_backward")
    return out


def btx_merge_average(tensors: Sequence[torch.Tensor], out: Optional[torch.Tensor] = None) -> torch.Tensor:
    lib = load_library()
    t0 = tensors[0]
    for t in tensors:
        assert t.shape == t0.shape and t.dtype == t0.dtype and t.is_cuda and t.is_contiguous()
    out = out if out is not None else torch.empty_like(t0)
    arr = (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
    st = lib.btx_merge_average(arr, len(tensors), _ptr(out), t0.numel(), _dtype_code(t0), _stream())
    _check(st, "btx_merge_average")
    return out


def btx_merge_weighted(tensors: Sequence[torch.Tensor], weights: Sequence[float],
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
    lib = load_library()
    t0 = tensors[0]
    assert len(weights) == len(tensors)
    for t in tensors:
        assert t.shape == t0.shape and t.dtype == t0.dtype and t.is_cuda and t.is_contiguous()
    out = out if out is not None else torch.empty_like(t0)
    arr = (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
    wts = (ctypes.c_float * len(tensors))(*[float(w) for w in weights])
    st = lib.btx_merge_weighted(arr, wts, len(tensors), _ptr(out), t0.numel(), _dtype_code(t0), _stream())
    _check(st, "btx_merge_weighted")
    return out


def btx_init() -> None:
    """One-time set-up of the library on the current device (see btx_moe.h)."""
    _check(load_library().btx_init(), "btx_init")


def btx_adamw_step(master: torch.Tensor, m: torch.Tensor, v: torch.Tensor, grad: torch.Tensor, step: int, lr: float,
                   beta1: float = 0.9, beta2: float = 0.95, eps: float = 1e-8, weight_decay: float = 0.1,
                   lowp: Optional[torch.Tensor] = None) -> None:
    """In-place fused AdamW on fp32 master weights and moments; lowp (bf16) receives the rounded weights."""
    lib = load_library()
    assert master.dtype == m.dtype == v.dtype == torch.float32 and master.numel() == m.numel() == v.numel() == grad.numel()
    assert lowp is None or (lowp.dtype == torch.bfloat16 and lowp.numel() == master.numel())
    st = lib.btx_adamw_step(_ptr(master), _ptr(m), _ptr(v), _ptr(grad), _dtype_code(grad), _ptr(lowp), master.numel(),
                            step, lr, beta1, beta2, eps, weight_decay, _stream())
    _check(st, "btx_adamw_step")


BTX_MIX_SPLIT, BTX_MIX_BLEND = 0, 1


def btx_mix_experts(W1: torch.Tensor, W3: torch.Tensor, W2: torch.Tensor, mode: int, C: int = 1):
    """Stacked experts [N,d,f] / [N,f,d] -> split ([N*C,d,f/C], [N*C,f/C,d]) or blended
    ([N,d,f], [N,f,d]) copies, made by the library's copy kernels."""
    lib = load_library()
    N, d, f = W1.shape
    assert W3.shape == W1.shape and W2.shape == (N, f, d) and W1.dtype == W3.dtype == W2.dtype
    n_out, fo = (N * C, f // max(C, 1)) if mode == BTX_MIX_SPLIT else (N, f)
    o1 = torch.empty((n_out, d, fo), dtype=W1.dtype, device=W1.device)
    o3 = torch.empty_like(o1)
    o2 = torch.empty((n_out, fo, d), dtype=W1.dtype, device=W1.device)
    st = lib.btx_mix_experts(_ptr(W1), _ptr(W3), _ptr(W2), _dtype_code(W1), N, d, f, mode, C, _ptr(o1), _ptr(o3),
                             _ptr(o2), _stream())
    _check(st, "btx_mix_experts")
    return o1, o3, o2


def split_experts(W1: torch.Tensor, W3: torch.Tensor, W2: torch.Tensor, C: int):
    """Sec. 3.3 "Splitting Experts": expert i*C+c owns columns c*f/C.. of W1_i, W3_i and the
    same rows of W2_i."""
    return btx_mix_experts(W1, W3, W2, BTX_MIX_SPLIT, C)


def blend_experts(W1: torch.Tensor, W3: torch.Tensor, W2: torch.Tensor):
    """Sec. 3.3 "Blending Experts": expert n = the n-th of N chunks of every FF, FF after FF."""
    return btx_mix_experts(W1, W3, W2, BTX_MIX_BLEND)
