"""ctypes binding of libmoe_mi355x.so: the entry points of include/moe.h under the same names.

Argument marshalling only: tensors are torch CUDA(HIP) tensors used for device memory
and the current stream; every step of the layer runs in the library's kernels.  There
is no fallback: a missing library, or a non-zero status, raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_mi355x.so")

MOE_F32, MOE_BF16 = 0, 1
FLAG_SHARED_BASE, FLAG_RESIDUAL = 1, 2
WEIGHT_FIELDS = ("router_w", "router_b", "w_gate", "w_up", "w_down",
                 "rg", "ru", "rd", "lg", "lu", "ld")
EXPORTS = ("moe_route", "moe_permute", "moe_expert_ffn", "moe_combine", "moe_forward",
           "moe_forward_static", "moe_stack_forward", "moe_forward_timed", "moe_workspace_bytes", "moe_status_string",
           "moe_expert_replacements", "moe_bles_workspace_bytes", "moe_bles_loss",
           "moe_offload_counters", "moe_delta_uniform")


class MoeShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_tokens", "d_model", "d_ff", "n_experts", "top_k",
                                          "rank", "act_dtype", "flags")]


class MoeWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class MoeError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed: {status_string(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` "
                              "(or paper_2503_00245_amd/build.py) to compile the HIP library")
        L = C.CDLL(LIB_PATH)
        L.moe_workspace_bytes.restype = C.c_size_t
        L.moe_workspace_bytes.argtypes = [C.POINTER(MoeShape)]
        L.moe_status_string.restype = C.c_char_p
        L.moe_status_string.argtypes = [C.c_int]
        vp, sz = C.c_void_p, C.c_size_t
        sp = C.POINTER(MoeShape)
        wp = C.POINTER(MoeWeights)
        L.moe_route.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp]
        L.moe_permute.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.moe_expert_ffn.argtypes = [sp, wp, vp, vp, vp, vp, sz, vp]
        L.moe_combine.argtypes = [sp, vp, vp, vp, vp, vp, vp]
        L.moe_forward.argtypes = [sp, wp, vp, vp, vp, vp, vp, sz, vp]
        L.moe_forward_static.argtypes = [sp, wp, vp, vp, vp, vp, vp]
        L.moe_stack_forward.argtypes = [sp, wp, C.c_int32, vp, vp, vp, vp, sz, vp]
        L.moe_forward_timed.argtypes = [sp, wp, vp, vp, vp, sz, vp, C.POINTER(C.c_float),
                                        C.POINTER(C.c_char_p), C.POINTER(C.c_int32)]
        i32 = C.c_int32
        L.moe_expert_replacements.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
        L.moe_bles_workspace_bytes.argtypes = [i32, i32, i32]
        L.moe_bles_workspace_bytes.restype = C.c_size_t
        L.moe_bles_loss.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
        L.moe_offload_counters.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
        L.moe_delta_uniform.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp]
        for fn in ("moe_route", "moe_permute", "moe_expert_ffn", "moe_combine", "moe_forward",
                   "moe_forward_static", "moe_stack_forward", "moe_forward_timed", "moe_expert_replacements",
                   "moe_bles_loss", "moe_offload_counters", "moe_delta_uniform"):
            getattr(L, fn).restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().moe_status_string(int(status)).decode()


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise MoeError(fn, status)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous")
    return t.data_ptr()


def _stream(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def _act_dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MOE_F32
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    raise TypeError(f"activation dtype must be float32 or bfloat16, got {t.dtype}")


def make_shape(n_tokens, d_model, d_ff, n_experts, top_k, rank=0, act_dtype=MOE_BF16,
               flags=0) -> MoeShape:
    return MoeShape(n_tokens, d_model, d_ff, n_experts, top_k, rank, act_dtype, flags)


def shape_for(weights: Dict[str, Optional[torch.Tensor]], n_tokens: int, top_k: int,
              act_dtype: int, residual: bool = False) -> MoeShape:
    """Shape struct read off a weights dict (keys as in the C struct)."""
    E, d = weights["router_w"].shape
    if weights.get("rg") is not None:
        r = weights["rg"].shape[1]
        F = weights["lg"].shape[1]
    else:
        r = 0
        F = weights["w_gate"].shape[1]
    flags = (FLAG_SHARED_BASE if (r > 0 and weights.get("w_gate") is not None) else 0) | \
            (FLAG_RESIDUAL if residual else 0)
    return make_shape(n_tokens, d, F, E, top_k, r, act_dtype, flags)


def make_weights(weights: Dict[str, Optional[torch.Tensor]]) -> MoeWeights:
    w = MoeWeights()
    for name in WEIGHT_FIELDS:
        setattr(w, name, _ptr(weights.get(name)))
    return w


def moe_workspace_bytes(shape: MoeShape) -> int:
    return int(lib().moe_workspace_bytes(C.byref(shape)))


def alloc_workspace(shape: MoeShape, device) -> torch.Tensor:
    n = moe_workspace_bytes(shape)
    if n == 0:
        raise MoeError("moe_workspace_bytes", -1)
    return torch.empty(n, dtype=torch.uint8, device=device)


def moe_route(shape: MoeShape, x, router_w, router_b, topk_idx, topk_gate, probs=None) -> None:
    _check("moe_route", lib().moe_route(C.byref(shape), _ptr(x), _ptr(router_w), _ptr(router_b),
                                        _ptr(topk_idx), _ptr(topk_gate), _ptr(probs),
                                        _stream(x.device)))


def moe_permute(shape: MoeShape, topk_idx, expert_offsets, perm, inv_perm, x=None, x_perm=None,
                workspace=None) -> None:
    _check("moe_permute", lib().moe_permute(
        C.byref(shape), _ptr(topk_idx), _ptr(expert_offsets), _ptr(perm), _ptr(inv_perm), _ptr(x),
        _ptr(x_perm), _ptr(workspace), 0 if workspace is None else workspace.numel(),
        _stream(expert_offsets.device)))


def moe_expert_ffn(shape: MoeShape, weights: MoeWeights, x_perm, expert_offsets, y_perm,
                   workspace) -> None:
    _check("moe_expert_ffn", lib().moe_expert_ffn(
        C.byref(shape), C.byref(weights), _ptr(x_perm), _ptr(expert_offsets), _ptr(y_perm),
        _ptr(workspace), workspace.numel(), _stream(y_perm.device)))


def moe_combine(shape: MoeShape, y_perm, inv_perm, topk_gate, residual, y) -> None:
    _check("moe_combine", lib().moe_combine(C.byref(shape), _ptr(y_perm), _ptr(inv_perm),
                                            _ptr(topk_gate), _ptr(residual), _ptr(y),
                                            _stream(y.device)))


def moe_forward(shape: MoeShape, weights: MoeWeights, x, y, topk_idx=None, topk_gate=None,
                workspace=None) -> None:
    _check("moe_forward", lib().moe_forward(
        C.byref(shape), C.byref(weights), _ptr(x), _ptr(y), _ptr(topk_idx), _ptr(topk_gate),
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream(y.device)))


STATIC_WORKSPACE_BYTES = 8 << 20


def moe_forward_static(shape: MoeShape, weights: MoeWeights, x, y, topk_idx=None, topk_gate=None) -> None:
    """moe_forward on the library's own scratch array: no workspace argument, no allocation."""
    _check("moe_forward_static", lib().moe_forward_static(
        C.byref(shape), C.byref(weights), _ptr(x), _ptr(y), _ptr(topk_idx), _ptr(topk_gate),
        _stream(y.device)))


def moe_stack_forward(shape: MoeShape, layers: Sequence[MoeWeights], x, y, topk_trace=None,
                      workspace=None) -> None:
    arr = (MoeWeights * len(layers))(*layers)
    _check("moe_stack_forward", lib().moe_stack_forward(
        C.byref(shape), arr, len(layers), _ptr(x), _ptr(y), _ptr(topk_trace), _ptr(workspace),
        0 if workspace is None else workspace.numel(), _stream(y.device)))


MAX_STAGES = 12


def moe_forward_timed(shape: MoeShape, weights: MoeWeights, x, y, workspace):
    """One forward with per-stage HIP-event timing; returns [(stage name, milliseconds)]."""
    ms = (C.c_float * MAX_STAGES)()
    names = (C.c_char_p * MAX_STAGES)()
    n = C.c_int32(0)
    _check("moe_forward_timed", lib().moe_forward_timed(
        C.byref(shape), C.byref(weights), _ptr(x), _ptr(y), _ptr(workspace), workspace.numel(),
        _stream(y.device), ms, names, C.byref(n)))
    return [(names[i].decode(), float(ms[i])) for i in range(n.value)]


def moe_expert_replacements(S, n_experts: int, H_e, H) -> None:
    """S int32 [B,T,K] device; H_e int64 [E], H int64 [1] device outputs."""
    B, T, K = S.shape
    _check("moe_expert_replacements", lib().moe_expert_replacements(
        _ptr(S), B, T, K, n_experts, _ptr(H_e), _ptr(H), _stream(S.device)))


def moe_bles_workspace_bytes(B: int, T: int, E: int) -> int:
    return int(lib().moe_bles_workspace_bytes(B, T, E))


def moe_bles_loss(probs, S, out, workspace) -> None:
    """probs f32 [B,T,E], S int32 [B,T,K]; out f64 [5] device: H, H_norm, L, L_norm, loss."""
    B, T, E = probs.shape
    K = S.shape[2]
    _check("moe_bles_loss", lib().moe_bles_loss(
        _ptr(probs), _ptr(S), B, T, K, E, _ptr(out), _ptr(workspace), workspace.numel(),
        _stream(probs.device)))


def moe_offload_counters(trace, n_experts: int, changes, loads) -> None:
    """trace int32 [L,T,K]; changes, loads int64 [L] device outputs."""
    L_, T, K = trace.shape
    _check("moe_offload_counters", lib().moe_offload_counters(
        _ptr(trace), L_, T, K, n_experts, _ptr(changes), _ptr(loads), _stream(trace.device)))


def moe_delta_uniform(trace, n_experts: int, counts, delta, mean) -> None:
    """trace int32 [L,T,K]; counts int64 [L,E], delta f64 [L] (or None), mean f64 [1]: device outputs."""
    L_, T, K = trace.shape
    _check("moe_delta_uniform", lib().moe_delta_uniform(
        _ptr(trace), L_, T, K, n_experts, _ptr(counts), _ptr(delta), _ptr(mean), _stream(trace.device)))
