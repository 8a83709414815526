"""ctypes front end of the C oracle (oracle/moe_oracle.c).  TEST INFRASTRUCTURE ONLY.

Arrays are numpy: fp32 tensors as float32, bf16 tensors as uint16 bit patterns.
Floating-point results come back as float64.  Nothing here does arithmetic; it
marshals arguments into the C functions, whose header states what each follows
in the paper.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None

FLAG_SHARED_BASE = 1
FLAG_RESIDUAL = 2


class _Layer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("d", "F", "E", "k", "r", "dtype", "flags")] + \
               [(n, C.c_void_p) for n in ("router_w", "router_b", "w_gate", "w_up", "w_down",
                                          "rg", "ru", "rd", "lg", "lu", "ld")]


def lib() -> C.CDLL:
    """The oracle library.  MOE_ORACLE_LIB names another build of the same source to load instead
    (the mutation check points it at deliberately broken copies)."""
    global _lib
    if _lib is None:
        path = os.environ.get("MOE_ORACLE_LIB") or _LIB_PATH
        if path == _LIB_PATH and not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        use_library(path)
    return _lib


def use_library(path: str) -> None:
    """Switch every call below to the build of the oracle at `path`."""
    global _lib
    _lib = C.CDLL(path)
    _lib.oracle_expert_replacements.restype = C.c_int64


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"activations/weights must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dtype=None):
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=dtype)


def route(x, router_w, router_b, k: int):
    """-> (topk_idx int32 [T,k], topk_gate f64 [T,k], probs f64 [T,E], logits f64 [T,E])"""
    x = _c(x)
    rw = _c(router_w, np.float32)
    rb = _c(router_b, np.float32)
    T, d = x.shape
    E = rw.shape[0]
    idx = np.zeros((T, k), np.int32)
    gate = np.zeros((T, k), np.float64)
    probs = np.zeros((T, E), np.float64)
    logits = np.zeros((T, E), np.float64)
    rc = lib().oracle_route(T, d, E, k, _dt(x), _p(x), _p(rw), _p(rb), _p(idx), _p(gate),
                            _p(probs), _p(logits))
    if rc != 0:
        raise ValueError(f"oracle_route rejected its arguments (rc={rc})")
    return idx, gate, probs, logits


def permute(topk_idx, n_experts: int):
    """-> (expert_offsets int32 [E+1], perm int32 [P], inv_perm int32 [P])"""
    flat = _c(topk_idx, np.int32).reshape(-1)
    P = flat.size
    off = np.zeros(n_experts + 1, np.int32)
    perm = np.zeros(P, np.int32)
    inv = np.zeros(P, np.int32)
    rc = lib().oracle_permute(P, n_experts, _p(flat), _p(off), _p(perm), _p(inv))
    if rc != 0:
        raise ValueError(f"oracle_permute rejected its arguments (rc={rc})")
    return off, perm, inv


def _layer(weights: Dict[str, Optional[np.ndarray]], k: int, flags: int, keep: list) -> _Layer:
    rw = _c(weights["router_w"], np.float32)
    E, d = rw.shape
    L = _Layer()
    r = 0
    ref = None
    for name in ("w_gate", "rg"):
        if weights.get(name) is not None:
            ref = weights[name]
    if ref is None:
        raise ValueError("layer has neither dense nor decomposed expert weights")
    if weights.get("rg") is not None:
        r = int(weights["rg"].shape[1])
        F = int(weights["lg"].shape[1])
    else:
        F = int(weights["w_gate"].shape[1])
    if r > 0 and weights.get("w_gate") is not None:
        flags |= FLAG_SHARED_BASE
        if weights["w_gate"].shape[0] != 1:
            raise ValueError("a base next to decomposed factors must be shared (leading dim 1)")
    L.d, L.F, L.E, L.k, L.r, L.dtype, L.flags = d, F, E, k, r, _dt(ref), flags
    for name in ("router_w", "router_b"):
        a = _c(weights.get(name), np.float32)
        keep.append(a)
        setattr(L, name, None if a is None else a.ctypes.data)
    for name in ("w_gate", "w_up", "w_down", "rg", "ru", "rd", "lg", "lu", "ld"):
        a = _c(weights.get(name))
        if a is not None and _dt(a) != L.dtype:
            raise TypeError(f"{name} dtype differs from the layer's")
        keep.append(a)
        setattr(L, name, None if a is None else a.ctypes.data)
    return L


def expert_ffn(weights, x_perm, expert_offsets, k: int = 1):
    """y_perm f64 [P,d]: each group's rows through that expert's SwiGLU block."""
    keep: list = []
    L = _layer(weights, k, 0, keep)
    xp = _c(x_perm)
    off = _c(expert_offsets, np.int32)
    P = xp.shape[0]
    y = np.zeros((P, L.d), np.float64)
    rc = lib().oracle_expert_ffn(C.byref(L), P, _p(xp), _p(off), _p(y))
    if rc != 0:
        raise ValueError(f"oracle_expert_ffn rejected its arguments (rc={rc})")
    return y


def combine(y_perm, inv_perm, topk_gate, residual=None):
    """y f64 [T,d] from y_perm f64 [P,d], inv_perm [P], gates f64 [T,k]."""
    yp = _c(y_perm, np.float64)
    g = _c(topk_gate, np.float64)
    inv = _c(inv_perm, np.int32).reshape(-1)
    T, k = g.shape
    d = yp.shape[1]
    res = _c(residual)
    y = np.zeros((T, d), np.float64)
    lib().oracle_combine(T, d, k, 0 if res is None else _dt(res), _p(yp), _p(inv), _p(g),
                         _p(res), _p(y))
    return y


def forward(weights, x, k: int, residual: bool = False):
    """-> (y f64 [T,d], topk_idx int32 [T,k], topk_gate f64 [T,k]); never permutes."""
    keep: list = []
    L = _layer(weights, k, FLAG_RESIDUAL if residual else 0, keep)
    x = _c(x)
    if _dt(x) != L.dtype:
        raise TypeError("x dtype differs from the expert weights'")
    T = x.shape[0]
    y = np.zeros((T, L.d), np.float64)
    idx = np.zeros((T, k), np.int32)
    gate = np.zeros((T, k), np.float64)
    rc = lib().oracle_forward(C.byref(L), T, _p(x), _p(y), _p(idx), _p(gate))
    if rc != 0:
        raise ValueError(f"oracle_forward rejected its arguments (rc={rc})")
    return y, idx, gate


def stack_forward(layers: Sequence[dict], x, k: int):
    """-> (y f64 [T,d], trace int32 [L,T,k], xs f64 [L+1,T,d] inputs of each layer + output)"""
    keep: list = []
    n = len(layers)
    arr = (_Layer * n)(*[_layer(w, k, FLAG_RESIDUAL, keep) for w in layers])
    x = _c(x)
    T, d = x.shape
    y = np.zeros((T, d), np.float64)
    trace = np.zeros((n, T, k), np.int32)
    xs = np.zeros((n + 1, T, d), np.float64)
    rc = lib().oracle_stack_forward(arr, n, T, _p(x), _p(y), _p(trace), _p(xs))
    if rc != 0:
        raise ValueError(f"oracle_stack_forward rejected its arguments (rc={rc})")
    return y, trace, xs


def expert_replacements(S, n_experts: int):
    """Eq. 4: (H, H_e[E]) for selected experts S int32 [B,T,K]."""
    S = _c(S, np.int32)
    B, T, K = S.shape
    He = np.zeros(n_experts, np.int64)
    H = lib().oracle_expert_replacements(B, T, K, n_experts, _p(S), _p(He))
    return int(H), He


def bles_loss(probs, S):
    """Eq. 4-7 forward value: dict(H, H_norm, L, L_norm, loss) for probs f32 [B,T,E], S int32 [B,T,K]."""
    W = _c(probs, np.float32)
    S = _c(S, np.int32)
    B, T, E = W.shape
    K = S.shape[2]
    out = np.zeros(5, np.float64)
    rc = lib().oracle_bles_loss(B, T, K, E, _p(W), _p(S), _p(out))
    if rc != 0:
        raise ValueError(f"oracle_bles_loss rejected its arguments (rc={rc})")
    return dict(H=int(out[0]), H_norm=out[1], L=out[2], L_norm=out[3], loss=out[4])


def offload_counters(trace, n_experts: int):
    """Sec. 3.4.2 offloading rule on a routing trace int32 [L,T,K] -> (changes int64 [L], loads int64 [L])."""
    tr = _c(trace, np.int32)
    L, T, K = tr.shape
    ch = np.zeros(L, np.int64)
    ld = np.zeros(L, np.int64)
    rc = lib().oracle_offload_counters(L, T, K, n_experts, _p(tr), _p(ch), _p(ld))
    if rc != 0:
        raise ValueError(f"oracle_offload_counters rejected its arguments (rc={rc})")
    return ch, ld


def delta_uniform(trace, n_experts: int):
    """Sec. 3.2 / Table 3 "Delta Uniform" of a routing trace int32 [L,T,K] ->
    (mean over layers, per-layer delta f64 [L], counts int64 [L,E]); fractions, not percent."""
    tr = _c(trace, np.int32)
    L, T, K = tr.shape
    counts = np.zeros((L, n_experts), np.int64)
    delta = np.zeros(L, np.float64)
    mean = np.zeros(1, np.float64)
    rc = lib().oracle_delta_uniform(L, T, K, n_experts, _p(tr), _p(counts), _p(delta), _p(mean))
    if rc != 0:
        raise ValueError(f"oracle_delta_uniform rejected its arguments (rc={rc})")
    return float(mean[0]), delta, counts
