"""Seeded tensor recipes for the five benchmark configurations.

Every tensor is drawn on the host from numpy's Philox generator, keyed by
(config seed, tensor id, sub-index), rounded once to its storage dtype, and
handed bit-for-bit to both the CPU oracle and the GPU library.  bf16 tensors
are carried as uint16 bit patterns (numpy has no bf16 type).

Shapes follow the layer as the paper states it (Sec. 2.1: a router plus E
experts replacing the dense feed-forward block; Sec. 3.1: eight experts, two
active per token; Sec. 2.2 / Eq. 1: an expert matrix M of shape n x m replaced
by L (n x r) times R (r x m)).  Widths are the benchmark's, not Table 1's.
"""
from __future__ import annotations

import json
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))

# tensor ids used to derive independent Philox streams from one config seed
_TID = {
    "x": 1, "router_w": 2, "w_gate": 3, "w_up": 4, "w_down": 5,
    "rg": 6, "ru": 7, "rd": 8, "lg": 9, "lu": 10, "ld": 11,
}


@dataclass(frozen=True)
class LayerConfig:
    name: str
    d_model: int
    d_ff: int
    n_experts: int
    top_k: int
    act_dtype: str            # "f32" or "bf16": storage type of x, y and expert weights
    seed: int
    rank: int = 0             # 0: dense experts; >0: weight-decomposed experts of this rank
    shared_base: bool = False  # True: one dense SwiGLU base shared by all experts, added to L.R
    zipf: bool = False        # True: router bias loaded from the stored calibration
    n_layers: int = 1
    weight_std: float = 0.02
    router_std: float = 0.02
    wd_product_std: float = 0.02  # target std of the entries of L.R
    down_std: Optional[float] = None  # std of the dense down projection; None: weight_std


CONFIGS: Dict[str, LayerConfig] = {
    # tiny fp32 case the oracle finishes at once
    "tiny": LayerConfig("tiny", 128, 256, 4, 2, "f32", 245001),
    # wearables-shaped layer (~200M-active class)
    "wearables": LayerConfig("wearables", 1024, 2816, 8, 2, "bf16", 245002),
    # phone-shaped layer (~1.4B-active class), Zipf(1.1)-skewed expert loads
    "phone": LayerConfig("phone", 2048, 5632, 8, 2, "bf16", 245003, zipf=True),
    # phone-shaped, weight-decomposed as the paper's text defines it: pure L.R, r = d_model/2
    "phone_wd": LayerConfig("phone_wd", 2048, 5632, 8, 2, "bf16", 245004, rank=1024),
    # phone-shaped, shared dense base plus a rank-64 expert-specific pair
    "phone_wd_base": LayerConfig("phone_wd_base", 2048, 5632, 8, 2, "bf16", 245014,
                                 rank=64, shared_base=True, wd_product_std=0.005),
    # 24 phone-shaped layers run back to back with residual adds.  The stack has no normalisation,
    # and a SwiGLU block is quadratic in the size of its input, so with every matrix at N(0, 0.02)
    # the residual stream squares its size every layer once it exceeds about 2 and overflows
    # (fp64 included) by the 13th layer.  The down projections are therefore drawn with the usual
    # residual-branch scaling 0.02 / sqrt(2 n_layers), which keeps the stream's rms near 1.
    "phone_stack": LayerConfig("phone_stack", 2048, 5632, 8, 2, "bf16", 245005, n_layers=24,
                               down_std=0.02 / (2 * 24) ** 0.5),
    # The paper's own model rows (Table 1: hidden size per row; d_ff taken as 8/3 of it, rounded to
    # a multiple of 8; 8 experts, 2 active as in Sec. 3.1).  Widths that are not multiples of 64.
    "paper_phone": LayerConfig("paper_phone", 1440, 3840, 8, 2, "bf16", 245021),
    "paper_wearables": LayerConfig("paper_wearables", 432, 1152, 8, 2, "bf16", 245022),
    # weight-decomposed rows: rank = half the hidden size (Sec. 2.2)
    "paper_phone_wd": LayerConfig("paper_phone_wd", 1600, 4264, 8, 2, "bf16", 245023, rank=800),
    "paper_wearables_wd": LayerConfig("paper_wearables_wd", 400, 1064, 8, 2, "bf16", 245024, rank=200),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + (np.uint32(0x7FFF) + lsb)
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(u: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the fp32 values they denote (exact)."""
    w = np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return w.view(np.float32)


def _rng(seed: int, tid: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, tid, sub])))


def normal_tensor(seed: int, tid: int, shape, std: float, dtype: str,
                  sub: int = 0) -> np.ndarray:
    """N(0, std) tensor; dtype 'f32' -> float32 array, 'bf16' -> uint16 bit patterns.

    A leading dimension > 1 is drawn slice by slice (one Philox stream per
    slice) so large expert stacks never hold a second full-size temporary.
    """
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.float32 if dtype == "f32" else np.uint16)
    lead = shape[0] if len(shape) > 1 else 1
    view = out.reshape((lead, -1))
    for i in range(lead):
        g = _rng(seed, tid, sub * 4096 + i)
        v = g.standard_normal(view.shape[1], dtype=np.float32)
        v *= np.float32(std)
        view[i] = v if dtype == "f32" else f32_to_bf16_bits(v)
    return out


def zipf_target_shares(n_experts: int, s: float = 1.1) -> np.ndarray:
    """Target share of the T*k assignments for expert i: proportional to (i+1)^-s."""
    w = np.arange(1, n_experts + 1, dtype=np.float64) ** (-s)
    return w / w.sum()


def stored_zipf_bias(name: str) -> Optional[np.ndarray]:
    """Router bias calibrated offline (by the oracle-side calibration script) for
    the named config, or None if none is stored."""
    path = os.path.join(_HERE, "zipf_bias.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    if name not in table:
        return None
    return np.asarray(table[name]["router_b"], dtype=np.float32)


def make_inputs(cfg: LayerConfig, n_tokens: int, step: int = 0) -> np.ndarray:
    """Token activations x [T, d_model] ~ N(0, 1) in cfg.act_dtype storage."""
    return normal_tensor(cfg.seed, _TID["x"], (1, n_tokens * cfg.d_model), 1.0,
                         cfg.act_dtype, sub=1 + step).reshape(n_tokens, cfg.d_model)


def make_layer_weights(cfg: LayerConfig, layer: int = 0,
                       with_bias: Optional[bool] = None) -> Dict[str, Optional[np.ndarray]]:
    """All weights of one layer as a dict keyed like the C weights struct.

    Dense experts (or the shared base): w_gate, w_up [Eb, F, d], w_down [Eb, d, F]
    with Eb = E, or 1 for a shared base.  Weight-decomposed experts: for each
    matrix M of shape out x in, R_M [E, r, in] (applied first) and L_M [E, out, r].
    """
    d, F, E, r = cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.rank
    seed = cfg.seed + 1000 * layer
    dt = cfg.act_dtype
    w: Dict[str, Optional[np.ndarray]] = {k: None for k in
                                          ("router_w", "router_b", "w_gate", "w_up", "w_down",
                                           "rg", "ru", "rd", "lg", "lu", "ld")}
    w["router_w"] = normal_tensor(seed, _TID["router_w"], (E, d), cfg.router_std, "f32")
    use_bias = cfg.zipf if with_bias is None else with_bias
    if use_bias:
        b = stored_zipf_bias(cfg.name)
        if b is None:
            raise RuntimeError(f"no stored router bias for config {cfg.name!r}")
        w["router_b"] = b
    if r == 0 or cfg.shared_base:
        eb = 1 if cfg.shared_base else E
        w["w_gate"] = normal_tensor(seed, _TID["w_gate"], (eb, F, d), cfg.weight_std, dt)
        w["w_up"] = normal_tensor(seed, _TID["w_up"], (eb, F, d), cfg.weight_std, dt)
        w["w_down"] = normal_tensor(seed, _TID["w_down"], (eb, d, F),
                                    cfg.weight_std if cfg.down_std is None else cfg.down_std, dt)
    if r > 0:
        sigma = float(np.sqrt(cfg.wd_product_std / np.sqrt(r)))
        w["rg"] = normal_tensor(seed, _TID["rg"], (E, r, d), sigma, dt)
        w["ru"] = normal_tensor(seed, _TID["ru"], (E, r, d), sigma, dt)
        w["rd"] = normal_tensor(seed, _TID["rd"], (E, r, F), sigma, dt)
        w["lg"] = normal_tensor(seed, _TID["lg"], (E, F, r), sigma, dt)
        w["lu"] = normal_tensor(seed, _TID["lu"], (E, F, r), sigma, dt)
        w["ld"] = normal_tensor(seed, _TID["ld"], (E, d, r), sigma, dt)
    return w


def make_stack_weights(cfg: LayerConfig, n_layers: Optional[int] = None, workers: int = 8):
    """Independent weights for each layer of a residual stack (list of dicts)."""
    n = cfg.n_layers if n_layers is None else n_layers
    with ThreadPoolExecutor(max_workers=max(1, min(workers, n))) as ex:
        return list(ex.map(lambda l: make_layer_weights(cfg, layer=l), range(n)))


def shrink(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of cfg with some fields replaced (tests use reduced widths)."""
    return replace(cfg, **kw)
