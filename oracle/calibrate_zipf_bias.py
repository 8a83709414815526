"""Writes workloads/zipf_bias.json: the router bias that skews the phone-shaped layer's expert
loads to a Zipf(1.1) distribution on its own seeded 2048-token batch.

Input preparation, run once and committed; it calls only the CPU oracle (for the routing
decision) and the seeded input recipes.  Deterministic fixed-point iteration on the shares
of the T*k assignments:  b_e <- b_e + eta * (log target_e - log observed_e),  stopped when
every share is within 0.5 % absolute of its target.  Expert 0 gets the largest share.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402
from oracle import moe_oracle  # noqa: E402

OUT = os.path.join(ROOT, "workloads", "zipf_bias.json")


def calibrate(name: str, n_tokens: int = 2048, s: float = 1.1, eta: float = 0.7,
              tol: float = 0.005, max_iter: int = 200):
    cfg = wl.CONFIGS[name]
    w = wl.make_layer_weights(cfg, with_bias=False)
    x = wl.make_inputs(cfg, n_tokens)
    target = wl.zipf_target_shares(cfg.n_experts, s)
    b = np.zeros(cfg.n_experts, np.float32)
    for it in range(max_iter):
        idx, _, _, _ = moe_oracle.route(x, w["router_w"], b, cfg.top_k)
        share = np.bincount(idx.reshape(-1), minlength=cfg.n_experts) / idx.size
        err = np.abs(share - target).max()
        if err < tol:
            break
        b = (b + eta * (np.log(target) - np.log(np.maximum(share, 1e-4)))).astype(np.float32)
        b -= b.mean(dtype=np.float32)
    else:
        raise RuntimeError(f"no convergence for {name}: max share error {err:.4f}")
    return {"router_b": [float(v) for v in b], "zipf_s": s, "n_tokens": n_tokens,
            "iterations": it, "realised_shares": [float(v) for v in share],
            "target_shares": [float(v) for v in target]}


if __name__ == "__main__":
    table = {name: calibrate(name) for name in ("phone",)}
    with open(OUT, "w") as f:
        json.dump(table, f, indent=1)
    print(json.dumps(table, indent=1))
