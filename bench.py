#!/usr/bin/env python3
"""Benchmark of the MoE feed-forward layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole layer (route -> dispatch -> expert FFN -> combine, the
moe_forward entry point) over one batch of seeded synthetic tokens that is already
resident in HBM.  W untimed steps, then exactly K timed steps bracketed by device
synchronisation; one JSON line is printed.

  value      tokens/s of the whole layer over the K timed steps
  roofline   for the dominant kernel of the workload: algorithmic flops (prefill, MFMA
             bound) or bytes (decode, HBM bound) per launch divided by that kernel's
             average duration, measured with HIP events on the launch stream in a
             second pass of K steps through moe_forward_timed (same kernels, same
             inputs; the events are kept out of the tokens/s pass)
  stages     average milliseconds of every stage kernel from that second pass
  latency_ms median / p10 / p90 of single steps (one event pair per step, own pass)
  graph_replay_ms_per_step  the same steps captured once into a HIP graph and replayed
  preheat    untimed steps of the same workload run before the warm-up until the board has left its
             idle power state (at least 0.3 s, until two power readings 50 ms apart agree within 3 %,
             at most 2 s); without it the first milliseconds after idle run at a ramping clock
  gpu_state  shader clock and board power from sysfs before the pre-heat, at its end (load on),
             while an untimed repeat of the timed steps is executing, and after it
  configs    (default run only) the other benchmark configurations, measured briefly in the same
             process: ms per step, dominant-kernel and whole-layer roofline fractions
  decode     (default workload only) the same layer at one token per step: ms per step, tokens/s
             and the HBM roofline of its dominant kernel -- the metric's third part
  cpu_baseline  the CPU oracle, as it stands, timed on this host on a bounded sample

Workloads (shapes of the benchmark configurations):
  phone_prefill (default)  d 2048, F 5632, E 8, k 2, bf16, T = 2048, Zipf(1.1) expert loads
  phone_decode             same layer, T = 1, fresh token per step, cold weights
  wearables_prefill        d 1024, F 2816, T = 512      wearables_decode   T = 1
  phone_wd_prefill / phone_wd_decode            pure L.R experts, r = 1024
  phone_wd_base_prefill / phone_wd_base_decode  shared base + rank-64 pair
  phone_stack_decode       24 phone-shaped layers with residual adds, T = 1, one step =
                           one token through all 24 layers (--steps 256 = the full loop)
Decode workloads rotate over several device copies of the layer so that consecutive
steps never find their weights in the 256 MB last-level cache.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published

WORKLOADS = {
    "phone_prefill": ("phone", 2048),
    "phone_decode": ("phone", 1),
    "wearables_prefill": ("wearables", 512),
    "wearables_decode": ("wearables", 1),
    "phone_wd_prefill": ("phone_wd", 2048),
    "phone_wd_decode": ("phone_wd", 1),
    "phone_wd_base_prefill": ("phone_wd_base", 2048),
    "phone_wd_base_decode": ("phone_wd_base", 1),
    "phone_stack_decode": ("phone_stack", 1),
    "paper_phone_prefill": ("paper_phone", 2048),
    "paper_phone_decode": ("paper_phone", 1),
    "paper_wearables_prefill": ("paper_wearables", 2048),
    "paper_wearables_decode": ("paper_wearables", 1),
    "paper_phone_wd_prefill": ("paper_phone_wd", 2048),
    "paper_phone_wd_decode": ("paper_phone_wd", 1),
    "paper_wearables_wd_prefill": ("paper_wearables_wd", 2048),
    "paper_wearables_wd_decode": ("paper_wearables_wd", 1),
}

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of
# this script (summaries under profiles/), each scaled by what the same counter reads for the 256 MiB
# device copy of --pmc-calibration (FETCH_SIZE x2.0, WRITE_SIZE x1.0).  TRAFFIC_SOURCE names, per workload,
# the summary and the kernel line the figures are read from (a CPU test keeps the two in step).
FETCH_SCALE, WRITE_SCALE = 2.0, 1.0
TRAFFIC_SOURCE = {
    # gate/up grouped GEMM with the SiLU * mul epilogue (256 x 256 tiles, 64-wide k-steps filled in halves)
    "phone_prefill": ("phone_prefill_kernels_and_hbm_traffic.txt",
                      r"gemm_bf16_deep_kernel<256, 256, 64, 64, 128, true, false"),
    # gate/up matrix-vector products + SwiGLU of the single-token step
    "phone_decode": ("phone_decode_kernels_and_hbm_traffic.txt", r"gemv_kernelIDF16bLi2E"),
}
MEASURED_KIB = {  # workload: (FETCH_SIZE mean, WRITE_SIZE mean), KiB per dispatch as the tool reports them
    "phone_prefill": (289396.7, 46923.4),
    "phone_decode": (45126.1, 44.0),
}
MEASURED_TRAFFIC_BYTES = {w: int((f * FETCH_SCALE + wr * WRITE_SCALE) * 1024) for w, (f, wr) in MEASURED_KIB.items()}


def layer_weight_bytes(cfg):
    d, F, E, r = cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.rank
    dense = 3 * d * F * 2
    fac = 3 * r * (d + F) * 2
    if r == 0:
        return E * dense
    return E * fac + (dense if cfg.shared_base else 0)


def dominant_kernel_work(cfg, T):
    """(stage name, bound, algorithmic work per launch, unit) of the dominant kernel."""
    d, F, k, r = cfg.d_model, cfg.d_ff, cfg.top_k, cfg.rank
    P = T * k
    if T == 1:
        # single token: the gate/up product streams k experts' gate and up matrices once
        if r == 0:
            nbytes = k * 2 * F * d * 2
        else:
            nbytes = k * 2 * F * r * 2 + (2 * F * d * 2 if cfg.shared_base else 0)
        return "gemv_gate_up_swiglu", "hbm", float(nbytes), "GB/s"
    if cfg.shared_base and k > 1:
        # the shared base meets every token once (not once per pair): its gate and up products
        # are one plain launch over T rows, the longest kernel of this workload
        return "gemm_base_gate_up", "mfma", 4.0 * T * F * d, "TFLOP/s"
    if cfg.shared_base:
        return "gemm_gate_up_swiglu", "mfma", 4.0 * P * F * (r + d), "TFLOP/s"
    return "gemm_gate_up_swiglu", "mfma", 4.0 * P * F * (r if r else d), "TFLOP/s"


def layer_algorithmic(cfg, T):
    """Whole-layer algorithmic (flops, expert-weight bytes streamed) per forward."""
    d, F, k, r, E = cfg.d_model, cfg.d_ff, cfg.top_k, cfg.rank, cfg.n_experts
    P = T * k
    if r == 0:
        flops = 6.0 * P * d * F
        per_expert = 3 * d * F * 2
        nbytes = min(P, E) * per_expert if T == 1 else E * per_expert
    else:
        # a shared base is applied once per token: gate/up on x_t, down on the gate-mixed hidden vector
        flops = 6.0 * P * r * (d + F) + (6.0 * T * d * F if cfg.shared_base else 0)
        per_expert = 3 * r * (d + F) * 2
        nbytes = (min(P, E) if T == 1 else E) * per_expert + (3 * d * F * 2 if cfg.shared_base else 0)
    return flops, float(nbytes)


def gpu_state():
    """Clock and power of the first GPU from sysfs (plain file reads; no child process)."""
    import glob
    out = {}
    for dev in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        try:
            with open(os.path.join(dev, "pp_dpm_sclk")) as f:
                cur = [ln.split(":")[1].strip() for ln in f if "*" in ln]
            out["sclk"] = cur[0].replace("*", "").strip() if cur else None
        except OSError:
            continue
        for name, key, scale in (("power1_average", "power_w", 1e-6), ("power1_input", "power_w", 1e-6),
                                 ("power1_cap", "power_cap_w", 1e-6)):
            for path in glob.glob(os.path.join(dev, "hwmon/hwmon*/" + name)):
                try:
                    with open(path) as f:
                        out.setdefault(key, round(int(f.read().strip()) * scale, 1))
                except (OSError, ValueError):
                    pass
        break
    return out or None


def preheat(step, sync, min_s=0.3, max_s=2.0):
    """Run untimed steps until the board power has stopped climbing; returns (seconds, steps, the
    last clock / power sample, read while the load was on)."""
    t0 = time.perf_counter()
    n = 0
    last = None
    while True:
        t1 = time.perf_counter()
        while time.perf_counter() - t1 < 0.05:
            for _ in range(4):
                step(n)
                n += 1
            sync()
        el = time.perf_counter() - t0
        st = gpu_state() or {}
        pw = st.get("power_w")
        if el >= max_s:
            break
        if el >= min_s and (pw is None or (last is not None and abs(pw - last) <= 0.03 * max(pw, 1.0))):
            break
        last = pw
    return time.perf_counter() - t0, n, st or None


def percentile(sorted_vals, q):
    return sorted_vals[min(len(sorted_vals) - 1, int(q * len(sorted_vals)))]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="phone_prefill", choices=sorted(WORKLOADS))
    ap.add_argument("--top-k", type=int, default=None, help="override k (active experts)")
    ap.add_argument("--experts", type=int, default=None, help="override E (total experts)")
    ap.add_argument("--tokens", type=int, default=None, help="override the workload's tokens per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode-leg", action="store_true",
                    help="default workload only: skip the single-token decode measurement appended as 'decode'")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="default workload only: skip the brief measurements of the other configurations ('configs')")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three 256 MiB device copies (a known-size kernel that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="target wall time of the CPU oracle sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported. Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2503_00245_amd as pkg
    import workloads as wl

    from paper_2503_00245_amd import build as hip_build
    hip_build.ensure_built()  # compiles only when no library is there
    pkg.lib()  # fails loudly if the HIP library is still missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    weight_cache = {}

    def run_workload(workload, tokens, steps_arg, warmup_arg, want_cpu, brief=False):
        cfg_name, T = WORKLOADS[workload]
        if tokens is not None:
            T = tokens
        cfg = wl.CONFIGS[cfg_name]
        if args.top_k is not None or args.experts is not None:
            # the paper's ablation grid (active experts k, total experts E); no stored Zipf bias then
            cfg = wl.shrink(cfg, top_k=args.top_k or cfg.top_k, n_experts=args.experts or cfg.n_experts,
                            zipf=False)
        decode = T == 1
        stack = cfg.n_layers > 1
        steps = steps_arg if steps_arg is not None else (256 if stack else (2000 if decode else 200))
        warmup = warmup_arg if warmup_arg is not None else (8 if stack else (50 if decode else 10))

        def dev_t(a):
            if a is None:
                return None
            if a.dtype == np.uint16:
                return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to(dev)
            return torch.from_numpy(a).to(dev)

        # ---- inputs: generated on the host from the seed, then resident in HBM ---------------
        t_gen = time.time()
        if stack:
            layers_np = wl.make_stack_weights(cfg, workers=8)
        else:
            if cfg.name not in weight_cache:
                weight_cache.clear()  # one layer's host copy at a time
                weight_cache[cfg.name] = wl.make_layer_weights(cfg)
            layers_np = [weight_cache[cfg.name]]
        layers_t = [{k: dev_t(v) for k, v in w.items()} for w in layers_np]
        n_inputs = 256 if decode else 4
        xs_np = [wl.make_inputs(cfg, T, step=i) for i in range(n_inputs)]
        xs = [dev_t(x) for x in xs_np]
        # cold-cache rotation for single-layer decode: enough copies to exceed the LLC several times
        copies = [layers_t]
        if decode and not stack:
            n_copies = max(2, int(np.ceil(1.5e9 / layer_weight_bytes(cfg))))
            for _ in range(n_copies - 1):
                copies.append([{k: (None if v is None else v.clone()) for k, v in layers_t[0].items()}])
        gen_s = time.time() - t_gen

        shape = pkg.shape_for(layers_t[0], T, cfg.top_k, pkg.MOE_BF16)
        ws = pkg.alloc_workspace(shape, dev)
        y = torch.empty_like(xs[0])
        w_structs = [[pkg.make_weights(w) for w in c] for c in copies]

        def step(i):
            ws_i = w_structs[i % len(w_structs)]
            if stack:
                pkg.moe_stack_forward(shape, ws_i, xs[i % n_inputs], y, None, ws)
            else:
                pkg.moe_forward(shape, ws_i[0], xs[i % n_inputs], y, None, None, ws)

        if args.pmc_calibration:
            src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst

        state_idle = gpu_state()
        # (no host work between the pre-heat and the warm-up: reading the power sensor takes
        # milliseconds, long enough for the board to start leaving its loaded state)
        preheat_s, preheat_steps, state_before = preheat(step, torch.cuda.synchronize)
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(warmup + i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ms_per_step = elapsed / steps * 1e3
        tokens_per_s = T * steps / elapsed
        # the same steps once more, untimed, with the clock and power read while they execute (the
        # read itself takes longer than a short timed region, so it stays out of it)
        state_during = None
        if not brief:
            for i in range(max(steps, 50)):
                step(warmup + i)
            state_during = gpu_state()
            torch.cuda.synchronize()
        state_after = gpu_state()

        # ---- per-step latency spread: one event pair around every step --------------------------
        n_lat = min(steps, 200)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_lat)]
        for i, (e0, e1) in enumerate(evs):
            e0.record()
            step(warmup + i)
            e1.record()
        torch.cuda.synchronize()
        lat = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        latency = {"n": n_lat, "median": round(percentile(lat, 0.5), 5), "p10": round(percentile(lat, 0.1), 5),
                   "p90": round(percentile(lat, 0.9), 5)}

        # ---- the same steps replayed from a HIP graph: launch gaps between kernels drop out ------
        graph_ms = None
        if not stack and not brief:
            n_in_graph = 4 * len(w_structs) if decode else 16
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for i in range(n_in_graph):
                    step(i)
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    for i in range(n_in_graph):
                        step(i)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            n_rep = max(5, min(steps, 200) // n_in_graph)
            for _ in range(2):
                graph.replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(n_rep):
                graph.replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - t1) / (n_rep * n_in_graph) * 1e3

        # ---- second pass: per-stage durations from HIP events on the launch stream ------------
        stage_sum = {}
        order = []
        n_timed = min(steps, 200) if not stack else min(steps, 8)
        single = pkg.shape_for(layers_t[0], T, cfg.top_k, pkg.MOE_BF16, residual=stack)
        for i in range(n_timed):
            ws_i = w_structs[i % len(w_structs)]
            for l, wst in enumerate(ws_i):
                for name, ms in pkg.moe_forward_timed(single, wst, xs[(i + l) % n_inputs], y, ws):
                    if name not in stage_sum:
                        stage_sum[name] = 0.0
                        order.append(name)
                    stage_sum[name] += ms
        n_launch = n_timed * len(w_structs[0])
        stages = {n: stage_sum[n] / n_launch for n in order}

        kname, bound, work, unit = dominant_kernel_work(cfg, T)
        if kname not in stages and "gemv_gate_up_swiglu" in stages:
            # a few tokens on the matrix-vector path: bound by streaming the experts they selected (at
            # most T k of them, each once) -- report against the upper bound of those bytes
            n_sel = min(T * cfg.top_k, cfg.n_experts)
            per = 2 * cfg.d_ff * (cfg.rank if cfg.rank else cfg.d_model) * 2
            kname, bound, work, unit = "gemv_gate_up_swiglu", "hbm", float(n_sel * per), "GB/s"
        if kname not in stages:  # a shape the per-token base path does not take: base work per pair
            kname, work = "gemm_gate_up_swiglu", 4.0 * T * cfg.top_k * cfg.d_ff * (cfg.rank + cfg.d_model)
        kms = stages[kname]
        if bound == "hbm":
            achieved = work / (kms * 1e-3) / 1e9
            peak = HBM_PEAK_GBS
        else:
            achieved = work / (kms * 1e-3) / 1e12
            peak = MFMA_BF16_PEAK_TFLOPS
        flops, wbytes = layer_algorithmic(cfg, T)
        n_l = cfg.n_layers
        layer = {"mfma_frac_of_peak": round(flops * n_l / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                 "hbm_frac_of_peak": round(wbytes * n_l / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                 "algorithmic_flops": flops * n_l, "algorithmic_weight_bytes": wbytes * n_l,
                 "sum_of_stage_ms": round(sum(stages.values()), 5)}
        # frac: the dominant kernel alone (its own launches); layer_frac: the whole step against the
        # same peak, every kernel and every gap between them included
        roofline = {"bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
                    "frac": round(achieved / peak, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(workload) if tokens is None else None,
                    "kernel": kname, "kernel_ms": round(kms, 5), "algorithmic_per_launch": work,
                    "layer_frac": layer["hbm_frac_of_peak"] if bound == "hbm" else layer["mfma_frac_of_peak"]}
        if brief:
            return {"tokens_per_step": T, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
                    "tokens_per_s": round(tokens_per_s, 2), "roofline": roofline,
                    "layer_mfma_frac_of_peak": layer["mfma_frac_of_peak"],
                    "layer_hbm_frac_of_peak": layer["hbm_frac_of_peak"],
                    "stages_ms": {k: round(v, 5) for k, v in stages.items()},
                    "latency_ms": latency, "preheat_s": round(preheat_s, 3),
                    "weight_copies_rotated": len(copies)}

        # ---- what the router does with the timed inputs: share of the (token, slot) pairs per expert
        # (first layer; for single-token steps over all the rotated input tokens) --------------------
        xcat = torch.cat(xs[:min(n_inputs, max(1, 4096 // T))], dim=0)
        n_routed = xcat.shape[0]
        rshape = pkg.shape_for(layers_t[0], n_routed, cfg.top_k, pkg.MOE_BF16)
        ridx = torch.empty((n_routed, cfg.top_k), dtype=torch.int32, device=dev)
        rgate = torch.empty((n_routed, cfg.top_k), dtype=torch.float32, device=dev)
        rprobs = torch.empty((n_routed, cfg.n_experts), dtype=torch.float32, device=dev)
        pkg.moe_route(rshape, xcat, layers_t[0]["router_w"], layers_t[0].get("router_b"), ridx, rgate, rprobs)
        torch.cuda.synchronize()
        counts = np.bincount(ridx.cpu().numpy().ravel(), minlength=cfg.n_experts)
        routing = {"tokens": int(n_routed), "expert_share": [round(float(c) / counts.sum(), 4) for c in counts]}
        du_c = torch.zeros((1, cfg.n_experts), dtype=torch.int64, device=dev)
        du_m = torch.zeros(1, dtype=torch.float64, device=dev)
        pkg.moe_delta_uniform(ridx.view(1, n_routed, cfg.top_k), cfg.n_experts, du_c, None, du_m)
        torch.cuda.synchronize()
        routing["delta_uniform_percent"] = round(100.0 * float(du_m.item()), 3)
        if n_routed > 1:
            # the same tokens read as one sequence: Eq. 4-7's replacement count and loss value
            bles = torch.zeros(5, dtype=torch.float64, device=dev)
            bws = torch.empty(max(1, pkg.moe_bles_workspace_bytes(1, n_routed, cfg.n_experts)),
                              dtype=torch.uint8, device=dev)
            pkg.moe_bles_loss(rprobs.view(1, n_routed, cfg.n_experts), ridx.view(1, n_routed, cfg.top_k), bles, bws)
            torch.cuda.synchronize()
            b = bles.cpu().numpy()
            routing["as_one_sequence"] = {"H": int(b[0]), "H_norm": round(float(b[1]), 5),
                                          "L_norm": round(float(b[3]), 5), "bles_loss": round(float(b[4]), 6)}
            del bles, bws
        del xcat, ridx, rgate, rprobs

        # ---- the paper's offloading cost model (Sec. 3.4.2) restated on this routing: run the stack
        # token by token, keep every layer's selection, count on the GPU how often a layer's
        # expert set changes and how many experts the rule would bring in ------------------------
        offload = None
        if stack:
            n_tr = min(steps, 256)
            trace_tl = torch.empty((n_tr, cfg.n_layers, cfg.top_k), dtype=torch.int32, device=dev)
            for i in range(n_tr):
                pkg.moe_stack_forward(shape, w_structs[0], xs[i % n_inputs], y, trace_tl[i], ws)
            trace = trace_tl.permute(1, 0, 2).contiguous()  # [layer, token, slot]
            changes = torch.zeros(cfg.n_layers, dtype=torch.int64, device=dev)
            loads = torch.zeros(cfg.n_layers, dtype=torch.int64, device=dev)
            h_e = torch.zeros(cfg.n_experts, dtype=torch.int64, device=dev)
            h_all = torch.zeros(1, dtype=torch.int64, device=dev)
            pkg.moe_offload_counters(trace, cfg.n_experts, changes, loads)
            pkg.moe_expert_replacements(trace, cfg.n_experts, h_e, h_all)
            torch.cuda.synchronize()
            expert_bytes = 3 * cfg.d_model * cfg.d_ff * 2
            n_loads = int(loads.sum().item())
            offload = {"tokens": n_tr, "layers": cfg.n_layers,
                       "set_changes_per_token_and_layer": round(int(changes.sum().item()) / (n_tr * cfg.n_layers), 4),
                       "experts_loaded_per_token": round(n_loads / n_tr, 3),
                       "bytes_loaded_per_token": int(n_loads / n_tr * expert_bytes),
                       "set_changes_first_and_last_layer": [round(int(changes[0].item()) / n_tr, 4),
                                                            round(int(changes[-1].item()) / n_tr, 4)],
                       "expert_replacements_half_H": int(h_all.item()) // 2,
                       "note": "independent random tokens, so consecutive tokens share experts only by chance"}
            # Delta Uniform (Sec. 3.2 / Table 3) of the same trace: per-layer L1 distance of the
            # realised expert shares from 1/E, averaged over the layers
            du_counts = torch.zeros((cfg.n_layers, cfg.n_experts), dtype=torch.int64, device=dev)
            du_layer = torch.zeros(cfg.n_layers, dtype=torch.float64, device=dev)
            du_mean = torch.zeros(1, dtype=torch.float64, device=dev)
            pkg.moe_delta_uniform(trace, cfg.n_experts, du_counts, du_layer, du_mean)
            torch.cuda.synchronize()
            offload["delta_uniform_percent"] = round(100.0 * float(du_mean.item()), 3)
            offload["delta_uniform_percent_first_and_last_layer"] = [
                round(100.0 * float(du_layer[0].item()), 3), round(100.0 * float(du_layer[-1].item()), 3)]
            del trace_tl, trace

        # ---- CPU oracle baseline on a bounded sample of the same workload -------------------------
        cpu = None
        if want_cpu:
            from oracle import build as oracle_builder, moe_oracle
            # the timing leg runs the oracle's source as it stands, compiled for this host's cores
            # (the checker used by the tests stays the generic -O2 build)
            try:
                moe_oracle.use_library(oracle_builder.build_native())
                oracle_build = "-O3 -march=native -fopenmp"
            except Exception:  # no compiler on this host: time the checker's own build
                oracle_build = "-O2 -fopenmp (generic x86-64)"
            k = cfg.top_k

            def run_oracle(n_tok):
                t1 = time.perf_counter()
                if stack:
                    for i in range(n_tok):
                        moe_oracle.stack_forward(layers_np, xs_np[i % n_inputs], k)
                elif decode:
                    for i in range(n_tok):
                        moe_oracle.forward(layers_np[0], xs_np[i % n_inputs], k)
                else:
                    moe_oracle.forward(layers_np[0], np.ascontiguousarray(xs_np[0][:n_tok]), k)
                return time.perf_counter() - t1

            probe_n = 1 if (decode or stack) else min(T, 2 * moe_oracle.num_threads())
            probe = run_oracle(probe_n)
            # three passes over the same sample, each about a third of the time allowed; the median counts
            n_sample = int(max(probe_n, min(T if not decode else 4096,
                                            probe_n * (args.cpu_seconds / 3.0) / max(probe, 1e-6))))
            if stack:
                n_sample = max(1, min(n_sample, 32))
            if not (decode or stack):
                n_sample = max(probe_n, n_sample // probe_n * probe_n)
            times = sorted(run_oracle(n_sample) for _ in range(3))
            took = times[1]
            cpu = {"value": round(n_sample / took, 3), "unit": "tokens/s",
                   "cores": moe_oracle.num_threads(), "kind": "oracle",
                   "sample": f"{n_sample} token(s) of the {workload} workload through the fp64 C oracle, "
                             f"median of 3 passes ({times[0]:.2f} / {times[1]:.2f} / {times[2]:.2f} s), "
                             f"oracle source built {oracle_build}"}

        out = {
            "metric": "moe_layer_tokens_per_s", "value": round(tokens_per_s, 2), "unit": "tokens/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
            "data": "synthetic",
            "config": {"workload": workload, "d_model": cfg.d_model, "d_ff": cfg.d_ff,
                       "n_experts": cfg.n_experts, "top_k": cfg.top_k, "rank": cfg.rank,
                       "shared_base": cfg.shared_base, "n_layers": cfg.n_layers, "tokens_per_step": T,
                       "zipf_router_bias": bool(cfg.zipf), "weight_copies_rotated": len(copies)},
            "roofline": roofline, "cpu_baseline": cpu, "stages_ms": {k: round(v, 5) for k, v in stages.items()},
            "layer": layer, "routing": routing, "offload_model": offload,
            "latency_ms": latency, "graph_replay_ms_per_step": None if graph_ms is None else round(graph_ms, 5),
            "preheat": {"seconds": round(preheat_s, 3), "steps": preheat_steps,
                        "note": "untimed steps of the same workload before the warm-up, until board power settles"},
            "gpu_state": {"idle": state_idle, "before": state_before, "during": state_during, "after": state_after},
            "input_generation_s": round(gen_s, 1),
        }
        return out

    out = run_workload(args.workload, args.tokens, args.steps, args.warmup, not args.no_cpu_baseline)
    plain = args.tokens is None and args.top_k is None and args.experts is None
    if args.workload == "phone_prefill" and plain and not args.no_decode_leg:
        # the metric has three parts: tokens/s and MFMA use at prefill (above), HBM use at
        # single-token decode (here, same layer, same process)
        d = run_workload("phone_decode", None, None, None, False)
        out["decode"] = {k: d[k] for k in ("ms_per_step", "value", "unit", "steps", "warmup", "roofline",
                                           "stages_ms", "latency_ms", "graph_replay_ms_per_step", "routing")}
        out["decode"]["workload"] = "phone_decode"
        out["decode"]["layer_hbm_frac_of_peak"] = d["layer"]["hbm_frac_of_peak"]
        out["decode"]["weight_copies_rotated"] = d["config"]["weight_copies_rotated"]
        out["decode"]["preheat"] = d["preheat"]
        if not args.no_other_configs:
            # the other benchmark configurations, briefly, in the same process (each: pre-heat, warm-up,
            # timed steps, a per-stage event pass); steps chosen so that the whole run stays short
            others = {}
            for name, n_steps, n_warm in (("wearables_prefill", 100, 10), ("wearables_decode", 1000, 50),
                                          ("phone_wd_prefill", 40, 5), ("phone_wd_decode", 500, 20),
                                          ("phone_wd_base_prefill", 40, 5), ("phone_wd_base_decode", 500, 20),
                                          ("phone_stack_decode", 48, 4)):
                weight_cache.clear()
                torch.cuda.empty_cache()
                others[name] = run_workload(name, None, n_steps, n_warm, False, brief=True)
            out["configs"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
