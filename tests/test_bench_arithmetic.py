"""bench.py's roofline arithmetic and argument handling (CPU only).

The algorithmic work it divides by is pinned to figures worked out by hand from the layer
definition (Sec. 2.1: k of E SwiGLU experts per token; Sec. 2.2: every product of a
weight-decomposed expert goes through a rank-r intermediate)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
import workloads as wl  # noqa: E402


def test_phone_prefill_flops_and_dominant_kernel():
    cfg = wl.CONFIGS["phone"]
    flops, wbytes = bench.layer_algorithmic(cfg, 2048)
    # 6 P d F with P = 4096 pairs
    assert flops == 6.0 * 4096 * 2048 * 5632 == pytest.approx(283.5e9, rel=1e-3)
    assert wbytes == 8 * 3 * 2048 * 5632 * 2 == pytest.approx(553.6e6, rel=1e-3)
    name, bound, work, unit = bench.dominant_kernel_work(cfg, 2048)
    assert (name, bound, unit) == ("gemm_gate_up_swiglu", "mfma", "TFLOP/s")
    assert work == pytest.approx(189.0e9, rel=1e-3)  # 4 P d F


def test_phone_decode_streams_only_the_selected_experts():
    cfg = wl.CONFIGS["phone"]
    flops, wbytes = bench.layer_algorithmic(cfg, 1)
    assert wbytes == 2 * 3 * 2048 * 5632 * 2 == pytest.approx(138.41e6, rel=1e-4)
    name, bound, work, unit = bench.dominant_kernel_work(cfg, 1)
    assert (name, bound, unit) == ("gemv_gate_up_swiglu", "hbm", "GB/s")
    assert work == pytest.approx(92.27e6, rel=1e-4)  # gate and up matrices of two experts


def test_weight_decomposed_work_counts_the_factors_not_the_products():
    cfg = wl.CONFIGS["phone_wd"]
    flops, wbytes = bench.layer_algorithmic(cfg, 2048)
    assert flops == pytest.approx(193.3e9, rel=1e-3)        # 6 P r (d + F)
    _, wdec = bench.layer_algorithmic(cfg, 1)
    assert wdec == pytest.approx(94.37e6, rel=1e-4)         # 2 experts x 3 r (d + F) bf16


def test_shared_base_is_counted_once_per_token():
    cfg = wl.CONFIGS["phone_wd_base"]
    flops, _ = bench.layer_algorithmic(cfg, 2048)
    assert flops == pytest.approx(153.8e9, rel=1e-3)        # 6 T d F + 6 P 64 (d + F)
    _, wdec = bench.layer_algorithmic(cfg, 1)
    assert wdec == pytest.approx(75.10e6, rel=1e-3)         # base + two rank-64 factor sets
    name, bound, work, _ = bench.dominant_kernel_work(cfg, 2048)
    assert name == "gemm_base_gate_up" and work == 4.0 * 2048 * 5632 * 2048


def test_layer_weight_bytes_match_the_configurations():
    assert bench.layer_weight_bytes(wl.CONFIGS["wearables"]) == pytest.approx(138.4e6, rel=1e-3)
    assert 24 * bench.layer_weight_bytes(wl.CONFIGS["phone_stack"]) == pytest.approx(13.29e9, rel=1e-3)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_every_workload_names_a_known_configuration():
    for name, (cfg_name, tokens) in bench.WORKLOADS.items():
        assert cfg_name in wl.CONFIGS and tokens >= 1, name


def _profile_means(fname, kernel_regex):
    """(FETCH_SIZE mean, WRITE_SIZE mean) in KiB of the kernel's line in a committed profile summary."""
    import re
    section, found = None, {}
    for ln in open(os.path.join(ROOT, "profiles", fname)):
        if ln.startswith("== "):
            section = "FETCH" if "FETCH_SIZE" in ln else "WRITE" if "WRITE_SIZE" in ln else None
        elif section and re.search(kernel_regex, ln):
            found[section] = float(re.search(r"mean\s+([\d.]+)", ln).group(1))
    return found["FETCH"], found["WRITE"]


def test_traffic_constants_are_the_committed_profiles_figures():
    # roofline.traffic must not go stale when a kernel changes: the constants in bench.py are the
    # counter means of the committed rocprofv3 summaries, scaled by the calibration copy's factors
    assert set(bench.TRAFFIC_SOURCE) == set(bench.MEASURED_KIB)
    for workload, (fname, regex) in bench.TRAFFIC_SOURCE.items():
        fetch, write = _profile_means(fname, regex)
        assert bench.MEASURED_KIB[workload] == (fetch, write), workload
        assert bench.MEASURED_TRAFFIC_BYTES[workload] == int((fetch * 2.0 + write * 1.0) * 1024)
    # and the calibration itself: the 256 MiB copy reads half its size on FETCH_SIZE, all of it on WRITE_SIZE
    text = open(os.path.join(ROOT, "profiles", "phone_prefill_kernels_and_hbm_traffic.txt")).read()
    import re
    copies = re.findall(r"__amd_rocclr_copyBuffer.*max\s+([\d.]+)", text)
    assert any(abs(float(c) - 131089) < 50 for c in copies) and any(float(c) == 262144.0 for c in copies)
