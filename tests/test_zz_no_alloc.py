"""The allocation-free entry point (moe_forward_static: the library's own scratch array in place
of a caller workspace) against moe_forward, through the C ABI: two calls in a row on one GPU, the
second on a smaller input, which finds the first call's leftovers in the scratch."""
import numpy as np
import pytest
import torch

import paper_2503_00245_amd as pkg
import workloads as wl
from tests.helpers import rel_err, to_device, to_f64, weights_to_device

pytestmark = pytest.mark.gpu


def _both(dev, w_t, x_np, k, residual):
    x_t = to_device(x_np, dev)
    T = x_t.shape[0]
    shape = pkg.shape_for(w_t, T, k, pkg.MOE_BF16, residual=residual)
    assert pkg.moe_workspace_bytes(shape) <= pkg.STATIC_WORKSPACE_BYTES
    out = []
    for static in (False, True):
        y = torch.full_like(x_t, float("nan"))
        idx = torch.full((T, k), -1, dtype=torch.int32, device=dev)
        gate = torch.full((T, k), -1.0, dtype=torch.float32, device=dev)
        if static:
            pkg.moe_forward_static(shape, pkg.make_weights(w_t), x_t, y, idx, gate)
        else:
            pkg.moe_forward(shape, pkg.make_weights(w_t), x_t, y, idx, gate, pkg.alloc_workspace(shape, dev))
        torch.cuda.synchronize()
        out.append((y, idx, gate))
    return out


@pytest.mark.parametrize("kind", ["dense", "shared_base"])
def test_static_entry_point_matches_moe_forward_on_two_calls_in_a_row(oracle, kind):
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    if kind == "dense":
        cfg = wl.shrink(wl.CONFIGS["wearables"], d_model=512, d_ff=1024)
    else:
        cfg = wl.LayerConfig("sb", 256, 448, 6, 3, "bf16", 7321, rank=64, shared_base=True,
                             weight_std=0.05, wd_product_std=0.0125)
    w_np = wl.make_layer_weights(cfg, with_bias=False)
    w_t = weights_to_device(w_np, dev)
    # 300 tokens (grouped GEMM path, several tiles), then 37, then a single token (decode path)
    for T, residual in ((300, False), (37, True), (1, False)):
        x_np = wl.make_inputs(cfg, T, step=T)
        (y0, i0, g0), (y1, i1, g1) = _both(dev, w_t, x_np, cfg.top_k, residual)
        assert torch.equal(i0, i1) and torch.equal(g0, g1)  # integer work bit-exact
        assert torch.equal(y0, y1)                           # same kernels, same bits
        ref, ridx, _ = oracle.forward(w_np, x_np, cfg.top_k, residual=residual)
        same = np.all(i1.cpu().numpy() == ridx, axis=1)
        assert same.mean() > 0.97
        assert rel_err(to_f64(y1)[same], ref[same]) < 2e-2


def test_static_entry_point_refuses_large_shapes_and_leaves_outputs_alone():
    dev = torch.device("cuda:0")
    cfg = wl.shrink(wl.CONFIGS["wearables"], d_model=512, d_ff=1024)
    w_t = weights_to_device(wl.make_layer_weights(cfg, with_bias=False), dev)
    T = 8192
    shape = pkg.shape_for(w_t, T, cfg.top_k, pkg.MOE_BF16)
    assert pkg.moe_workspace_bytes(shape) > pkg.STATIC_WORKSPACE_BYTES
    x = torch.zeros((T, cfg.d_model), dtype=torch.bfloat16, device=dev)
    y = torch.full_like(x, 3.0)
    with pytest.raises(pkg.MoeError) as e:
        pkg.moe_forward_static(shape, pkg.make_weights(w_t), x, y)
    assert e.value.status == -3
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())
