"""The C-ABI library without a GPU: it loads, exports what include/moe.h declares, sizes
workspaces, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import pytest

import paper_2503_00245_amd as pkg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    return re.findall(r"MOE_API\s+[\w\s\*]+?\b(moe_\w+)\s*\(", text)


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert set(names) == set(pkg.EXPORTS) and len(names) == 15
    L = pkg.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert pkg.status_string(0) == "ok"
    assert len({pkg.status_string(s) for s in (0, -1, -2, -3, -4, -99)}) == 6


def test_workspace_bytes_by_shape():
    small = pkg.moe_workspace_bytes(pkg.make_shape(32, 128, 256, 4, 2, 0, pkg.MOE_F32))
    big = pkg.moe_workspace_bytes(pkg.make_shape(2048, 2048, 5632, 8, 2, 0, pkg.MOE_BF16))
    assert 0 < small < big
    # the phone prefill workspace must hold h [P,F] and y_perm [P,d] in bf16
    assert big >= 4096 * (5632 + 2048) * 2
    assert big % 256 == 0
    assert pkg.moe_workspace_bytes(pkg.make_shape(0, 128, 256, 4, 2)) > 0


@pytest.mark.parametrize("kw,status", [
    (dict(top_k=0), -1), (dict(top_k=5), -1), (dict(n_tokens=-1), -1), (dict(rank=-8), -1),
    (dict(flags=1), -1),                 # shared base without a rank
    (dict(flags=8), -1),                 # unknown flag
    (dict(n_experts=65, top_k=2), -2), (dict(d_model=100), -2), (dict(d_ff=100), -2),
    (dict(rank=12), -2), (dict(act_dtype=7), -2), (dict(n_tokens=1 << 23), -2),
])
def test_bad_shapes_are_rejected_on_the_host(kw, status):
    base = dict(n_tokens=8, d_model=128, d_ff=256, n_experts=4, top_k=2, rank=0,
                act_dtype=pkg.MOE_BF16, flags=0)
    base.update(kw)
    shape = pkg.make_shape(**base)
    assert pkg.moe_workspace_bytes(shape) == 0
    L = pkg.lib()
    dummy = C.c_void_p(4096)
    assert L.moe_route(C.byref(shape), dummy, dummy, None, dummy, dummy, None, None) == status
    assert L.moe_combine(C.byref(shape), dummy, dummy, dummy, None, dummy, None) == status
    w = pkg.MoeWeights()
    assert L.moe_forward(C.byref(shape), C.byref(w), dummy, dummy, None, None, dummy, 1 << 30,
                         None) == status


def test_null_misaligned_and_short_workspace_arguments():
    L = pkg.lib()
    shape = pkg.make_shape(8, 128, 256, 4, 2)
    ok, odd = C.c_void_p(4096), C.c_void_p(4100)
    assert L.moe_route(C.byref(shape), None, ok, None, ok, ok, None, None) == -1
    assert L.moe_route(C.byref(shape), odd, ok, None, ok, ok, None, None) == -1
    assert L.moe_route(None, ok, ok, None, ok, ok, None, None) == -1
    assert L.moe_combine(C.byref(shape), ok, ok, ok, odd, ok, None) == -1
    assert L.moe_permute(C.byref(shape), ok, None, ok, ok, None, None, ok, 1 << 20, None) == -1
    assert L.moe_permute(C.byref(shape), ok, ok, ok, ok, ok, None, ok, 1 << 20, None) == -1
    w = pkg.MoeWeights()
    assert L.moe_forward(C.byref(shape), C.byref(w), ok, ok, None, None, ok, 1 << 30, None) == -1
    for n in ("router_w", "w_gate", "w_up", "w_down"):
        setattr(w, n, 4096)
    need = pkg.moe_workspace_bytes(shape)
    y = C.c_void_p(8192)
    assert L.moe_forward(C.byref(shape), C.byref(w), ok, y, None, None, ok, need - 1, None) == -3
    assert L.moe_forward(C.byref(shape), C.byref(w), ok, y, None, None, None, need, None) == -3
    assert L.moe_forward(C.byref(shape), C.byref(w), ok, ok, None, None, ok, need, None) == -1  # y aliases x
    assert L.moe_expert_ffn(C.byref(shape), C.byref(w), ok, ok, ok, ok, 16, None) == -3
    w.rg = 4096  # factors without a rank are ignored, a dense block without the flag is not
    wd = pkg.make_shape(8, 128, 256, 4, 2, rank=16)
    assert L.moe_forward(C.byref(wd), C.byref(w), ok, C.c_void_p(8192), None, None, ok, 1 << 30, None) == -1
    assert L.moe_stack_forward(C.byref(shape), C.byref(w), 0, ok, C.c_void_p(8192), None, ok, 1 << 30, None) == -1


def test_zero_tokens_is_a_no_op_without_touching_pointers():
    L = pkg.lib()
    shape = pkg.make_shape(0, 128, 256, 4, 2)
    assert L.moe_route(C.byref(shape), None, None, None, None, None, None, None) == 0
    assert L.moe_combine(C.byref(shape), None, None, None, None, None, None) == 0
    w = pkg.MoeWeights()
    for n in ("router_w", "w_gate", "w_up", "w_down"):
        setattr(w, n, 4096)
    assert L.moe_forward(C.byref(shape), C.byref(w), None, None, None, None, None, 0, None) == 0
    assert L.moe_expert_ffn(C.byref(shape), C.byref(w), None, None, None, None, 0, None) == 0


def test_trace_metric_entry_points_reject_bad_shapes_on_the_host():
    L = pkg.lib()
    ok = C.c_void_p(4096)
    assert L.moe_expert_replacements(ok, 1, 8, 3, 2, ok, ok, None) == -1      # K > E
    assert L.moe_expert_replacements(ok, 1, 8, 2, 65, ok, ok, None) == -2     # E > 64
    assert L.moe_expert_replacements(None, 1, 8, 2, 8, ok, ok, None) == -1
    assert L.moe_offload_counters(ok, 0, 8, 2, 8, ok, ok, None) == -1
    assert L.moe_offload_counters(ok, 2, 8, 2, 8, None, ok, None) == -1
    assert pkg.moe_bles_workspace_bytes(4, 128, 8) >= 8 * 65 + 4 * (4 * 127 * 8 // 256)
    assert pkg.moe_bles_workspace_bytes(4, 128, 65) == 0
    assert L.moe_bles_loss(ok, ok, 4, 128, 2, 8, ok, ok, 16, None) == -3       # short workspace
    assert L.moe_bles_loss(ok, ok, 4, 128, 2, 8, None, ok, 1 << 20, None) == -1


def test_static_entry_point_refuses_what_its_scratch_cannot_hold():
    # checked on the host, before the scratch array is even looked up
    L = pkg.lib()
    w = pkg.MoeWeights()
    for n in ("router_w", "w_gate", "w_up", "w_down"):
        setattr(w, n, 4096)
    ok, y = C.c_void_p(4096), C.c_void_p(8192)
    big = pkg.make_shape(2048, 2048, 5632, 8, 2)
    assert pkg.moe_workspace_bytes(big) > pkg.STATIC_WORKSPACE_BYTES
    assert L.moe_forward_static(C.byref(big), C.byref(w), ok, y, None, None, None) == -3
    assert L.moe_forward_static(C.byref(big), C.byref(w), ok, ok, None, None, None) == -1  # y aliases x
    assert L.moe_forward_static(C.byref(pkg.make_shape(8, 100, 256, 4, 2)), C.byref(w), ok, y, None, None, None) == -2
    one = pkg.make_shape(1, 2048, 5632, 8, 2)
    assert 0 < pkg.moe_workspace_bytes(one) <= pkg.STATIC_WORKSPACE_BYTES
