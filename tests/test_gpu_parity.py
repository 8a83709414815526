"""GPU parity: every C-ABI entry point against the CPU oracle, element by element, on the
same seeded inputs.  Integer outputs (expert indices, offsets, permutations) must be
bit-exact; fp32 outputs within 1e-4 relative, bf16 outputs within 2e-2 relative
(per-tensor max-abs and L2 relative error, whichever is larger).

Routing on random inputs: the GPU sums logits in fp32, the oracle in fp64, so a token
whose k-th and (k+1)-th logits are closer than the fp32 rounding bound of the dot product
is "ambiguous"; indices must match exactly on every other token, and on ambiguous ones
the GPU's choice must still be admissible.  Tie-break tests use inputs whose fp32 dot
products are exact in any order, so equality there is genuinely bit-exact.
"""
import numpy as np
import pytest
import torch

import paper_2503_00245_amd as pkg
import workloads as wl
from tests.helpers import (ambiguous_tokens, bits_of, elementwise_rel_err, rel_err, row_rel_err,
                           stored_f64, to_device, to_f64, weights_to_device)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
# Worst element-wise relative error over the elements above a tenth of the tensor's rms.  bf16: the
# path rounds the hidden tensor, the grouped output rows and the result to bf16 (2^-9 relative
# each, independent), which leaves an absolute error of about 1.5e-3 rms per element, 5 sigma
# = 8e-3 rms over millions of elements, i.e. 0.08 relative at the magnitude floor; the bound
# leaves a factor 2.5.  fp32: fp32 accumulation over a few thousand terms, about 1e-6 rms.
ELEMENTWISE_TOL = {"f32": 1e-3, "bf16": 0.2}
DT = {"f32": pkg.MOE_F32, "bf16": pkg.MOE_BF16}


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    pkg.lib()  # fail loudly if the HIP library is not built
    return torch.device("cuda:0")


def _cfg(name="t", d=128, F=256, E=4, k=2, dtype="bf16", seed=1, r=0, base=False, std=0.02):
    return wl.LayerConfig(name, d, F, E, k, dtype, seed, rank=r, shared_base=base,
                          weight_std=std, wd_product_std=std if not base else std / 4)


def _check_routing(oracle, x_np, w_np, k, idx_gpu, gate_gpu, probs_gpu=None):
    """Bit-exact indices off the ambiguous set; gates/probs to fp32 accuracy. Returns mask of
    tokens whose routing equals the oracle's."""
    idx, gate, probs, logits = oracle.route(x_np, w_np["router_w"], w_np["router_b"], k)
    amb = ambiguous_tokens(logits, x_np, w_np["router_w"], k)
    same = np.all(idx_gpu == idx, axis=1)
    assert np.all(same[~amb]), f"routing differs on {int((~same & ~amb).sum())} unambiguous tokens"
    # an ambiguous token may pick differently, but only experts within the rounding band
    for t in np.flatnonzero(~same):
        kth = np.sort(logits[t])[::-1][k - 1]
        assert len(set(idx_gpu[t])) == k
        assert np.all(logits[t, idx_gpu[t]] >= kth - 1e-4), "inadmissible choice on ambiguous token"
    # k + 1 adjacent ranks can each be a near-tie, so the allowance grows with k
    assert amb.sum() <= max(2, x_np.shape[0] * k // 400), "too many ambiguous tokens for this recipe"
    assert np.allclose(gate_gpu[same], gate[same], rtol=2e-5, atol=1e-7)
    assert np.allclose(gate_gpu.sum(1), 1.0, atol=1e-6)
    if probs_gpu is not None:
        assert np.allclose(probs_gpu, probs, rtol=2e-5, atol=1e-8)
    return same, idx, gate


def _route_gpu(dev, x_t, w_t, E, k, act, want_probs=True):
    T, d = x_t.shape
    shape = pkg.make_shape(T, d, 8, E, k, 0, act)
    idx = torch.full((T, k), -7, dtype=torch.int32, device=dev)
    gate = torch.full((T, k), -7.0, dtype=torch.float32, device=dev)
    probs = torch.full((T, E), -7.0, dtype=torch.float32, device=dev) if want_probs else None
    pkg.moe_route(shape, x_t, w_t["router_w"], w_t["router_b"], idx, gate, probs)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), gate.cpu().numpy().astype(np.float64), \
        None if probs is None else probs.cpu().numpy().astype(np.float64)


# ------------------------------------------------------------------------------- moe_route

@pytest.mark.parametrize("T,d,E,k,dtype,bias", [
    (32, 128, 4, 2, "f32", False),      # tiny config
    (77, 1024, 8, 2, "bf16", False),    # wearables width, ragged token count
    (300, 2048, 8, 2, "bf16", True),    # phone width with a router bias
    (1, 2048, 8, 2, "bf16", True),      # single-token decode
    (65, 256, 64, 8, "bf16", True),     # one expert per lane
    (33, 264, 5, 1, "f32", False),      # k = 1, d not a multiple of the wave stride
    (40, 512, 6, 6, "bf16", False),     # k = E
    (19, 128, 64, 64, "bf16", True),    # the largest E and k the library takes
    (1500, 1024, 8, 2, "bf16", True),   # many tokens: eight per workgroup, ragged last tile
    (1028, 256, 64, 8, "f32", False),
    (2048, 2048, 8, 2, "bf16", True),   # phone prefill
    # 8192 tokens and more with at most 16 experts: the kernel that stages the router in LDS
    (8200, 2048, 8, 2, "bf16", True),   # phone width, three tokens per wave, ragged token count
    (8192, 264, 5, 1, "f32", False),    # d not a multiple of the wave stride
    (8192, 2048, 16, 4, "bf16", False), # the largest router that fits (128 KB)
    (20000, 512, 8, 8, "bf16", True),   # five tokens per wave, k = E
])
def test_route_matches_oracle(dev, oracle, T, d, E, k, dtype, bias):
    cfg = _cfg(d=d, E=E, k=k, dtype=dtype, seed=300 + T)
    w_np = wl.make_layer_weights(cfg, with_bias=False)
    if bias:
        w_np["router_b"] = wl.normal_tensor(cfg.seed, 99, (E,), 0.5, "f32")
    x_np = wl.make_inputs(cfg, T)
    w_t = weights_to_device({"router_w": w_np["router_w"], "router_b": w_np["router_b"]}, dev)
    idx, gate, probs = _route_gpu(dev, to_device(x_np, dev), w_t, E, k, DT[dtype])
    _check_routing(oracle, x_np, w_np, k, idx, gate, probs)
    if k == 1:
        assert np.all(gate == 1.0)


def test_route_large_batch_kernel_is_bit_identical_to_the_small_batch_one(dev):
    # the same tokens routed as one batch of 9000 (router staged in LDS, wave per token) and in
    # slices of 3000 (wave per expert): logits are summed in the same order, so every output
    # matches bit for bit
    cfg = _cfg(d=1024, E=8, k=2, dtype="bf16", seed=321)
    w_np = wl.make_layer_weights(cfg, with_bias=False)
    w_np["router_b"] = wl.normal_tensor(cfg.seed, 99, (8,), 0.5, "f32")
    x_np = wl.make_inputs(cfg, 9000)
    w_t = weights_to_device({"router_w": w_np["router_w"], "router_b": w_np["router_b"]}, dev)
    idx, gate, probs = _route_gpu(dev, to_device(x_np, dev), w_t, 8, 2, pkg.MOE_BF16)
    for lo in range(0, 9000, 3000):
        i2, g2, p2 = _route_gpu(dev, to_device(np.ascontiguousarray(x_np[lo:lo + 3000]), dev), w_t, 8, 2,
                                pkg.MOE_BF16)
        assert np.array_equal(idx[lo:lo + 3000], i2)
        assert np.array_equal(gate[lo:lo + 3000], g2) and np.array_equal(probs[lo:lo + 3000], p2)


@pytest.mark.parametrize("T", [512, 8704])
def test_route_tie_break_is_lowest_index_bit_exact(dev, oracle, T):
    # entries in {-1, -.5, 0, .5, 1} and a 0/1 router: every partial sum is exact in fp32
    rng = np.random.default_rng(5)
    E, d, k = 8, 64, 3
    x = (rng.integers(-2, 3, size=(T, d)) * 0.5).astype(np.float32)
    rw = np.zeros((E, d), np.float32)
    for e in range(E):
        rw[e, rng.choice(d, size=4, replace=False)] = 1.0
    rw[5] = rw[2]          # duplicated router rows: permanent ties between experts 2 and 5
    rw[7] = rw[0]
    w_np = {"router_w": rw, "router_b": None}
    for dtype in ("f32", "bf16"):
        x_np = x if dtype == "f32" else wl.f32_to_bf16_bits(x)
        idx, gate, _ = _route_gpu(dev, to_device(x_np, dev), weights_to_device(w_np, dev), E, k,
                                  DT[dtype])
        ref_idx, ref_gate, _, logits = oracle.route(x_np, rw, None, k)
        assert np.array_equal(idx, ref_idx)
        assert np.allclose(gate, ref_gate, rtol=1e-5)
        assert (np.sort(logits, 1)[:, -k] == np.sort(logits, 1)[:, -k - 1]).sum() > 20  # ties at the cut
    # all-zero router: every logit equal -> experts 0..k-1, gates exactly 1/k when k is a power of 2
    z = {"router_w": np.zeros((E, d), np.float32), "router_b": None}
    idx, gate, probs = _route_gpu(dev, to_device(x, dev), weights_to_device(z, dev), E, 2, pkg.MOE_F32)
    assert np.array_equal(idx, np.tile(np.arange(2, dtype=np.int32), (T, 1)))
    assert np.all(gate == 0.5) and np.all(probs == 0.125)


# ------------------------------------------------------------------------------- moe_permute

@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (1, 2, 8), (37, 2, 4), (512, 2, 8), (2048, 2, 8),
                                   (4096, 2, 8), (4097, 2, 8), (1000, 8, 64), (50000, 3, 7)])
def test_permute_matches_oracle_bit_exact(dev, oracle, T, k, E):
    rng = np.random.default_rng(T * 31 + E)
    # k distinct experts per token, skewed so some experts are empty or tiny
    scores = rng.standard_normal((T, E)) + np.linspace(2, -2, E)
    if E > 2:
        scores[:, 1] = -100  # expert 1 never chosen
    keys = np.argsort(-scores, axis=1)[:, :k].astype(np.int32)
    d = 64
    x_np = wl.normal_tensor(T, 1, (T, d), 1.0, "bf16")
    shape = pkg.make_shape(T, d, 64, E, k, 0, pkg.MOE_BF16)
    P = T * k
    off = torch.full((E + 1,), -1, dtype=torch.int32, device=dev)
    perm = torch.full((P,), -1, dtype=torch.int32, device=dev)
    inv = torch.full((P,), -1, dtype=torch.int32, device=dev)
    x_t = to_device(x_np, dev)
    xp = torch.zeros((P, d), dtype=torch.bfloat16, device=dev)
    ws = pkg.alloc_workspace(shape, dev)
    pkg.moe_permute(shape, to_device(keys, dev), off, perm, inv, x_t, xp, ws)
    torch.cuda.synchronize()
    r_off, r_perm, r_inv = oracle.permute(keys, E)
    assert np.array_equal(off.cpu().numpy(), r_off)
    assert np.array_equal(perm.cpu().numpy(), r_perm)
    assert np.array_equal(inv.cpu().numpy(), r_inv)
    assert np.array_equal(bits_of(xp), x_np[r_perm // k])
    # unpermute(permute(x)) is the identity on the payload
    assert np.array_equal(bits_of(xp)[r_inv].reshape(T, k, d)[:, 0], x_np)


@pytest.mark.parametrize("T,k,E", [(1_000_000, 4, 64), ((1 << 21) - 1, 8, 8)])
def test_permute_large_without_payload(dev, oracle, T, k, E):
    # several hundred workgroups per kernel of the multi-pass sort; the second case is the
    # largest pair count the library accepts (T k just under 2^24)
    rng = np.random.default_rng(E * 1000 + k)
    keys = np.argsort(rng.random((T, E), dtype=np.float32) + np.linspace(0.6, 0, E, dtype=np.float32),
                      axis=1)[:, :k].astype(np.int32)
    shape = pkg.make_shape(T, 8, 8, E, k, 0, pkg.MOE_BF16)
    P = T * k
    assert P < (1 << 24)
    off = torch.full((E + 1,), -1, dtype=torch.int32, device=dev)
    perm = torch.full((P,), -1, dtype=torch.int32, device=dev)
    inv = torch.full((P,), -1, dtype=torch.int32, device=dev)
    ws = pkg.alloc_workspace(shape, dev)
    pkg.moe_permute(shape, to_device(keys, dev), off, perm, inv, None, None, ws)
    torch.cuda.synchronize()
    r_off, r_perm, r_inv = oracle.permute(keys, E)
    assert np.array_equal(off.cpu().numpy(), r_off)
    assert np.array_equal(perm.cpu().numpy(), r_perm)
    assert np.array_equal(inv.cpu().numpy(), r_inv)


# ------------------------------------------------------------------------------- moe_expert_ffn

def _ffn_case(dev, oracle, cfg, offsets, tol):
    w_np = wl.make_layer_weights(cfg, with_bias=False)
    P = int(offsets[-1])
    xp_np = wl.normal_tensor(cfg.seed, 77, (P, cfg.d_model), 1.0, cfg.act_dtype)
    w_t = weights_to_device(w_np, dev)
    # the staged call sees P rows as P "tokens" with k = 1
    shape = pkg.shape_for(w_t, P, 1, DT[cfg.act_dtype])
    ws = pkg.alloc_workspace(shape, dev)
    xp = to_device(xp_np, dev)
    yp = torch.full_like(xp, float("nan"))
    pkg.moe_expert_ffn(shape, pkg.make_weights(w_t), xp, to_device(offsets, dev), yp, ws)
    torch.cuda.synchronize()
    ref = oracle.expert_ffn(w_np, xp_np, offsets)
    got = to_f64(yp)
    assert np.all(np.isfinite(got))
    err = rel_err(got, ref)
    assert err < tol, f"relative error {err:.3e} >= {tol}"
    return err


def test_expert_ffn_tiny_fp32(dev, oracle):
    cfg = _cfg(d=128, F=256, E=4, dtype="f32", seed=401, std=0.05)
    _ffn_case(dev, oracle, cfg, np.array([0, 20, 20, 49, 64], np.int32), TOL["f32"])


@pytest.mark.parametrize("d,F,offsets", [
    (256, 384, [0, 130, 130, 257, 300]),          # several m-tiles, an empty expert, ragged tails
    (200, 328, [0, 1, 3, 70, 71]),                # K and N not multiples of the tile, tiny groups
    (1024, 2816, [0, 64, 200, 200, 333, 333, 400, 401, 520]),  # wearables widths, 8 experts
    # 585 gate/up tiles of 256 x 256: 74 (or 67) per XCD = two rounds of 32 and a thin third one, whose
    # tiles are cut into upper and lower halves; the cut tiles include ragged ones (164 and 120 live rows)
    (128, 5760, [0, 1700, 3100]),
    # 540 gate/up tiles of 256 x 256: 68 per XCD = two rounds and 4 tiles that are cut
    (128, 5760, [0, 1700, 2900]),
    # the same for a kernel that runs two workgroups per CU: 576 down tiles of 128 x 128, 72 per XCD =
    # one round of 64 and 8 tiles cut into halves (the last tile of the second group holds 74 rows)
    (2048, 192, [0, 2304, 4554]),
    # K tails in the 256-row kernel: K = 72 is two k-steps of 32 and a tail of 8; the down product
    # then has K = 4008 (a tail of 40 in a 64-wide step)
    (72, 4008, [0, 1700, 3100]),
    # K shorter than one k-step: the only step is the tail
    (24, 4104, [0, 1500, 3000]),
])
def test_expert_ffn_dense_bf16(dev, oracle, d, F, offsets):
    cfg = _cfg(d=d, F=F, E=len(offsets) - 1, dtype="bf16", seed=402 + d, std=0.05)
    _ffn_case(dev, oracle, cfg, np.array(offsets, np.int32), TOL["bf16"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("base", [False, True])
def test_expert_ffn_weight_decomposed(dev, oracle, dtype, base):
    cfg = _cfg(d=256, F=448, E=4, dtype=dtype, seed=410, r=(40 if base else 128), base=base, std=0.05)
    _ffn_case(dev, oracle, cfg, np.array([0, 150, 150, 161, 300], np.int32), TOL[dtype])


# ------------------------------------------------------------------------------- moe_combine

@pytest.mark.parametrize("dtype,residual", [("f32", False), ("bf16", True), ("bf16", False)])
def test_combine_matches_oracle(dev, oracle, dtype, residual):
    T, k, d, E = 75, 3, 264, 6
    rng = np.random.default_rng(9)
    keys = np.argsort(rng.standard_normal((T, E)), axis=1)[:, :k].astype(np.int32)
    _, _, inv = oracle.permute(keys, E)
    yp_np = wl.normal_tensor(9, 1, (T * k, d), 1.0, dtype)
    res_np = wl.normal_tensor(9, 2, (T, d), 1.0, dtype) if residual else None
    g = rng.random((T, k)).astype(np.float32)
    g /= g.sum(1, keepdims=True)
    shape = pkg.make_shape(T, d, 64, E, k, 0, DT[dtype])
    y = torch.empty((T, d), dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device=dev)
    pkg.moe_combine(shape, to_device(yp_np, dev), to_device(inv, dev), to_device(g, dev),
                    to_device(res_np, dev), y)
    torch.cuda.synchronize()
    ref = oracle.combine(stored_f64(yp_np), inv, g.astype(np.float64), residual=res_np)
    assert rel_err(to_f64(y), ref) < (1e-6 if dtype == "f32" else 5e-3)


# ------------------------------------------------------------------------------- moe_forward

def _forward_gpu(dev, w_t, x_t, k, act, residual=False):
    T = x_t.shape[0]
    shape = pkg.shape_for(w_t, T, k, act, residual=residual)
    ws = pkg.alloc_workspace(shape, dev)
    y = torch.full_like(x_t, float("nan"))
    idx = torch.full((T, k), -1, dtype=torch.int32, device=dev)
    gate = torch.zeros((T, k), dtype=torch.float32, device=dev)
    pkg.moe_forward(shape, pkg.make_weights(w_t), x_t, y, idx, gate, ws)
    torch.cuda.synchronize()
    return y, idx.cpu().numpy(), gate.cpu().numpy().astype(np.float64)


def _forward_case(dev, oracle, cfg, T, w_np=None, w_t=None, sample=None, residual=False):
    """moe_forward vs the oracle.  sample: compare y only on that many seeded tokens (routing
    is always compared on all of them)."""
    if w_np is None:
        w_np = wl.make_layer_weights(cfg)
    if w_t is None:
        w_t = weights_to_device(w_np, dev)
    x_np = wl.make_inputs(cfg, T)
    y, idx, gate = _forward_gpu(dev, w_t, to_device(x_np, dev), cfg.top_k, DT[cfg.act_dtype], residual)
    same, _, _ = _check_routing(oracle, x_np, w_np, cfg.top_k, idx, gate)
    got = to_f64(y)
    assert np.all(np.isfinite(got))
    toks = np.arange(T)
    if sample is not None and sample < T:
        toks = np.sort(np.random.default_rng(cfg.seed).choice(T, size=sample, replace=False))
    toks = toks[same[toks]]
    ref, ridx, _ = oracle.forward(w_np, np.ascontiguousarray(x_np[toks]), cfg.top_k, residual=residual)
    assert np.array_equal(ridx, idx[toks])
    err = rel_err(got[toks], ref)
    tol = TOL[cfg.act_dtype]
    assert err < tol, f"{cfg.name} T={T}: relative error {err:.3e} >= {tol}"
    # no row may hide behind the norm of the whole tensor, and no sizeable element may be far off
    row_err = row_rel_err(got[toks], ref)
    assert row_err < tol, f"{cfg.name} T={T}: worst row's relative error {row_err:.3e} >= {tol}"
    elem_err = elementwise_rel_err(got[toks], ref)
    assert elem_err < ELEMENTWISE_TOL[cfg.act_dtype], \
        f"{cfg.name} T={T}: worst element-wise relative error {elem_err:.3e}"
    print(f"[parity] {cfg.name} T={T} tokens compared={len(toks)} tensor={err:.3e} worst-row={row_err:.3e} "
          f"worst-element={elem_err:.3e}")
    return err


def test_forward_tiny_fp32_config(dev, oracle):
    cfg = wl.CONFIGS["tiny"]
    _forward_case(dev, oracle, cfg, 32)
    _forward_case(dev, oracle, cfg, 1)
    _forward_case(dev, oracle, cfg, 5, residual=True)


@pytest.mark.parametrize("T", [1, 2, 3, 130, 512, 1024, 20000])
def test_forward_wearables_config(dev, oracle, T):
    # 130 and 512: 64-row GEMM tiles (and two k-groups for the down product); 1024: 128-row tiles;
    # 20000: 256-row tiles over many m-tiles and the multi-workgroup sort inside the forward
    _forward_case(dev, oracle, wl.CONFIGS["wearables"], T, sample=1024)  # all tokens but at T = 20000


@pytest.mark.parametrize("T", [1, 40, 700])
def test_forward_many_experts(dev, oracle, T):
    cfg = _cfg(name="e64", d=256, F=512, E=64, k=8, dtype="bf16", seed=640, std=0.05)
    _forward_case(dev, oracle, cfg, T)


@pytest.fixture(scope="module")
def phone(dev):
    cfg = wl.CONFIGS["phone"]
    w_np = wl.make_layer_weights(cfg)
    return cfg, w_np, weights_to_device(w_np, dev)


def test_forward_phone_config_decode_and_prefill(dev, oracle, phone):
    cfg, w_np, w_t = phone
    _forward_case(dev, oracle, cfg, 1, w_np, w_t)
    _forward_case(dev, oracle, cfg, 2048, w_np, w_t)  # every token's output is compared
    # the stored router bias must realise the Zipf(1.1) expert loads it was calibrated for
    x_np = wl.make_inputs(cfg, 2048)
    idx, _, _, _ = oracle.route(x_np, w_np["router_w"], w_np["router_b"], cfg.top_k)
    share = np.bincount(idx.reshape(-1), minlength=8) / idx.size
    assert np.abs(share - wl.zipf_target_shares(8, 1.1)).max() < 0.01


def test_staged_calls_at_the_phone_prefill_size(dev, oracle, phone):
    # route -> permute (with the gather) -> expert FFN -> combine through the four staged entry
    # points at the size the benchmark runs: the staged expert FFN takes the single-output down
    # projection (128 x 128 tiles), which moe_forward no longer does at this size
    cfg, w_np, w_t = phone
    T, k, E, d = 2048, cfg.top_k, cfg.n_experts, cfg.d_model
    x_np = wl.make_inputs(cfg, T)
    x_t = to_device(x_np, dev)
    shape = pkg.shape_for(w_t, T, k, pkg.MOE_BF16)
    P = T * k
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    gate = torch.empty((T, k), dtype=torch.float32, device=dev)
    pkg.moe_route(shape, x_t, w_t["router_w"], w_t["router_b"], idx, gate, None)
    off = torch.empty(E + 1, dtype=torch.int32, device=dev)
    perm = torch.empty(P, dtype=torch.int32, device=dev)
    inv = torch.empty(P, dtype=torch.int32, device=dev)
    xp = torch.empty((P, d), dtype=torch.bfloat16, device=dev)
    pkg.moe_permute(shape, idx, off, perm, inv, x_t, xp, pkg.alloc_workspace(shape, dev))
    yp = torch.full_like(xp, float("nan"))
    ffn_shape = pkg.shape_for(w_t, P, 1, pkg.MOE_BF16)
    pkg.moe_expert_ffn(ffn_shape, pkg.make_weights(w_t), xp, off, yp, pkg.alloc_workspace(ffn_shape, dev))
    y = torch.full_like(x_t, float("nan"))
    pkg.moe_combine(shape, yp, inv, gate, None, y)
    torch.cuda.synchronize()
    idx_np = idx.cpu().numpy()
    same, _, _ = _check_routing(oracle, x_np, w_np, k, idx_np, gate.cpu().numpy().astype(np.float64))
    r_off, r_perm, r_inv = oracle.permute(idx_np, E)
    assert np.array_equal(off.cpu().numpy(), r_off) and np.array_equal(perm.cpu().numpy(), r_perm)
    assert np.array_equal(inv.cpu().numpy(), r_inv)
    toks = np.sort(np.random.default_rng(5).choice(T, size=512, replace=False))
    toks = toks[same[toks]]
    ref, _, _ = oracle.forward(w_np, np.ascontiguousarray(x_np[toks]), k)
    got = to_f64(y)
    assert np.all(np.isfinite(got))
    assert rel_err(got[toks], ref) < TOL["bf16"] and row_rel_err(got[toks], ref) < TOL["bf16"]
    # and against moe_forward on the same input (k-parts in its down projection: close, not equal)
    y_fwd, idx_fwd, _ = _forward_gpu(dev, w_t, x_t, k, pkg.MOE_BF16)
    assert np.array_equal(idx_fwd, idx_np)
    assert rel_err(to_f64(y_fwd), got) < 1e-2


@pytest.mark.parametrize("static", [False, True])
def test_forward_replayed_from_a_hip_graph_matches_eager(dev, static):
    # a prefill step and a single-token step captured into one graph and replayed several times with
    # eager work and synchronisations between the replays: every replay must reproduce the eager bits
    cfg = wl.shrink(wl.CONFIGS["wearables"], d_model=512, d_ff=1024)
    w_t = weights_to_device(wl.make_layer_weights(cfg), dev)
    k = cfg.top_k
    xs = [to_device(wl.make_inputs(cfg, T, step=T), dev) for T in (96, 1)]
    shapes = [pkg.shape_for(w_t, x.shape[0], k, pkg.MOE_BF16) for x in xs]
    wss = [pkg.alloc_workspace(sh, dev) for sh in shapes]
    weights = pkg.make_weights(w_t)

    def run(outs):
        for x, sh, ws, (y, idx, gate) in zip(xs, shapes, wss, outs):
            if static:
                pkg.moe_forward_static(sh, weights, x, y, idx, gate)
            else:
                pkg.moe_forward(sh, weights, x, y, idx, gate, ws)

    def fresh():
        return [(torch.full_like(x, float("nan")), torch.full((x.shape[0], k), -1, dtype=torch.int32, device=dev),
                 torch.zeros((x.shape[0], k), dtype=torch.float32, device=dev)) for x in xs]

    eager = fresh()
    run(eager)
    torch.cuda.synchronize()
    captured = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(captured)  # warm-up on the capture stream (one-time set-up calls happen here, not under capture)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            run(captured)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(4):
        for y, idx, gate in captured:  # clear with fill kernels, outside the graph
            y.fill_(float("nan"))
            idx.fill_(-1)
        other = fresh()
        run(other)  # eager work between the replays, on the same scratch
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (y, idx, gate), (ye, ie, ge), (yo, io, go) in zip(captured, eager, other):
            assert torch.equal(y, ye) and torch.equal(idx, ie) and torch.equal(gate, ge), f"replay {rep}"
            assert torch.equal(yo, ye)


@pytest.mark.parametrize("T", [2, 3, 5, 8])
def test_forward_phone_config_few_tokens(dev, oracle, phone, T):
    # two tokens take the matrix-vector path (their pairs are walked like one token's), three and
    # more the grouped GEMM with a row or two per expert
    cfg, w_np, w_t = phone
    _forward_case(dev, oracle, cfg, T, w_np, w_t)
    _forward_case(dev, oracle, cfg, T, w_np, w_t, residual=True)


@pytest.mark.parametrize("name,T", [("phone_wd", 2), ("phone_wd", 7), ("phone_wd_base", 2)])
def test_forward_weight_decomposed_few_tokens(dev, oracle, name, T):
    # pure L R experts: four matrix-vector stages with per-token and per-pair inputs; a shared base
    # keeps the grouped GEMM at these sizes
    cfg = wl.CONFIGS[name]
    _forward_case(dev, oracle, cfg, T)


@pytest.mark.parametrize("k,E,T,dtype", [(32, 64, 2, "bf16"), (33, 64, 2, "bf16"), (3, 5, 2, "f32"), (1, 4, 2, "bf16"),
                                         (7, 9, 2, "bf16"), (8, 64, 3, "bf16")])
def test_forward_few_tokens_pair_limits(dev, oracle, k, E, T, dtype):
    # two tokens on the matrix-vector path: 64 pairs is the most it takes (2 x 33 go to the grouped
    # GEMM); odd k makes a group of two pairs span both tokens; k = 1 is one pair per token
    cfg = _cfg(name=f"ft{k}{E}", d=264, F=520, E=E, k=k, dtype=dtype, seed=1300 + k + E + T, std=0.05)
    _forward_case(dev, oracle, cfg, T, residual=bool(k % 2))


@pytest.mark.parametrize("name", ["phone_wd", "phone_wd_base"])
def test_forward_phone_weight_decomposed_configs(dev, oracle, name):
    cfg = wl.CONFIGS[name]
    w_np = wl.make_layer_weights(cfg)
    w_t = weights_to_device(w_np, dev)
    _forward_case(dev, oracle, cfg, 1, w_np, w_t)
    _forward_case(dev, oracle, cfg, 2048, w_np, w_t)  # every token's output is compared


def test_forward_small_shapes_all_expert_kinds(dev, oracle):
    for dtype in ("f32", "bf16"):
        for r, base in ((0, False), (64, False), (24, True)):
            cfg = _cfg(name=f"s{r}{base}", d=192, F=328, E=5, k=3, dtype=dtype, seed=500 + r,
                       r=r, base=base, std=0.05)
            for T in (1, 7, 150):
                _forward_case(dev, oracle, cfg, T, residual=(T == 7))


def _sweep_cases(n, seed):
    """n seeded (d, F, E, k, r, base, dtype, T) combinations: widths any multiple of 8, from
    narrower than one k-step of the GEMM to a few tiles wide; token counts from one to a few
    hundred; every expert kind."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        d = 8 * int(rng.integers(1, 41))
        F = 8 * int(rng.integers(1, 65))
        E = int(rng.integers(1, 13))
        k = int(rng.integers(1, E + 1))
        kind = int(rng.integers(0, 3))  # dense / pure L R / shared base + L R
        r = 0 if kind == 0 else 8 * int(rng.integers(1, 9))
        dtype = "f32" if rng.integers(0, 4) == 0 else "bf16"
        T = int(rng.choice([1, 2, 3, 5, 17, 64, 129, 300, 400]))
        cases.append((d, F, E, k, r, kind == 2, dtype, T))
    return cases


@pytest.mark.parametrize("d,F,E,k,r,base,dtype,T", _sweep_cases(28, 20250300245))
def test_forward_seeded_shape_sweep(dev, oracle, d, F, E, k, r, base, dtype, T):
    cfg = _cfg(name="sw", d=d, F=F, E=E, k=k, dtype=dtype, seed=7000 + d + F + E + k + r + T, r=r,
               base=base, std=0.08)
    _forward_case(dev, oracle, cfg, T, residual=bool((d + T) % 2))


def _prefill_sweep_cases(n, seed):
    """n seeded prefill-sized combinations: a few hundred rows per expert and widths up to a dozen
    tiles, so the 256- and 128-row GEMM kernels run with K tails, ragged groups and cut tiles."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        d = 8 * int(rng.integers(16, 160))
        F = 8 * int(rng.integers(32, 400))
        E = int(rng.integers(2, 9))
        k = int(rng.integers(1, min(E, 4) + 1))
        kind = int(rng.integers(0, 3))
        r = 0 if kind == 0 else 8 * int(rng.integers(2, 33))
        T = int(rng.integers(600, 3000))
        cases.append((d, F, E, k, r, kind == 2, T))
    return cases


@pytest.mark.parametrize("d,F,E,k,r,base,T", _prefill_sweep_cases(10, 2503))
def test_forward_seeded_prefill_sweep(dev, oracle, d, F, E, k, r, base, T):
    cfg = _cfg(name="pf", d=d, F=F, E=E, k=k, dtype="bf16", seed=8000 + d + F + E + k + r + T, r=r,
               base=base, std=0.04)
    _forward_case(dev, oracle, cfg, T, sample=256)


@pytest.mark.parametrize("d,F,E,k,T", [
    (256, 2048, 3, 2, 1500),   # 32 steps of 64 cut into 4 parts of 8
    (256, 2080, 2, 1, 2000),   # 32 whole steps and a tail of 32: only the last part holds the tail
    (512, 4128, 2, 2, 1100),   # 64.5 steps, two output tiles per row tile
])
def test_forward_down_projection_cut_along_k(dev, oracle, d, F, E, k, T):
    # tall groups, a narrow output and a long K: the down projection's 256 x 256 tiles are too few
    # for the chip, so moe_forward cuts every tile's k-steps into parts whose partial outputs the
    # combine adds; the result must still match the oracle and the staged calls (one part) closely
    cfg = _cfg(name="kp", d=d, F=F, E=E, k=k, dtype="bf16", seed=1200 + F, std=0.04)
    w_np = wl.make_layer_weights(cfg, with_bias=False)
    w_t = weights_to_device(w_np, dev)
    _forward_case(dev, oracle, cfg, T, w_np, w_t, sample=300)
    # staged calls on the same input
    x_t = to_device(wl.make_inputs(cfg, T), dev)
    y1, idx1, _ = _forward_gpu(dev, w_t, x_t, k, pkg.MOE_BF16)
    shape = pkg.shape_for(w_t, T, k, pkg.MOE_BF16)
    P = T * k
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    gate = torch.empty((T, k), dtype=torch.float32, device=dev)
    pkg.moe_route(shape, x_t, w_t["router_w"], None, idx, gate, None)
    off = torch.empty(E + 1, dtype=torch.int32, device=dev)
    perm = torch.empty(P, dtype=torch.int32, device=dev)
    inv = torch.empty(P, dtype=torch.int32, device=dev)
    xp = torch.empty((P, d), dtype=torch.bfloat16, device=dev)
    pkg.moe_permute(shape, idx, off, perm, inv, x_t, xp, pkg.alloc_workspace(shape, dev))
    yp = torch.empty_like(xp)
    ffn_shape = pkg.shape_for(w_t, P, 1, pkg.MOE_BF16)
    pkg.moe_expert_ffn(ffn_shape, pkg.make_weights(w_t), xp, off, yp, pkg.alloc_workspace(ffn_shape, dev))
    y3 = torch.empty_like(x_t)
    pkg.moe_combine(shape, yp, inv, gate, None, y3)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), idx1)
    assert rel_err(to_f64(y1), to_f64(y3)) < 1e-2  # parts are rounded to bf16 one by one


@pytest.mark.parametrize("k,E,T", [(2, 8, 2), (2, 8, 37), (2, 8, 600), (3, 5, 150), (8, 8, 64), (2, 16, 9)])
def test_forward_shared_base_once_per_token(dev, oracle, k, E, T):
    # bf16 layers with k > 1 take the path that applies the shared base once per token (plain
    # products over T rows, low-rank terms per pair, the shared down term added in the combine);
    # T = 9 with 16 experts leaves most groups empty, T = 600 spans several tiles
    cfg = _cfg(name=f"tb{k}{E}", d=256, F=448, E=E, k=k, dtype="bf16", seed=900 + k + E, r=64,
               base=True, std=0.05)
    _forward_case(dev, oracle, cfg, T, residual=(T == 37))


@pytest.mark.parametrize("T", [5, 300, 1500])
def test_forward_shared_base_once_per_token_ragged_widths(dev, oracle, T):
    # the same path with widths that are multiples of 8 only: every product has a K tail
    # (200 = 3 x 64 + 8, 328 = 5 x 64 + 8, rank 40 is shorter than one k-step)
    cfg = _cfg(name="tbr", d=200, F=328, E=4, k=2, dtype="bf16", seed=931, r=40, base=True, std=0.05)
    _forward_case(dev, oracle, cfg, T)


def test_forward_is_deterministic_and_matches_the_staged_calls(dev, oracle):
    cfg = wl.shrink(wl.CONFIGS["wearables"], d_model=512, d_ff=1024)
    w_np = wl.make_layer_weights(cfg)
    w_t = weights_to_device(w_np, dev)
    T, k = 200, cfg.top_k
    x_t = to_device(wl.make_inputs(cfg, T), dev)
    y1, idx1, gate1 = _forward_gpu(dev, w_t, x_t, k, pkg.MOE_BF16)
    y2, idx2, gate2 = _forward_gpu(dev, w_t, x_t, k, pkg.MOE_BF16)
    assert torch.equal(y1, y2) and np.array_equal(idx1, idx2) and np.array_equal(gate1, gate2)
    # staged pipeline through the same ABI
    shape = pkg.shape_for(w_t, T, k, pkg.MOE_BF16)
    ws = pkg.alloc_workspace(shape, dev)
    P = T * k
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    gate = torch.empty((T, k), dtype=torch.float32, device=dev)
    pkg.moe_route(shape, x_t, w_t["router_w"], None, idx, gate, None)
    off = torch.empty(cfg.n_experts + 1, dtype=torch.int32, device=dev)
    perm = torch.empty(P, dtype=torch.int32, device=dev)
    inv = torch.empty(P, dtype=torch.int32, device=dev)
    xp = torch.empty((P, cfg.d_model), dtype=torch.bfloat16, device=dev)
    pkg.moe_permute(shape, idx, off, perm, inv, x_t, xp, ws)
    yp = torch.empty_like(xp)
    ffn_shape = pkg.shape_for(w_t, P, 1, pkg.MOE_BF16)
    pkg.moe_expert_ffn(ffn_shape, pkg.make_weights(w_t), xp, off, yp, pkg.alloc_workspace(ffn_shape, dev))
    y3 = torch.empty_like(x_t)
    pkg.moe_combine(shape, yp, inv, gate, None, y3)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), idx1)          # routing bit-identical
    assert np.array_equal(gate.cpu().numpy().astype(np.float64), gate1)
    assert torch.equal(y3, y1)                               # same kernels, same bits


# ------------------------------------------------------------------------------- moe_stack_forward

def _stack_case(dev, oracle, cfg, n_layers, T):
    layers_np = wl.make_stack_weights(cfg, n_layers)
    layers_t = [weights_to_device(w, dev) for w in layers_np]
    x_np = wl.make_inputs(cfg, T)
    act = DT[cfg.act_dtype]
    shape = pkg.shape_for(layers_t[0], T, cfg.top_k, act)
    ws = pkg.alloc_workspace(shape, dev)
    x_t = to_device(x_np, dev)
    y = torch.empty_like(x_t)
    trace = torch.full((n_layers, T, cfg.top_k), -1, dtype=torch.int32, device=dev)
    pkg.moe_stack_forward(shape, [pkg.make_weights(w) for w in layers_t], x_t, y, trace, ws)
    torch.cuda.synchronize()
    y_ref, trace_ref, xs = oracle.stack_forward(layers_np, x_np, cfg.top_k)
    trace = trace.cpu().numpy()
    # free-running: compare the final residual on tokens whose routing never flipped
    clean = np.all(trace == trace_ref, axis=(0, 2))
    assert clean.mean() > 0.9, "too many routing flips for near-tie noise"
    err = rel_err(to_f64(y)[clean], y_ref[clean])
    assert err < TOL[cfg.act_dtype], f"stack error {err:.3e}"
    # teacher-forced: each GPU layer fed the oracle's (storage-rounded) input of that layer
    for l in range(n_layers):
        xin = xs[l].astype(np.float32)
        xin = xin if cfg.act_dtype == "f32" else wl.f32_to_bf16_bits(xin)
        yl, idx, gate = _forward_gpu(dev, layers_t[l], to_device(xin, dev), cfg.top_k, act, residual=True)
        same, _, _ = _check_routing(oracle, xin, layers_np[l], cfg.top_k, idx, gate)
        ref, _, _ = oracle.forward(layers_np[l], xin, cfg.top_k, residual=True)
        assert rel_err(to_f64(yl)[same], ref[same]) < TOL[cfg.act_dtype]


def test_stack_small(dev, oracle):
    cfg = wl.shrink(wl.CONFIGS["phone_stack"], d_model=256, d_ff=512, weight_std=0.05)
    _stack_case(dev, oracle, cfg, 5, 1)
    _stack_case(dev, oracle, cfg, 4, 40)


def test_stack_phone_width_decode(dev, oracle):
    _stack_case(dev, oracle, wl.CONFIGS["phone_stack"], 3, 1)


def test_stack_phone_full_depth_decode_loop(dev, oracle):
    """The fifth benchmark configuration at its stated size: 24 phone-shaped layers with
    residual adds, one token per step, several steps with a fresh N(0,1) token each.
    Teacher-forced, every layer of every step: the GPU layer is fed the oracle's input of that
    layer (rounded to bf16); routing must be bit-exact off the ambiguous set and the output
    within tolerance.  Free-running, to the end of the stack: the final residual stream is
    compared on the steps whose routing never left the oracle's; flips are counted and printed."""
    cfg = wl.CONFIGS["phone_stack"]
    n_layers, n_steps, k = cfg.n_layers, 6, cfg.top_k
    assert n_layers == 24
    layers_np = wl.make_stack_weights(cfg, n_layers)
    layers_t = [weights_to_device(w, dev) for w in layers_np]
    structs = [pkg.make_weights(w) for w in layers_t]
    shape = pkg.shape_for(layers_t[0], 1, k, pkg.MOE_BF16)
    ws = pkg.alloc_workspace(shape, dev)
    clean_steps, free_errs, forced_worst, n_amb = 0, [], 0.0, 0
    for step in range(n_steps):
        x_np = wl.make_inputs(cfg, 1, step=step)
        x_t = to_device(x_np, dev)
        y = torch.full_like(x_t, float("nan"))
        trace = torch.full((n_layers, 1, k), -1, dtype=torch.int32, device=dev)
        pkg.moe_stack_forward(shape, structs, x_t, y, trace, ws)
        torch.cuda.synchronize()
        y_ref, trace_ref, xs = oracle.stack_forward(layers_np, x_np, k)
        tr = trace.cpu().numpy()
        flips = int(np.any(tr != trace_ref, axis=(1, 2)).sum())
        first_flip = int(np.argmax(np.any(tr != trace_ref, axis=(1, 2)))) if flips else -1
        got = to_f64(y)
        assert np.all(np.isfinite(got))
        err = rel_err(got, y_ref)
        growth = float(np.sqrt(np.mean(y_ref ** 2)))
        print(f"[stack24] step {step}: layers whose routing differs {flips} (first at {first_flip}), "
              f"free-running error of the final stream {err:.3e}, rms of the final stream {growth:.2f}")
        if flips == 0:
            clean_steps += 1
            free_errs.append(err)
            assert err < TOL["bf16"], f"step {step}: free-running error {err:.3e} at depth {n_layers}"
        # teacher-forced, layer by layer
        for l in range(n_layers):
            xin = wl.f32_to_bf16_bits(xs[l].astype(np.float32))
            yl, idx, gate = _forward_gpu(dev, layers_t[l], to_device(xin, dev), k, pkg.MOE_BF16, residual=True)
            same, _, _ = _check_routing(oracle, xin, layers_np[l], k, idx, gate)
            n_amb += int((~same).sum())
            if same[0]:
                ref, _, _ = oracle.forward(layers_np[l], xin, k, residual=True)
                e = rel_err(to_f64(yl), ref)
                assert e < TOL["bf16"], f"step {step} layer {l}: teacher-forced error {e:.3e}"
                # the stream is mostly the residual, so also compare the layer's own contribution
                yc, idx_c, _ = _forward_gpu(dev, layers_t[l], to_device(xin, dev), k, pkg.MOE_BF16)
                assert np.array_equal(idx_c, idx)
                ref_c, _, _ = oracle.forward(layers_np[l], xin, k)
                ec = rel_err(to_f64(yc), ref_c)
                assert ec < TOL["bf16"], f"step {step} layer {l}: error of the layer's contribution {ec:.3e}"
                forced_worst = max(forced_worst, e, ec)
    print(f"[stack24] {clean_steps}/{n_steps} steps without a routing flip, worst free-running error on them "
          f"{max(free_errs) if free_errs else float('nan'):.3e}; worst teacher-forced layer error {forced_worst:.3e}; "
          f"teacher-forced ambiguous picks {n_amb}")
    assert clean_steps >= 1, "every step's routing left the oracle's somewhere in the 24 layers"


# ------------------------------------------------------------------------------- routing-trace metrics

def _fig5_trace(name):
    import os
    m = np.loadtxt(os.path.join(os.path.dirname(__file__), "golden", name), dtype=np.int64, comments="#")
    return np.stack([np.flatnonzero(m[:, t]) for t in range(m.shape[1])]).astype(np.int32)[None]


def _random_trace(seed, B, T, K, E, sticky=0.7):
    """Selections that change only now and then, like a router with temporal locality."""
    rng = np.random.default_rng(seed)
    S = np.zeros((B, T, K), np.int32)
    for b in range(B):
        cur = rng.permutation(E)[:K]
        for t in range(T):
            if rng.random() > sticky:
                cur = cur.copy()
                cur[rng.integers(K)] = rng.choice(np.setdiff1d(np.arange(E), cur)) if E > K else cur[0]
            S[b, t] = rng.permutation(cur)
    return S


@pytest.mark.parametrize("case", ["fig5_bles", "fig5_moe", "random", "single_token", "wide", "long"])
def test_expert_replacements_match_oracle_bit_exact(dev, oracle, case):
    if case.startswith("fig5"):
        S, E = _fig5_trace(case + ".txt"), 8
    elif case == "random":
        S, E = _random_trace(1, 5, 333, 2, 8), 8
    elif case == "single_token":
        S, E = _random_trace(2, 4, 1, 2, 8), 8
    elif case == "wide":
        S, E = _random_trace(3, 2, 700, 8, 64, sticky=0.3), 64
    else:
        S, E = _random_trace(4, 24, 4096, 2, 8), 8
    He = torch.full((E,), -1, dtype=torch.int64, device=dev)
    H = torch.full((1,), -1, dtype=torch.int64, device=dev)
    pkg.moe_expert_replacements(to_device(S, dev), E, He, H)
    torch.cuda.synchronize()
    rH, rHe = oracle.expert_replacements(S, E)
    assert int(H.item()) == rH and np.array_equal(He.cpu().numpy(), rHe)
    if case == "fig5_bles":
        assert rH // 2 == 11
    if case == "fig5_moe":
        assert rH // 2 == 21


@pytest.mark.parametrize("B,T,K,E", [(1, 2, 1, 2), (3, 257, 2, 8), (2, 2048, 2, 8), (1, 1, 2, 4), (4, 100, 8, 64)])
def test_bles_loss_value_matches_oracle(dev, oracle, B, T, K, E):
    rng = np.random.default_rng(B * 1000 + T)
    W = rng.random((B, T, E)).astype(np.float32) ** 3
    W /= W.sum(-1, keepdims=True)
    S = np.argsort(-W, axis=-1, kind="stable")[..., :K].astype(np.int32)
    out = torch.full((5,), float("nan"), dtype=torch.float64, device=dev)
    ws = torch.empty(pkg.moe_bles_workspace_bytes(B, T, E), dtype=torch.uint8, device=dev)
    pkg.moe_bles_loss(to_device(W, dev), to_device(S, dev), out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ref = oracle.bles_loss(W, S)
    assert got[0] == ref["H"] and got[1] == ref["H_norm"]          # integer part exact
    for i, key in ((2, "L"), (3, "L_norm"), (4, "loss")):            # fp32 block sums, fp64 total
        assert abs(got[i] - ref[key]) <= 2e-6 * max(abs(ref[key]), 1e-30), (key, got[i], ref[key])


def test_bles_loss_from_the_routers_own_probabilities(dev, oracle):
    cfg = _cfg(d=256, E=8, k=2, dtype="bf16", seed=77, std=0.3)
    w_np = wl.make_layer_weights(cfg, with_bias=False)
    B, T = 3, 200
    x_np = wl.make_inputs(cfg, B * T)
    w_t = weights_to_device({"router_w": w_np["router_w"], "router_b": None}, dev)
    idx, gate, probs = _route_gpu(dev, to_device(x_np, dev), w_t, 8, 2, pkg.MOE_BF16)
    probs_t = to_device(probs.astype(np.float32).reshape(B, T, 8), dev)
    S_t = to_device(idx.reshape(B, T, 2), dev)
    out = torch.zeros(5, dtype=torch.float64, device=dev)
    ws = torch.empty(pkg.moe_bles_workspace_bytes(B, T, 8), dtype=torch.uint8, device=dev)
    pkg.moe_bles_loss(probs_t, S_t, out, ws)
    torch.cuda.synchronize()
    ref = oracle.bles_loss(probs.astype(np.float32).reshape(B, T, 8), idx.reshape(B, T, 2))
    got = out.cpu().numpy()
    assert got[0] == ref["H"] and abs(got[4] - ref["loss"]) <= 2e-6 * ref["loss"]
    assert 0.0 < ref["loss"] < 2.0


@pytest.mark.parametrize("L,T,K,E", [(1, 35, 2, 8), (24, 256, 2, 8), (3, 1, 2, 4), (2, 1000, 4, 16), (5, 300, 8, 64)])
def test_offload_counters_match_oracle_bit_exact(dev, oracle, L, T, K, E):
    tr = _fig5_trace("fig5_moe.txt") if (L, T) == (1, 35) else _random_trace(L + T, L, T, K, E, sticky=0.6)
    ch = torch.full((L,), -1, dtype=torch.int64, device=dev)
    ld = torch.full((L,), -1, dtype=torch.int64, device=dev)
    pkg.moe_offload_counters(to_device(tr, dev), E, ch, ld)
    torch.cuda.synchronize()
    rch, rld = oracle.offload_counters(tr, E)
    assert np.array_equal(ch.cpu().numpy(), rch) and np.array_equal(ld.cpu().numpy(), rld)
    if (L, T) == (1, 35):
        assert rld[0] == 2 + 21  # the paper's 21 replacements after the initial fill


@pytest.mark.parametrize("case", ["fig5", "random", "single_token", "wide", "long", "collapsed", "stray"])
def test_delta_uniform_matches_oracle(dev, oracle, case):
    if case == "fig5":
        tr, E = _fig5_trace("fig5_moe.txt"), 8
    elif case == "random":
        tr, E = _random_trace(21, 5, 333, 2, 8), 8
    elif case == "single_token":
        tr, E = _random_trace(22, 4, 1, 2, 8), 8
    elif case == "wide":
        tr, E = _random_trace(23, 3, 700, 8, 64, sticky=0.3), 64
    elif case == "long":
        tr, E = _random_trace(24, 3, 70000, 2, 8), 8   # several chunks per layer
    elif case == "collapsed":
        tr, E = np.tile(np.array([[6, 1]], np.int32), (2, 50, 1)), 8
    else:
        tr, E = _random_trace(25, 2, 90, 2, 8), 8
    L = tr.shape[0]
    counts = torch.full((L, E), -1, dtype=torch.int64, device=dev)
    delta = torch.full((L,), float("nan"), dtype=torch.float64, device=dev)
    mean = torch.full((1,), float("nan"), dtype=torch.float64, device=dev)
    tr_gpu = tr.copy()
    if case == "stray":
        tr_gpu[1, 7, 0] = -3   # entries outside [0, E) are ignored by the library (the oracle rejects them)
        tr_gpu[0, 3, 1] = E
    pkg.moe_delta_uniform(to_device(tr_gpu, dev), E, counts, delta, mean)
    torch.cuda.synchronize()
    r_mean, r_delta, r_counts = oracle.delta_uniform(tr, E)
    if case == "stray":
        r_counts[1, tr[1, 7, 0]] -= 1
        r_counts[0, tr[0, 3, 1]] -= 1
        assert np.array_equal(counts.cpu().numpy(), r_counts)
        return
    assert np.array_equal(counts.cpu().numpy(), r_counts)            # integer part bit-exact
    # fp64 on both sides, the same operations in the same order
    assert np.allclose(delta.cpu().numpy(), r_delta, rtol=1e-14, atol=1e-16)
    assert abs(mean.item() - r_mean) <= 1e-14 * max(r_mean, 1e-30) + 1e-16
    if case == "collapsed":
        assert mean.item() == 1.5


def test_stack_trace_feeds_the_trace_metrics(dev, oracle):
    cfg = wl.shrink(wl.CONFIGS["phone_stack"], d_model=256, d_ff=512, weight_std=0.05)
    n_layers, T = 6, 64
    layers_np = wl.make_stack_weights(cfg, n_layers)
    layers_t = [weights_to_device(w, dev) for w in layers_np]
    shape = pkg.shape_for(layers_t[0], T, cfg.top_k, pkg.MOE_BF16)
    ws = pkg.alloc_workspace(shape, dev)
    x_t = to_device(wl.make_inputs(cfg, T), dev)
    y = torch.empty_like(x_t)
    trace = torch.empty((n_layers, T, cfg.top_k), dtype=torch.int32, device=dev)
    pkg.moe_stack_forward(shape, [pkg.make_weights(w) for w in layers_t], x_t, y, trace, ws)
    ch = torch.empty(n_layers, dtype=torch.int64, device=dev)
    ld = torch.empty(n_layers, dtype=torch.int64, device=dev)
    He = torch.empty(cfg.n_experts, dtype=torch.int64, device=dev)
    H = torch.empty(1, dtype=torch.int64, device=dev)
    pkg.moe_offload_counters(trace, cfg.n_experts, ch, ld)
    pkg.moe_expert_replacements(trace, cfg.n_experts, He, H)
    torch.cuda.synchronize()
    tr = trace.cpu().numpy()
    rch, rld = oracle.offload_counters(tr, cfg.n_experts)
    rH, rHe = oracle.expert_replacements(tr, cfg.n_experts)
    assert np.array_equal(ch.cpu().numpy(), rch) and np.array_equal(ld.cpu().numpy(), rld)
    assert int(H.item()) == rH and np.array_equal(He.cpu().numpy(), rHe)
    # loads after the initial fill of k experts per layer are exactly the replacements
    assert int(rld.sum()) - n_layers * cfg.top_k == rH // 2


# ------------------------------------------------------------------------------- the paper's own shapes

@pytest.mark.parametrize("d,F,r", [
    (1440, 3840, 0),     # phone-sized MoE row of Table 1 (hidden 1440, F = 8h/3)
    (432, 1152, 0),      # wearable-sized MoE row (hidden 432)
    (1600, 4264, 800),   # phone-sized WD row: hidden 1600, rank = hidden / 2
    (400, 1064, 200),    # wearable-sized WD row
])
def test_forward_table1_shapes(dev, oracle, d, F, r):
    # widths that are not multiples of the GEMM's K tile exercise its K tail
    cfg = _cfg(name=f"t1_{d}", d=d, F=F, E=8, k=2, dtype="bf16", seed=600 + d, r=r, std=0.03)
    w_np = wl.make_layer_weights(cfg, with_bias=False)
    w_t = weights_to_device(w_np, dev)
    _forward_case(dev, oracle, cfg, 1, w_np, w_t)
    _forward_case(dev, oracle, cfg, 150, w_np, w_t)
    # a prefill batch: 512 rows per expert on average, the 256-row tiles with their K tails
    _forward_case(dev, oracle, cfg, 2048, w_np, w_t, sample=512)


@pytest.mark.parametrize("E", [2, 4, 8, 16])
@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_forward_active_and_total_expert_grid(dev, oracle, k, E):
    # the ablation grid of Sec. 3.5 (k active of 8 total; 2 active of E total), at a small width
    if k > E:
        pytest.skip("k cannot exceed E")
    cfg = _cfg(name=f"g{k}_{E}", d=256, F=384, E=E, k=k, dtype="bf16", seed=700 + 10 * k + E, std=0.05)
    w_np = wl.make_layer_weights(cfg, with_bias=False)
    w_t = weights_to_device(w_np, dev)
    _forward_case(dev, oracle, cfg, 1, w_np, w_t)
    _forward_case(dev, oracle, cfg, 70, w_np, w_t)
