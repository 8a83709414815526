"""Shared test plumbing: host arrays <-> device tensors, error measures, routing margins."""
import numpy as np
import torch

import workloads as wl


def to_device(a, dev):
    """numpy float32 / int32 / bf16-bit (uint16) array -> torch tensor on dev (bf16 for uint16)."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(dev)
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def weights_to_device(w, dev):
    return {k: to_device(v, dev) for k, v in w.items()}


def to_f64(t):
    """device tensor -> float64 numpy (exact widening)"""
    return t.detach().float().cpu().numpy().astype(np.float64)


def bits_of(t):
    """device bf16/float tensor -> the host storage array the oracle takes"""
    if t.dtype == torch.bfloat16:
        return t.detach().cpu().view(torch.int16).numpy().view(np.uint16).copy()
    return t.detach().cpu().numpy().copy()


def stored_f64(a):
    if a.dtype == np.uint16:
        a = wl.bf16_bits_to_f32(a)
    return a.astype(np.float64)


def rel_err(y, ref):
    """max of (max-abs error / max-abs ref) and (L2 error / L2 ref): the per-tensor relative
    error both tolerances (1e-4 fp32, 2e-2 bf16) are stated in."""
    y = np.asarray(y, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    den_max = max(np.abs(ref).max(), 1e-300)
    den_l2 = max(np.linalg.norm(ref), 1e-300)
    return float(max(np.abs(y - ref).max() / den_max, np.linalg.norm(y - ref) / den_l2))


def row_rel_err(y, ref):
    """Worst row: max over rows of (L2 error of the row / L2 norm of the reference row).  A wrong
    value confined to a few rows cannot hide behind the norm of the whole tensor here."""
    y = np.asarray(y, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    den = np.maximum(np.linalg.norm(ref, axis=-1), 1e-300)
    return float((np.linalg.norm(y - ref, axis=-1) / den).max())


def elementwise_rel_err(y, ref, floor=0.1):
    """Worst element-wise relative error over the elements whose reference magnitude exceeds
    `floor` times the tensor's rms (element-wise relative error means nothing near zero)."""
    y = np.asarray(y, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref * ref))
    big = np.abs(ref) > floor * rms
    if not big.any():
        return 0.0
    return float((np.abs(y - ref)[big] / np.abs(ref)[big]).max())


def ambiguous_tokens(logits, x, router_w, k):
    """Tokens whose k-th and (k+1)-th largest fp64 logits are closer than the fp32 rounding
    bound of a length-d dot product: delta = 8 d 2^-24 max|x_t| max|W_r| (any summation order).
    Routing must match exactly everywhere else."""
    T, E = logits.shape
    if k >= E:
        return np.zeros(T, bool)
    d = router_w.shape[1]
    srt = -np.sort(-logits, axis=1)
    gap = np.min(srt[:, :k] - srt[:, 1:k + 1], axis=1)  # smallest gap among ranks 0..k
    xa = np.abs(stored_f64(x)).max(axis=1)
    delta = 8.0 * d * 2.0 ** -24 * xa * np.abs(router_w).max()
    return gap < delta


def gpu_available():
    return torch.cuda.is_available()
