"""Shared test plumbing: move a synthetic workload to the GPU, widen GPU
results exactly to fp64, and the error metric of the parity bar."""
from __future__ import annotations

import numpy as np


def to_torch(a: np.ndarray, kind: str, device="cuda"):
    """numpy storage array -> torch tensor (bf16 bits are re-viewed, not converted)."""
    import torch
    if kind == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


class DeviceWorkload:
    """Device-resident copy of a synth.Workload."""

    def __init__(self, w, device="cuda"):
        self.w = w
        io = w.io_dtype
        self.q_nope = to_torch(w.q_nope, io, device)
        self.q_rope = to_torch(w.q_rope, io, device)
        self.W_UK = to_torch(w.W_UK, io, device)
        self.W_UV = to_torch(w.W_UV, io, device)
        ck = "bf16" if w.cache_dtype == "bf16" else w.cache_dtype
        self.pool = to_torch(w.pool, ck, device)
        self.kv_scale = None if w.kv_scale is None else to_torch(w.kv_scale, "f32", device)
        self.page_table = to_torch(w.page_table, "i32", device)
        self.seq_lens = to_torch(w.seq_lens, "i32", device)


def widen_gpu(t) -> np.ndarray:
    """GPU tensor (fp32 / bf16) -> float64 numpy, exactly."""
    import torch
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).numpy().view(np.uint16)
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return t.double().numpy()


def storage_bits(t) -> np.ndarray:
    """GPU tensor -> numpy array of its storage words (for bit-exact comparisons)."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy().view(np.uint32)
    return t.numpy()


def max_abs_rel(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| over the tensor (the parity metric)."""
    denom = float(np.abs(ref).max())
    if denom == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / denom)


def lse_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max abs error of the log-sum-exp where it is finite; -inf must match exactly."""
    inf = np.isneginf(ref)
    assert (np.isneginf(got) == inf).all(), "lse -inf pattern differs"
    if inf.all():
        return 0.0
    return float(np.abs(got[~inf] - ref[~inf]).max())


TOL = {"f32": 1e-5, "bf16": 2e-2}
