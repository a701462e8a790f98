"""Shared test plumbing: widen GPU results exactly to fp64 and the error metric of the
parity bar (moving a synthetic workload to the GPU lives in ``workloads.device``)."""
from __future__ import annotations

import numpy as np


from workloads.device import DeviceWorkload, to_torch  # noqa: F401  (re-exported for the tests)


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
