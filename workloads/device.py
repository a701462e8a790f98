"""Device-resident copies of generated workloads (torch is used for device memory only)."""
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
