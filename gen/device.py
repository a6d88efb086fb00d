"""Move a Workload's numpy tensors onto a torch device in the workload's storage dtype (data plumbing only)."""
from __future__ import annotations

import numpy as np
import torch

from .workloads import Workload, bf16_bits


def _to(x: np.ndarray, dtype: str, device) -> torch.Tensor:
    if dtype == "bf16":
        bits = torch.from_numpy(bf16_bits(x).view(np.int16))
        return bits.to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device)


def to_torch(w: Workload, device="cuda:0") -> dict:
    """Returns {"q","k","v","kc","vc"} tensors plus "kv_lens"/"budgets" int32 tensors on `device`."""
    out = {n: _to(getattr(w, a), w.dtype, device)
           for n, a in (("q", "Q"), ("k", "K"), ("v", "V"), ("kc", "Kc"), ("vc", "Vc"))}
    out["kv_lens"] = torch.tensor(w.kv_lens, dtype=torch.int32, device=device)
    out["budgets"] = torch.tensor(w.budgets, dtype=torch.int32, device=device)
    return out


def from_torch(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float64 / int64 numpy (exact for bf16, fp32 and int32 contents)."""
    if t.dtype in (torch.int32, torch.int64):
        return t.detach().cpu().numpy().astype(np.int64)
    return t.detach().float().cpu().numpy().astype(np.float64)
