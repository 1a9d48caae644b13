"""Host <-> device marshalling of the synthetic workloads (numpy arrays <-> torch device tensors).

Plumbing only: no arithmetic of the verification step.  Used by the benchmark, the smoke run and the GPU tests.
"""
from __future__ import annotations

import numpy as np
import torch

from . import synth

DEV = "cuda:0"


def to_dev(a, dtype=None):
    """numpy -> device tensor; uint16 bf16 bit patterns become torch.bfloat16, uint64 mask words int64."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if dtype == "bf16" or a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def to_host_f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


def bits_of(t):
    """device tensor -> numpy with the exact bits (bf16 -> uint16)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class DevWorkload:
    """Device copies of a synth.Workload (same names)."""

    def __init__(self, wl: synth.Workload):
        self.wl = wl
        for name in ("parent", "n_nodes", "tokens", "retrieve", "prefix_len", "capacity", "block_table", "q", "kt",
                     "vt", "k_cache", "v_cache", "logits"):
            setattr(self, name, to_dev(getattr(wl, name)))
        self.P_max = int(wl.prefix_len.max()) if wl.B else 0
