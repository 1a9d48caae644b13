"""Helpers for the GPU parity tests: host<->device marshalling of the synthetic workloads."""
import numpy as np
import torch

from paper_2603_08088_amd import api, synth

DEV = "cuda:0"


def to_dev(a, dtype=None):
    """numpy -> device tensor; uint16 bf16 bit patterns become torch.bfloat16."""
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
    """device tensor -> numpy with the exact bits (bf16 -> uint16, int64 mask words -> uint64)."""
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


def gpu_attention(d: DevWorkload, bitmask, **kw):
    return api.tree_verify_attention(d.q, d.k_cache, d.v_cache, d.prefix_len, d.kt, d.vt, bitmask, d.n_nodes,
                                     P_max=d.P_max, block_table=d.block_table, **kw)


def attention_errors(out_gpu, out_ref, n_nodes):
    """(max-abs error, max scaled error, padded rows are zero).  The scaled error of an element is
    |gpu - ref| / (|ref| + rms(ref)): relative for the large elements, relative to the typical output size
    for the small ones, so a flat softmax (tiny outputs) cannot hide behind the absolute tolerance."""
    g = to_host_f64(out_gpu)
    diff = np.abs(g - out_ref)
    rms = float(np.sqrt((out_ref ** 2).mean())) if out_ref.size else 1.0
    padded_zero = True
    for b, n in enumerate(np.asarray(n_nodes)):
        padded_zero &= bool(np.all(g[b, int(n):] == 0))
    if not diff.size:
        return 0.0, 0.0, padded_zero
    return float(diff.max()), float((diff / (np.abs(out_ref) + rms)).max()), padded_zero
