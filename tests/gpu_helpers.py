"""Helpers for the GPU parity tests: host<->device marshalling of the synthetic workloads."""
import numpy as np
import torch

from paper_2603_08088_amd import api, synth

from paper_2603_08088_amd.devio import DEV, DevWorkload, bits_of, to_dev, to_host_f64  # noqa: F401


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
