"""Test-side helpers: brute-force definitions written independently of oracle.c."""
import json
import os

import numpy as np

from paper_2603_08088_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def brute_mask(parent, n):
    """Walk parent pointers from every node to the root (Section 2.4 ancestor predicate)."""
    T = len(parent)
    m = np.zeros((T, T), dtype=np.uint8)
    for k in range(n):
        cur = k
        m[k, cur] = 1
        while cur != 0:
            cur = int(parent[cur])
            m[k, cur] = 1
    return m


def path_to(parent, k):
    p = [k]
    while p[-1] != 0:
        p.append(int(parent[p[-1]]))
    return p[::-1]


def as_f64(x, dtype):
    return (synth.bf16_bits_to_f32(x) if dtype == "bf16" else x).astype(np.float64)


def random_tree(rng, T):
    par = np.zeros(T, dtype=np.int32)
    for k in range(1, T):
        par[k] = rng.integers(0, k)
    return par


def logits_from_argmax(rng, g, V):
    """Random logits whose row argmax is exactly g (unique maximum)."""
    lg = rng.standard_normal((len(g), V)).astype(np.float32)
    for n, t in enumerate(g):
        lg[n, t] = 20.0
    return lg
