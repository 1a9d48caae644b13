"""Seeded synthetic workloads for the tree-verify step.

Everything here is input preparation: draft-tree shapes, candidate tokens,
per-path index tables, teacher logits with planted greedy matches, Q/K/V values
and paged-cache block tables.  None of the verification step's arithmetic lives
here; the CPU oracle and the HIP path both consume these arrays unchanged.

The shapes follow the paper's evaluation (Section 5): prompts of a few hundred
to a few thousand tokens, node budgets 16..256 and depth bounds 4..16 from the
budget sweep (Table 2), accepted draft lengths of about 3 on average (Table 1).
The paper's prompt sets and model weights are not available, so these inputs
stand in for them.

Conventions (numpy, host memory):
  parent    int32 [B, T_max]   parent[b, 0] = 0 (root row), parent[b, k] < k, padded with 0
  n_nodes   int32 [B]          number of valid node rows, root included
  tokens    int32 [B, T_max]   candidate token of each node (root: last accepted token)
  retrieve  int32 [B, L_max, W]  node indices root->leaf of every path, -1 padded
  q         [B, T_max, Hq, d]; kt, vt [B, T_max, Hkv, d]
  k_cache, v_cache: contiguous [B, P_cap, Hkv, d] or paged [num_blocks, Hkv, block, d]
  block_table int32 [B, max_blocks]; prefix_len int32 [B]; capacity int32 [B]
  logits    float32 [B, T_max, V]
bf16 tensors are carried as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 26030808 * 10
BLOCK = 16  # tokens per block of the paged prefix cache


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (storage format only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# tree shapes (parent arrays in topological order, root = 0)
# --------------------------------------------------------------------------
def tree_chain(T: int) -> np.ndarray:
    p = np.arange(-1, T - 1, dtype=np.int32)
    p[0] = 0
    return p


def tree_star(T: int) -> np.ndarray:
    return np.zeros(T, dtype=np.int32)


def tree_bfs(rng: np.random.Generator, T: int, max_depth: int, max_children: int) -> np.ndarray:
    """Breadth-first growth: every expanded node gets U{1..max_children} children until
    T nodes exist or max_depth is reached; one node of depth max_depth is forced
    (when T > max_depth) by reserving a spine."""
    assert T >= 1
    depth_goal = min(max_depth, T - 1)
    parent = [0]
    depth = [0]
    # reserve a spine so the depth bound is reached
    for dd in range(1, depth_goal + 1):
        parent.append(len(parent) - 1 if dd > 1 else 0)
        depth.append(dd)
    frontier = list(range(len(parent)))
    qi = 0
    while len(parent) < T and qi < len(frontier):
        u = frontier[qi]
        qi += 1
        if depth[u] >= max_depth:
            continue
        nch = int(rng.integers(1, max_children + 1))
        for _ in range(nch):
            if len(parent) >= T:
                break
            parent.append(u)
            depth.append(depth[u] + 1)
            frontier.append(len(parent) - 1)
    while len(parent) < T:  # budget left but nothing expandable: hang leaves on the root
        parent.append(0)
        depth.append(1)
    return _renumber_level_order(np.asarray(parent, dtype=np.int32))


def tree_eagle(rng: np.random.Generator, T: int, depth: int, topk: int = 10) -> np.ndarray:
    """Draft tree shaped like a top-k expansion pruned to a node budget: the root
    proposes ``topk`` children with seeded log-scores; at every further level the
    ``topk`` best frontier nodes each propose ``topk`` children (cumulative
    log-score = parent's + log of a Dirichlet(0.5) draw); finally the T-1
    best-scoring nodes are kept (ancestor-closed because scores fall along a
    path) and renumbered level by level."""
    par = [0]
    score = [0.0]
    dep = [0]
    frontier = [0]
    for lvl in range(1, depth + 1):
        if lvl > 1:
            frontier = sorted(frontier, key=lambda n: -score[n])[:topk]
        new_frontier = []
        for u in frontier:
            probs = rng.dirichlet(np.full(topk, 0.5))
            probs = np.maximum(probs, 1e-30)
            for c in range(topk):
                par.append(u)
                score.append(score[u] + float(np.log(probs[c])))
                dep.append(lvl)
                new_frontier.append(len(par) - 1)
        frontier = new_frontier
    order = sorted(range(1, len(par)), key=lambda n: (-score[n], n))[: T - 1]
    keep = set(order) | {0}
    for n in list(keep):  # exact ties could break closure: close it explicitly
        while n not in keep or par[n] not in keep:
            keep.add(par[n])
            n = par[n]
    kept = sorted(keep, key=lambda n: (dep[n], -score[n], n))[:T]
    remap = {n: i for i, n in enumerate(kept)}
    parent = np.zeros(len(kept), dtype=np.int32)
    for n in kept[1:]:
        parent[remap[n]] = remap[par[n]]
    return parent


def tree_spine_leaves(T: int, D: int, shallow: Optional[int] = None) -> np.ndarray:
    """One spine root..depth D, the remaining budget spent on leaf children of the
    first ``shallow`` spine nodes (default max(1, D//2)), giving many short paths."""
    D = min(D, T - 1)
    parent = [0]
    for dd in range(1, D + 1):
        parent.append(dd - 1)
    shallow = max(1, D // 2) if shallow is None else max(1, shallow)
    i = 0
    while len(parent) < T:
        parent.append(i % shallow)  # spine node i has index i
        i += 1
    return _renumber_level_order(np.asarray(parent, dtype=np.int32))


def node_depths(parent: np.ndarray) -> np.ndarray:
    d = np.zeros(len(parent), dtype=np.int32)
    for k in range(1, len(parent)):
        d[k] = d[parent[k]] + 1
    return d


def _renumber_level_order(parent: np.ndarray) -> np.ndarray:
    T = len(parent)
    dep = np.zeros(T, dtype=np.int64)
    for k in range(1, T):
        n, s = k, 0
        while n != 0:
            n = parent[n]
            s += 1
        dep[k] = s
    order = sorted(range(T), key=lambda n: (dep[n], n))
    remap = {n: i for i, n in enumerate(order)}
    out = np.zeros(T, dtype=np.int32)
    for n in order[1:]:
        out[remap[n]] = remap[parent[n]]
    return out


def build_retrieve(parent: np.ndarray, W: int) -> np.ndarray:
    """One row per leaf (ascending leaf index): node indices root -> leaf, -1 padded to W."""
    T = len(parent)
    has_child = np.zeros(T, dtype=bool)
    has_child[parent[1:]] = True
    if T == 1:
        has_child[0] = False
    rows = []
    for leaf in range(T):
        if has_child[leaf]:
            continue
        path = [leaf]
        while path[-1] != 0:
            path.append(int(parent[path[-1]]))
        path.reverse()
        assert len(path) <= W, (len(path), W)
        rows.append(path + [-1] * (W - len(path)))
    return np.asarray(rows, dtype=np.int32).reshape(len(rows), W)


def draw_tokens(rng: np.random.Generator, parent: np.ndarray, V: int) -> np.ndarray:
    """tau ~ U[0, V) with distinct tokens among siblings."""
    T = len(parent)
    tok = rng.integers(0, V, size=T).astype(np.int32)
    by_parent: Dict[int, List[int]] = {}
    for k in range(1, T):
        by_parent.setdefault(int(parent[k]), []).append(k)
    for kids in by_parent.values():
        assert len(kids) <= V
        seen = set()
        for k in kids:
            while int(tok[k]) in seen:
                tok[k] = np.int32(rng.integers(0, V))
            seen.add(int(tok[k]))
    return tok


def plant_logits(rng: np.random.Generator, logits: np.ndarray, parent: np.ndarray, tokens: np.ndarray,
                 retrieve: np.ndarray, want_depth: int, boost: float = 12.0) -> Tuple[int, int]:
    """Raise logits along one seeded root-to-leaf path so that greedy acceptance takes
    exactly ``a`` draft tokens, a = min(want_depth, path depth): the next path
    token gets +boost at each of the first a nodes, and at the a-th node a token
    carried by none of its children gets +boost.  Returns (path row, a)."""
    L = retrieve.shape[0]
    p = int(rng.integers(0, L))
    path = [int(n) for n in retrieve[p] if n >= 0]
    a = min(want_depth, len(path) - 1)
    V = logits.shape[1]
    for i in range(a):
        logits[path[i], tokens[path[i + 1]]] += boost
    stop = path[a]
    child_tokens = {int(tokens[k]) for k in range(1, len(parent)) if parent[k] == stop}
    t = int(rng.integers(0, V))
    while t in child_tokens:
        t = (t + 1) % V
    logits[stop, t] += boost
    return p, a


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    B: int
    T_max: int
    Hq: int
    Hkv: int
    d: int
    dtype: str                      # "f32" | "bf16"
    V: int
    W: int                          # retrieve width = depth bound + 1
    paged: bool
    parent: np.ndarray = None
    n_nodes: np.ndarray = None
    tokens: np.ndarray = None
    retrieve: np.ndarray = None
    n_paths: np.ndarray = None
    prefix_len: np.ndarray = None
    capacity: np.ndarray = None
    P_cap: int = 0                  # contiguous: rows per sequence
    num_blocks: int = 0
    max_blocks: int = 0
    block_table: Optional[np.ndarray] = None
    q: np.ndarray = None
    kt: np.ndarray = None
    vt: np.ndarray = None
    k_cache: np.ndarray = None
    v_cache: np.ndarray = None
    logits: Optional[np.ndarray] = None
    planted: List[Tuple[int, int]] = field(default_factory=list)

    @property
    def L_max(self) -> int:
        return self.retrieve.shape[1]


def _values(rng: np.random.Generator, shape, dtype: str, scale: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def assemble(name: str, rng: np.random.Generator, parents: List[np.ndarray], prefix_lens: List[int], *,
             Hq: int, Hkv: int, d: int, dtype: str, V: int, W: int, paged: bool,
             T_max: Optional[int] = None, spare_blocks: int = 64, want_depths: Optional[List[int]] = None,
             with_logits: bool = True, q_scale: float = 1.0, with_cache: bool = True,
             tail_room: int = 0) -> Workload:
    """Pack per-sequence trees into padded batch arrays and draw all values.  The cache has room for W more
    positions behind every prefix (the longest accepted path), or for tail_room if that is larger (a branch
    cache that holds the whole tree in place)."""
    B = len(parents)
    T_max = T_max or max(len(p) for p in parents)
    wl = Workload(name=name, B=B, T_max=T_max, Hq=Hq, Hkv=Hkv, d=d, dtype=dtype, V=V, W=W, paged=paged)
    wl.parent = np.zeros((B, T_max), dtype=np.int32)
    wl.n_nodes = np.asarray([len(p) for p in parents], dtype=np.int32)
    wl.tokens = np.zeros((B, T_max), dtype=np.int32)
    rets = [build_retrieve(p, W) for p in parents]
    L_max = max(r.shape[0] for r in rets)
    wl.retrieve = np.full((B, L_max, W), -1, dtype=np.int32)
    wl.n_paths = np.asarray([r.shape[0] for r in rets], dtype=np.int32)
    for b, p in enumerate(parents):
        wl.parent[b, : len(p)] = p
        wl.tokens[b, : len(p)] = draw_tokens(rng, p, V)
        wl.retrieve[b, : rets[b].shape[0]] = rets[b]
    wl.prefix_len = np.asarray(prefix_lens, dtype=np.int32)
    wl.q = _values(rng, (B, T_max, Hq, d), dtype, q_scale)
    wl.kt = _values(rng, (B, T_max, Hkv, d), dtype)
    wl.vt = _values(rng, (B, T_max, Hkv, d), dtype)
    if paged:
        need = [(int(P) + max(W, tail_room) + BLOCK - 1) // BLOCK for P in prefix_lens]
        wl.max_blocks = max(need)
        wl.num_blocks = sum(need) + spare_blocks
        perm = rng.permutation(wl.num_blocks).astype(np.int32)
        wl.block_table = np.zeros((B, wl.max_blocks), dtype=np.int32)
        at = 0
        for b in range(B):
            wl.block_table[b, : need[b]] = perm[at: at + need[b]]
            at += need[b]
        wl.capacity = np.asarray([n * BLOCK for n in need], dtype=np.int32)
        if with_cache:
            wl.k_cache = _values(rng, (wl.num_blocks, Hkv, BLOCK, d), dtype)
            wl.v_cache = _values(rng, (wl.num_blocks, Hkv, BLOCK, d), dtype)
    else:
        wl.P_cap = max(int(P) for P in prefix_lens) + max(W, tail_room)
        wl.capacity = np.full(B, wl.P_cap, dtype=np.int32)
        if with_cache:
            wl.k_cache = _values(rng, (B, wl.P_cap, Hkv, d), dtype)
            wl.v_cache = _values(rng, (B, wl.P_cap, Hkv, d), dtype)
    if with_logits:
        wl.logits = rng.standard_normal(size=(B, T_max, V), dtype=np.float32)
        for b, p in enumerate(parents):
            want = int(want_depths[b]) if want_depths is not None else int(rng.integers(0, W))
            wl.planted.append(plant_logits(rng, wl.logits[b], p, wl.tokens[b], rets[b], want))
    return wl


def config1(seed_offset: int = 0, **kw) -> Workload:
    """Tiny CPU-seconds case: B=1, 4/4 heads, d=64, fp32, P=128, 15-node tree of depth 4."""
    rng = np.random.default_rng(BASE_SEED + 1 + 1000 * seed_offset)
    par = tree_bfs(rng, 15, 4, 3)
    return assemble("c1_tiny", rng, [par], [128], Hq=4, Hkv=4, d=64, dtype="f32", V=1000, W=5, paged=False, **kw)


def config2(paged: bool = False, seed_offset: int = 0, P: int = 2048, **kw) -> Workload:
    """7B-class GQA verify step: B=1, 32/8 heads, d=128, bf16, P=2048, 60-node top-k tree."""
    rng = np.random.default_rng(BASE_SEED + 2 + 1000 * seed_offset)
    par = tree_eagle(rng, 60, 6, 10)
    return assemble("c2_7b_gqa" + ("_paged" if paged else ""), rng, [par], [P], Hq=32, Hkv=8, d=128,
                    dtype="bf16", V=32000, W=7, paged=paged, **kw)


def config3(seed_offset: int = 0, B: int = 8, lo: int = 512, hi: int = 8192, **kw) -> Workload:
    """Ragged batch: 8 sequences, prefix ~ U[512, 8192], paged cache with a shuffled block table."""
    rng = np.random.default_rng(BASE_SEED + 3 + 1000 * seed_offset)
    parents = [tree_eagle(np.random.default_rng(BASE_SEED + 3 + 1000 * seed_offset + 7 * (b + 1)), 60, 6, 10)
               for b in range(B)]
    P = [int(x) for x in rng.integers(lo, hi + 1, size=B)]
    return assemble("c3_ragged", rng, parents, P, Hq=32, Hkv=8, d=128, dtype="bf16", V=32000, W=7,
                    paged=True, T_max=60, **kw)


def config4(paged: bool = False, seed_offset: int = 0, P: int = 32768, **kw) -> Workload:
    """Long context: B=1, P=32768, 128-node tree of depth 8, branching up to 4."""
    rng = np.random.default_rng(BASE_SEED + 4 + 1000 * seed_offset)
    par = tree_bfs(rng, 128, 8, 4)
    return assemble("c4_long" + ("_paged" if paged else ""), rng, [par], [P], Hq=32, Hkv=8, d=128,
                    dtype="bf16", V=32000, W=9, paged=paged, **kw)


def config5(T: int, D: int, B: int = 32, P: int = 4096, seed_offset: int = 0, **kw) -> Workload:
    """Budget-sweep cell, padding-heavy: B=32, P=4096 paged, spine + many short leaves."""
    rng = np.random.default_rng(BASE_SEED + 5 + 1000 * seed_offset + 17 * T + D)
    Dc = min(D, T - 1)
    # widest leaf attachment that still leaves at least half of the path table as padding
    # (not attainable at T=8, where the spine dominates: the shallowest attachment is used)
    for shallow in range(max(1, Dc // 2), 0, -1):
        par = tree_spine_leaves(T, Dc, shallow)
        if padding_fraction(build_retrieve(par, Dc + 1)) >= 0.5:
            break
    wl = assemble(f"c5_T{T}_D{Dc}", rng, [par.copy() for _ in range(B)], [P] * B, Hq=32, Hkv=8, d=128,
                  dtype="bf16", V=32000, W=Dc + 1, paged=True, **kw)
    return wl


def padding_fraction(retrieve: np.ndarray) -> float:
    return float((retrieve < 0).mean())
