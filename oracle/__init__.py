"""ctypes wrapper around the CPU oracle (``oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  Nothing on the product path
may import this package, and this package imports nothing from the HIP side.

Every function takes and returns numpy arrays in host memory; bf16 tensors are
uint16 bit patterns (dtype "bf16"), fp32 tensors are float32 (dtype "f32").
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRC = os.path.join(_HERE, "oracle.c")
_lib = None

TREE_RANGE, TREE_CYCLE, TREE_CLOSURE = 1, 2, 4
COMMIT_CAPACITY, COMMIT_BAD_NODE, COMMIT_BAD_LEN, COMMIT_BAD_BLOCK = 1, 2, 4, 8
BRANCH_NO_BLOCKS, BRANCH_BAD_FREE = 16, 32


def build(force: bool = True) -> str:
    """Compile oracle.c with gcc (-O2, OpenMP, no fast-math) into liboracle.so."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_SO)
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _dt(dtype: str) -> int:
    return {"f32": 0, "bf16": 1}[dtype]


def num_threads() -> int:
    return int(lib().orc_num_threads())


def build_tree_mask(parent, n_nodes):
    parent, n_nodes = _i32(parent), _i32(n_nodes)
    B, T = parent.shape
    words = (T + 63) // 64
    bitmask = np.zeros((B, T, words), dtype=np.uint64)
    dense = np.zeros((B, 1, T, T), dtype=np.uint8)
    depth = np.zeros((B, T), dtype=np.int32)
    status = np.zeros(B, dtype=np.int32)
    rc = lib().orc_build_tree_mask(_p(parent), _p(n_nodes), B, T, _p(bitmask), _p(dense), _p(depth), _p(status))
    assert rc == 0, rc
    return dict(bitmask=bitmask, dense=dense, depth=depth, status=status)


def tensorize_tree(parent, n_nodes, prefix_len, L_max: int, W: int):
    """depth, position ids, root-to-leaf paths (retrieve [B,L_max,W], -1 padded), path counts, status."""
    parent, n_nodes, prefix_len = _i32(parent), _i32(n_nodes), _i32(prefix_len)
    B, T = parent.shape
    depth = np.zeros((B, T), dtype=np.int32)
    pos = np.zeros((B, T), dtype=np.int32)
    retrieve = np.zeros((B, L_max, W), dtype=np.int32)
    n_paths = np.zeros(B, dtype=np.int32)
    status = np.zeros(B, dtype=np.int32)
    rc = lib().orc_tensorize_tree(_p(parent), _p(n_nodes), _p(prefix_len), B, T, L_max, W, _p(depth), _p(pos),
                                  _p(retrieve), _p(n_paths), _p(status))
    assert rc == 0, rc
    return dict(depth=depth, position_ids=pos, retrieve=retrieve, n_paths=n_paths, status=status)


def lm_head_argmax(hidden, weight, n_nodes, *, dtype: str, want_logits: bool = False):
    """hidden [B,T,D], weight [V,D] -> argmax int32 [B,T] (lowest index on ties, -1 for padding), max logit
    float64 [B,T], and the fp64 logits [B,T,V] on request."""
    B, T, D = hidden.shape
    V = weight.shape[0]
    argmax = np.zeros((B, T), dtype=np.int32)
    maxval = np.zeros((B, T), dtype=np.float64)
    logits = np.zeros((B, T, V), dtype=np.float64) if want_logits else None
    f = lib().orc_lm_head_argmax
    f.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p] + [C.c_int] * 4 + [C.c_void_p] * 3
    rc = f(_p(np.ascontiguousarray(hidden)), _p(np.ascontiguousarray(weight)), _dt(dtype), _p(_i32(n_nodes)), B, T, D,
           V, _p(argmax), _p(maxval), _p(logits))
    assert rc == 0, rc
    return dict(argmax=argmax, maxval=maxval, logits=logits)


def tree_verify_attention(q, k_cache, v_cache, prefix_len, kt, vt, dense, n_nodes, *, dtype: str,
                          block_table=None, scale: float = 0.0, want_lse: bool = True):
    """q [B,T,Hq,d]; kt/vt [B,T,Hkv,d]; cache contiguous [B,P_cap,Hkv,d] or paged [nb,Hkv,bs,d]."""
    B, T, Hq, d = q.shape
    Hkv = kt.shape[2]
    if block_table is not None:
        block_table = _i32(block_table)
        bs, max_blocks, P_cap = k_cache.shape[2], block_table.shape[1], 0
    else:
        bs, max_blocks, P_cap = 0, 0, k_cache.shape[1]
    out = np.zeros((B, T, Hq, d), dtype=np.float64)
    lse = np.zeros((B, Hq, T), dtype=np.float64) if want_lse else None
    f = lib().orc_tree_verify_attention
    f.argtypes = [C.c_int] * 6 + [C.c_void_p] * 4 + [C.c_int] * 3 + [C.c_void_p] * 5 + [C.c_double] + [C.c_void_p] * 2
    rc = f(B, T, Hq, Hkv, d, _dt(dtype), _p(q), _p(k_cache), _p(v_cache), _p(block_table), bs, max_blocks, P_cap,
           _p(_i32(prefix_len)), _p(kt), _p(vt), _p(np.ascontiguousarray(dense, dtype=np.uint8)), _p(_i32(n_nodes)),
           float(scale), _p(out), _p(lse))
    assert rc == 0, rc
    return out, lse


def safe_gather_paths(retrieve, n_nodes, T_max: int, dummy: int = 0, src: Optional[np.ndarray] = None):
    """src [B,T_max,...] of any dtype; returns safe, pvalid and (if src) gathered [B,L,W,...]."""
    retrieve = _i32(retrieve)
    B, L, W = retrieve.shape
    safe = np.zeros((B, L, W), dtype=np.int32)
    pvalid = np.zeros((B, L, W), dtype=np.uint8)
    gathered, row_bytes = None, 0
    if src is not None:
        src = np.ascontiguousarray(src)
        assert src.shape[0] == B and src.shape[1] == T_max
        row_bytes = src.nbytes // (B * T_max)
        gathered = np.zeros((B, L, W) + src.shape[2:], dtype=src.dtype)
    f = lib().orc_safe_gather_paths
    f.argtypes = [C.c_void_p, C.c_void_p] + [C.c_int] * 5 + [C.c_void_p, C.c_size_t] + [C.c_void_p] * 3
    rc = f(_p(retrieve), _p(_i32(n_nodes)) if n_nodes is not None else None, B, L, W, T_max, dummy, _p(src),
           row_bytes, _p(safe), _p(pvalid), _p(gathered))
    if rc != 0:
        raise ValueError(f"orc_safe_gather_paths rc={rc}")
    return dict(safe=safe, pvalid=pvalid, gathered=gathered)


def evaluate_posterior(logits, tokens, retrieve, n_nodes, dummy: int = 0):
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    tokens, retrieve, n_nodes = _i32(tokens), _i32(retrieve), _i32(n_nodes)
    B, T, V = logits.shape
    _, L, W = retrieve.shape
    g = np.zeros((B, T), dtype=np.int32)
    ln = np.zeros((B, L), dtype=np.int32)
    best = np.zeros(B, dtype=np.int32)
    A = np.zeros(B, dtype=np.int32)
    acc = np.zeros((B, W), dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    rc = lib().orc_evaluate_posterior(_p(logits), _p(tokens), _p(retrieve), _p(n_nodes), B, T, V, L, W, dummy,
                                      _p(g), _p(ln), _p(best), _p(A), _p(acc), _p(bonus))
    if rc != 0:
        raise ValueError(f"orc_evaluate_posterior rc={rc}")
    return dict(argmax=g, len=ln, best=best, accept_len=A, acc_nodes=acc, bonus=bonus)


def commit_accepted_kv(kt, vt, k_cache, v_cache, prefix_len, capacity, n_nodes, acc_nodes, accept_len, *,
                       block_table=None, T_max=None):
    """kt/vt [Lyr,B,T,Hkv,d]; caches [Lyr, ...] (contiguous [B,P_cap,Hkv,d] or paged [nb,Hkv,bs,d]).
    kt = vt = None (with T_max): the tree rows sit in the cache itself at positions prefix_len + node.
    Caches are updated IN PLACE; returns prefix_len_out, slot_map, status."""
    assert k_cache.flags["C_CONTIGUOUS"] and v_cache.flags["C_CONTIGUOUS"]
    if kt is not None:
        Lyr, B, T, Hkv, d = kt.shape
        eb = kt.dtype.itemsize
    else:
        Lyr, B, T, eb = k_cache.shape[0], len(prefix_len), int(T_max), k_cache.dtype.itemsize
        Hkv, d = (k_cache.shape[2], k_cache.shape[4]) if block_table is not None else (k_cache.shape[3], k_cache.shape[4])
    assert k_cache.shape[0] == Lyr
    layer_stride = int(np.prod(k_cache.shape[1:]))
    if block_table is not None:
        block_table = _i32(block_table)
        bs, max_blocks, nb, P_cap = k_cache.shape[3], block_table.shape[1], k_cache.shape[1], 0
    else:
        bs, max_blocks, nb, P_cap = 0, 0, 0, k_cache.shape[2]
    acc_nodes = _i32(acc_nodes)
    W = acc_nodes.shape[1]
    plo = np.zeros(B, dtype=np.int32)
    slot = np.zeros((B, W), dtype=np.int32)
    st = np.zeros(B, dtype=np.int32)
    f = lib().orc_commit_accepted_kv
    f.argtypes = ([C.c_int] * 6 + [C.c_void_p] * 4 + [C.c_size_t, C.c_void_p] + [C.c_int] * 4 + [C.c_void_p] * 5
                  + [C.c_int] + [C.c_void_p] * 3)
    rc = f(B, T, Hkv, d, eb, Lyr, _p(kt), _p(vt), _p(k_cache), _p(v_cache), layer_stride, _p(block_table), bs,
           max_blocks, nb, P_cap, _p(_i32(prefix_len)), _p(_i32(capacity)), _p(_i32(n_nodes)), _p(acc_nodes),
           _p(_i32(accept_len)), W, _p(plo), _p(slot), _p(st))
    assert rc == 0, rc
    return dict(prefix_len_out=plo, slot_map=slot, status=st)


def replicate_branches(k_cache, v_cache, block_table, prefix_len, tail_len, N: int, free_blocks):
    """Paged caches [Lyr, nb, Hkv, bs, d] (the partly filled blocks are copied IN PLACE into the branches' own
    blocks); returns branch_table [B, N, max_blocks], block_base [B], n_taken, status [B]."""
    assert k_cache.flags["C_CONTIGUOUS"] and v_cache.flags["C_CONTIGUOUS"]
    Lyr, nb, Hkv, bs, d = k_cache.shape
    block_table, free_blocks = _i32(block_table), _i32(free_blocks)
    B, max_blocks = block_table.shape
    bt = np.zeros((B, N, max_blocks), dtype=np.int32)
    base = np.zeros(B, dtype=np.int32)
    taken = np.zeros(1, dtype=np.int32)
    st = np.zeros(B, dtype=np.int32)
    f = lib().orc_replicate_branches
    f.argtypes = ([C.c_int] * 6 + [C.c_void_p] * 2 + [C.c_size_t, C.c_void_p] + [C.c_int] * 3 + [C.c_void_p] * 3
                  + [C.c_int] + [C.c_void_p] * 4)
    rc = f(B, N, Hkv, d, k_cache.dtype.itemsize, Lyr, _p(k_cache), _p(v_cache), int(np.prod(k_cache.shape[1:])),
           _p(block_table), bs, max_blocks, nb, _p(_i32(prefix_len)), _p(_i32(tail_len)), _p(free_blocks),
           len(free_blocks), _p(bt), _p(base), _p(taken), _p(st))
    assert rc == 0, rc
    return dict(branch_table=bt, block_base=base, n_taken=int(taken[0]), status=st)


def commit_path_indices(src_k, src_v, dst_k, dst_v, path_indices, src_len, new_len, *, src_table=None,
                        dst_table=None, fast: bool = False):
    """Caches [Lyr, ...]: contiguous [B, P_cap, Hkv, d] (source and destination are different arrays) or paged
    [nb, Hkv, bs, d] (one pool may serve as both; dst_table is then updated IN PLACE with the shared blocks).
    The destination cache is written IN PLACE; returns kept_len, status."""
    for a in (src_k, src_v, dst_k, dst_v):
        assert a.flags["C_CONTIGUOUS"]
    assert src_k.shape == dst_k.shape
    path_indices = _i32(path_indices)
    B, L_cap = path_indices.shape
    Lyr, eb = src_k.shape[0], src_k.dtype.itemsize
    if src_table is not None:
        src_table = _i32(src_table)
        assert dst_table.dtype == np.int32 and dst_table.flags["C_CONTIGUOUS"] and dst_table.shape == src_table.shape
        nb, Hkv, bs, d = src_k.shape[1:]
        max_blocks, P_cap = src_table.shape[1], 0
    else:
        P_cap, Hkv, d = src_k.shape[2:]
        nb = bs = max_blocks = 0
    kept = np.zeros(B, dtype=np.int32)
    st = np.zeros(B, dtype=np.int32)
    f = lib().orc_commit_path_indices
    f.argtypes = ([C.c_int] * 5 + [C.c_void_p] * 4 + [C.c_size_t] + [C.c_void_p] * 2 + [C.c_int] * 4 + [C.c_void_p]
                  + [C.c_int] + [C.c_void_p] * 2 + [C.c_int] + [C.c_void_p] * 2)
    rc = f(B, Hkv, d, eb, Lyr, _p(src_k), _p(src_v), _p(dst_k), _p(dst_v), int(np.prod(src_k.shape[1:])),
           _p(src_table), _p(dst_table), bs, max_blocks, nb, P_cap, _p(path_indices), L_cap, _p(_i32(src_len)),
           _p(_i32(new_len)), int(fast), _p(kept), _p(st))
    assert rc == 0, rc
    return dict(kept_len=kept, status=st)
