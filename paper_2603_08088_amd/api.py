"""Thin Python binding of libeagletv.so: argument marshalling only.

Each function has the name of the C entry point it calls (``include/eagletv.h``)
and takes torch tensors that already live on the GPU; outputs are allocated
with ``torch.empty`` unless passed in.  No step of the verification path runs
in Python or in torch ops.  The library must have been built
(``python -m paper_2603_08088_amd.build``); loading fails loudly otherwise -
there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libeagletv.so")
_lib = None

F32, BF16 = 0, 1
TREE_RANGE, TREE_CYCLE, TREE_CLOSURE = 1, 2, 4
COMMIT_CAPACITY, COMMIT_BAD_NODE, COMMIT_BAD_LEN, COMMIT_BAD_BLOCK = 1, 2, 4, 8
BRANCH_NO_BLOCKS, BRANCH_BAD_FREE = 16, 32
ATTN_FLAG_GENERIC = 1
ATTN_FLAG_SMALL_WG = 2
ATTN_FLAG_WHOLE_TILE = 4
ATTN_FLAG_KEY_HALVES = 8
ATTN_FLAG_LARGE_WG = 16
ATTN_FLAG_UNIFORM_SPLITS = 32
MAX_TREE, ATTN_MAX_TREE = 256, 256
ATTN_STATIC_WORKSPACE_BYTES = 64 << 20

EXPORTS = ("etv_status_string", "etv_version", "etv_last_hip_error", "etv_build_tree_mask",
           "etv_tensorize_tree",
           "etv_tree_verify_attention_workspace_bytes", "etv_tree_verify_attention_plan", "etv_tree_verify_attention",
           "etv_tree_verify_attention_static", "etv_safe_gather_paths",
           "etv_evaluate_posterior_workspace_bytes", "etv_evaluate_posterior", "etv_commit_accepted_kv",
           "etv_verify_epilogue", "etv_lm_head_argmax_workspace_bytes", "etv_lm_head_argmax",
           "etv_lm_head_packed_bytes", "etv_pack_lm_head", "etv_replicate_branches", "etv_commit_path_indices")


class AttnDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "T_max", "Hq", "Hkv", "d", "dtype", "block_size", "max_blocks",
                                         "num_blocks", "P_cap", "P_max")] + \
               [("scale", C.c_float), ("kv_split", C.c_int32), ("flags", C.c_int32)]


class AttnPlan(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("mfma", "wavefronts", "key_halves", "ring_stages", "row_groups", "kv_split",
                                         "n_splits", "balanced_splits")] + [("workgroups", C.c_int64)]


class CommitDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "T_max", "Hkv", "d", "elem_bytes", "n_layers", "W", "block_size",
                                         "max_blocks", "num_blocks", "P_cap", "reserved")] + \
               [("cache_layer_stride", C.c_int64)]


class CacheDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hkv", "d", "elem_bytes", "n_layers", "block_size", "max_blocks",
                                         "num_blocks", "P_cap", "reserved")] + [("cache_layer_stride", C.c_int64)]


class EtvError(RuntimeError):
    def __init__(self, fn: str, rc: int):
        l = lib()
        msg = l.etv_status_string(rc).decode()
        super().__init__(f"{fn}: {msg} (rc={rc}, hip={l.etv_last_hip_error()})")
        self.rc = rc


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_08088_amd.build` "
                               "(there is no fallback path)")
        l = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        l.etv_status_string.restype = C.c_char_p
        l.etv_status_string.argtypes = [i32]
        l.etv_version.restype = C.c_char_p
        l.etv_last_hip_error.restype = i32
        l.etv_build_tree_mask.restype = i32
        l.etv_build_tree_mask.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp]
        l.etv_tensorize_tree.restype = i32
        l.etv_tensorize_tree.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        l.etv_tree_verify_attention_workspace_bytes.restype = sz
        l.etv_tree_verify_attention_workspace_bytes.argtypes = [C.POINTER(AttnDesc)]
        l.etv_tree_verify_attention_plan.restype = i32
        l.etv_tree_verify_attention_plan.argtypes = [C.POINTER(AttnDesc), C.POINTER(AttnPlan)]
        l.etv_tree_verify_attention.restype = i32
        l.etv_tree_verify_attention.argtypes = [C.POINTER(AttnDesc)] + [vp] * 12 + [sz, vp]
        l.etv_tree_verify_attention_static.restype = i32
        l.etv_tree_verify_attention_static.argtypes = [C.POINTER(AttnDesc)] + [vp] * 12
        l.etv_safe_gather_paths.restype = i32
        l.etv_safe_gather_paths.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, sz, vp, vp, vp, vp]
        l.etv_lm_head_argmax_workspace_bytes.restype = sz
        l.etv_lm_head_argmax_workspace_bytes.argtypes = [i32, i32, i32]
        l.etv_lm_head_argmax.restype = i32
        l.etv_lm_head_argmax.argtypes = [vp, vp, i32, vp, i32, i32, i32, i32, vp, vp, vp, sz, vp]
        l.etv_lm_head_packed_bytes.restype = sz
        l.etv_lm_head_packed_bytes.argtypes = [i32, i32]
        l.etv_pack_lm_head.restype = i32
        l.etv_pack_lm_head.argtypes = [vp, i32, i32, vp, vp]
        l.etv_verify_epilogue.restype = i32
        l.etv_verify_epilogue.argtypes = [C.POINTER(CommitDesc), vp, i32, vp, vp, i32, i32, vp, sz] + [vp] * 21 + [sz, vp]
        l.etv_evaluate_posterior_workspace_bytes.restype = sz
        l.etv_evaluate_posterior_workspace_bytes.argtypes = [i32, i32, i32]
        l.etv_evaluate_posterior.restype = i32
        l.etv_evaluate_posterior.argtypes = [vp] * 4 + [i32] * 6 + [vp] * 7 + [sz, vp]
        l.etv_commit_accepted_kv.restype = i32
        l.etv_commit_accepted_kv.argtypes = [C.POINTER(CommitDesc)] + [vp] * 14
        l.etv_replicate_branches.restype = i32
        l.etv_replicate_branches.argtypes = [C.POINTER(CacheDesc)] + [vp] * 5 + [i32, vp, i32] + [vp] * 5
        l.etv_commit_path_indices.restype = i32
        l.etv_commit_path_indices.argtypes = [C.POINTER(CacheDesc)] + [vp] * 7 + [i32, vp, vp, i32, vp, vp, vp]
        _lib = l
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(fn: str, rc: int):
    if rc != 0:
        raise EtvError(fn, rc)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise EtvError("dtype", -2)


# ------------------------------------------------------------------------------------------------
def build_tree_mask(parent: torch.Tensor, n_nodes: torch.Tensor, *, want_dense: bool = True,
                    want_depth: bool = True, out: Optional[Dict[str, torch.Tensor]] = None):
    """parent int32 [B,T_max], n_nodes int32 [B] -> bitmask u64-as-int64 [B,T_max,words], dense u8
    [B,1,T_max,T_max], depth int32 [B,T_max], status int32 [B]."""
    B, T = parent.shape
    dev = parent.device
    words = (T + 63) // 64
    o = out or {}
    bitmask = o.get("bitmask", None)
    if bitmask is None:
        bitmask = torch.empty((B, T, words), dtype=torch.int64, device=dev)
    dense = o.get("dense") if out else (torch.empty((B, 1, T, T), dtype=torch.uint8, device=dev) if want_dense else None)
    depth = o.get("depth") if out else (torch.empty((B, T), dtype=torch.int32, device=dev) if want_depth else None)
    status = o.get("status") if out else None
    if status is None:
        status = torch.empty((B,), dtype=torch.int32, device=dev)
    rc = lib().etv_build_tree_mask(_ptr(parent), _ptr(n_nodes), B, T, _ptr(bitmask), _ptr(dense), _ptr(depth),
                                   _ptr(status), _stream())
    _check("etv_build_tree_mask", rc)
    return dict(bitmask=bitmask, dense=dense, depth=depth, status=status)


def tensorize_tree(parent: torch.Tensor, n_nodes: torch.Tensor, prefix_len: torch.Tensor, L_max: int, W: int, *,
                   want_dense: bool = True, out: Optional[Dict[str, torch.Tensor]] = None):
    """parent int32 [B,T_max], n_nodes, prefix_len int32 [B] -> the outputs of build_tree_mask plus position_ids
    int32 [B,T_max], retrieve int32 [B,L_max,W] (root-to-leaf paths, -1 padded) and n_paths int32 [B]."""
    B, T = parent.shape
    dev = parent.device
    words = (T + 63) // 64
    o = out or {}
    i32 = dict(dtype=torch.int32, device=dev)

    def get(name, shape, dtype=torch.int32):
        t = o.get(name)
        return t if t is not None else torch.empty(shape, dtype=dtype, device=dev)
    bitmask = get("bitmask", (B, T, words), torch.int64)
    dense = o.get("dense") if out else (torch.empty((B, 1, T, T), dtype=torch.uint8, device=dev) if want_dense else None)
    depth, pos = get("depth", (B, T)), get("position_ids", (B, T))
    retrieve, n_paths, status = get("retrieve", (B, L_max, W)), get("n_paths", (B,)), get("status", (B,))
    rc = lib().etv_tensorize_tree(_ptr(parent), _ptr(n_nodes), _ptr(prefix_len), B, T, L_max, W, _ptr(bitmask),
                                  _ptr(dense), _ptr(depth), _ptr(pos), _ptr(retrieve), _ptr(n_paths), _ptr(status),
                                  _stream())
    _check("etv_tensorize_tree", rc)
    return dict(bitmask=bitmask, dense=dense, depth=depth, position_ids=pos, retrieve=retrieve, n_paths=n_paths,
                status=status)


def attn_desc(q: torch.Tensor, kt: torch.Tensor, k_cache: Optional[torch.Tensor], block_table: Optional[torch.Tensor],
              P_max: int, scale: float = 0.0, kv_split: int = 0, flags: int = 0) -> AttnDesc:
    B, T, Hq, d = q.shape
    # kt None: in-place branch cache, the tree rows are in k_cache / v_cache behind the prefix
    Hkv = kt.shape[2] if kt is not None else (k_cache.shape[1] if block_table is not None else k_cache.shape[2])
    dsc = AttnDesc(B=B, T_max=T, Hq=Hq, Hkv=Hkv, d=d, dtype=_dtype_code(q), block_size=0, max_blocks=0,
                   num_blocks=0, P_cap=0, P_max=int(P_max), scale=float(scale), kv_split=int(kv_split),
                   flags=int(flags))
    if block_table is not None:
        dsc.block_size = k_cache.shape[2]
        dsc.max_blocks = block_table.shape[1]
        dsc.num_blocks = k_cache.shape[0]
    elif k_cache is not None:
        dsc.P_cap = k_cache.shape[1]
    return dsc


def tree_verify_attention_workspace_bytes(dsc: AttnDesc) -> int:
    return int(lib().etv_tree_verify_attention_workspace_bytes(C.byref(dsc)))


def tree_verify_attention_plan(dsc: AttnDesc) -> Dict[str, int]:
    """The launch shape the library picks for this descriptor (host only)."""
    pl = AttnPlan()
    _check("etv_tree_verify_attention_plan", lib().etv_tree_verify_attention_plan(C.byref(dsc), C.byref(pl)))
    return {n: int(getattr(pl, n)) for n, _ in AttnPlan._fields_ if n != "reserved"}


def tree_verify_attention(q, k_cache, v_cache, prefix_len, kt, vt, bitmask, n_nodes, *, P_max: int,
                          block_table=None, scale: float = 0.0, kv_split: int = 0, flags: int = 0,
                          out=None, lse=None, want_lse: bool = True, workspace=None, desc: Optional[AttnDesc] = None):
    """q [B,T,Hq,d]; kt/vt [B,T,Hkv,d]; cache contiguous [B,P_cap,Hkv,d] or paged [nb,Hkv,16,d] + block_table.
    Returns (out [B,T,Hq,d] in q's dtype, lse float32 [B,Hq,T] or None)."""
    dsc = desc or attn_desc(q, kt, k_cache, block_table, P_max, scale, kv_split, flags)
    B, T, Hq, d = q.shape
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((B, Hq, T), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty((max(256, tree_verify_attention_workspace_bytes(dsc)),), dtype=torch.uint8,
                                device=q.device)
    rc = lib().etv_tree_verify_attention(C.byref(dsc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                         _ptr(prefix_len), _ptr(kt), _ptr(vt), _ptr(bitmask), _ptr(n_nodes),
                                         _ptr(out), _ptr(lse), _ptr(workspace), workspace.numel(), _stream())
    _check("etv_tree_verify_attention", rc)
    return out, lse


def tree_verify_attention_static(q, k_cache, v_cache, prefix_len, kt, vt, bitmask, n_nodes, out, lse=None, *,
                                 P_max: int, block_table=None, scale: float = 0.0, kv_split: int = 0, flags: int = 0,
                                 desc: Optional[AttnDesc] = None):
    """tree_verify_attention with the split partials in the library's own fixed device array: the caller passes
    every input and output (`out`, optionally `lse`) and nothing is allocated, here or in the library."""
    dsc = desc or attn_desc(q, kt, k_cache, block_table, P_max, scale, kv_split, flags)
    rc = lib().etv_tree_verify_attention_static(C.byref(dsc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                                _ptr(block_table), _ptr(prefix_len), _ptr(kt), _ptr(vt),
                                                _ptr(bitmask), _ptr(n_nodes), _ptr(out), _ptr(lse), _stream())
    _check("etv_tree_verify_attention_static", rc)
    return out, lse


def safe_gather_paths(retrieve, n_nodes, T_max: int, dummy: int = 0, src: Optional[torch.Tensor] = None,
                      out: Optional[Dict[str, torch.Tensor]] = None):
    """retrieve int32 [B,L,W]; src [B,T_max,...] any dtype -> safe int32, pvalid u8, gathered [B,L,W,...]."""
    B, L, W = retrieve.shape
    dev = retrieve.device
    o = out or {}
    safe = o.get("safe") if out else torch.empty((B, L, W), dtype=torch.int32, device=dev)
    pvalid = o.get("pvalid") if out else torch.empty((B, L, W), dtype=torch.uint8, device=dev)
    gathered, row_bytes = None, 0
    if src is not None:
        assert src.shape[0] == B and src.shape[1] == T_max
        row_bytes = src.element_size() * (src.numel() // max(1, B * T_max))
        gathered = o.get("gathered") if out else None
        if gathered is None:
            gathered = torch.empty((B, L, W) + tuple(src.shape[2:]), dtype=src.dtype, device=dev)
    rc = lib().etv_safe_gather_paths(_ptr(retrieve), _ptr(n_nodes), B, L, W, T_max, dummy, _ptr(src), row_bytes,
                                     _ptr(safe), _ptr(pvalid), _ptr(gathered), _stream())
    _check("etv_safe_gather_paths", rc)
    return dict(safe=safe, pvalid=pvalid, gathered=gathered)


def evaluate_posterior_workspace_bytes(B: int, T_max: int, V: int) -> int:
    return int(lib().etv_evaluate_posterior_workspace_bytes(B, T_max, V))


def evaluate_posterior(logits, tokens, retrieve, n_nodes, dummy: int = 0, workspace=None,
                       out: Optional[Dict[str, torch.Tensor]] = None, head_V: int = 0):
    """logits f32 [B,T,V]; tokens int32 [B,T]; retrieve int32 [B,L,W] -> argmax, len, best, accept_len,
    acc_nodes, bonus (all int32).  With logits=None, out["argmax"] is an input (e.g. from lm_head_argmax), or,
    with head_V > 0, `workspace` is the one lm_head_argmax(..., finish=False) returned for that vocabulary size."""
    if logits is None:
        (B, T), V = tokens.shape, int(head_V)
        assert workspace is not None if V else (out is not None and out.get("argmax") is not None)
    else:
        B, T, V = logits.shape
    _, L, W = retrieve.shape
    dev = tokens.device
    o = out or {}
    i32 = dict(dtype=torch.int32, device=dev)
    def get(name, shape):
        t = o.get(name)
        return t if t is not None else torch.empty(shape, **i32)
    g, ln, best = get("argmax", (B, T)), get("len", (B, L)), get("best", (B,))
    A, acc, bonus = get("accept_len", (B,)), get("acc_nodes", (B, W)), get("bonus", (B,))
    if workspace is None and logits is not None:
        workspace = torch.empty((max(256, evaluate_posterior_workspace_bytes(B, T, V)),), dtype=torch.uint8, device=dev)
    rc = lib().etv_evaluate_posterior(_ptr(logits), _ptr(tokens), _ptr(retrieve), _ptr(n_nodes), B, T, V, L, W,
                                      dummy, _ptr(g), _ptr(ln), _ptr(best), _ptr(A), _ptr(acc), _ptr(bonus),
                                      _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream())
    _check("etv_evaluate_posterior", rc)
    return dict(argmax=g, len=ln, best=best, accept_len=A, acc_nodes=acc, bonus=bonus)


def pack_lm_head(weight: torch.Tensor) -> torch.Tensor:
    """weight bf16 [V,D] -> the same weights in the tile order lm_head_argmax streams fastest (flat bf16 tensor)."""
    V, D = weight.shape
    n = int(lib().etv_lm_head_packed_bytes(V, D))
    if n == 0:
        raise EtvError("etv_lm_head_packed_bytes", -2)
    packed = torch.empty((n // 2,), dtype=weight.dtype, device=weight.device)
    _check("etv_pack_lm_head", lib().etv_pack_lm_head(_ptr(weight), V, D, _ptr(packed), _stream()))
    return packed


def lm_head_argmax(hidden, weight, n_nodes, *, V: Optional[int] = None, want_max: bool = True, workspace=None,
                   out: Optional[Dict[str, torch.Tensor]] = None, finish: bool = True):
    """hidden bf16 [B,T,D]; weight bf16 [V,D], or the flat tensor of pack_lm_head together with V
    -> argmax int32 [B,T] (-1 for padding), maxval float32 [B,T].  finish=False stops after the weight pass and
    returns the workspace, to be handed to evaluate_posterior / verify_epilogue with head_V=V."""
    B, T, D = hidden.shape
    packed = weight.dim() == 1
    if not packed:
        V = weight.shape[0]
    assert V is not None
    dev = hidden.device
    o = out or {}
    g = o.get("argmax")
    if g is None:
        g = torch.empty((B, T), dtype=torch.int32, device=dev)
    mx = o.get("maxval") if out else (torch.empty((B, T), dtype=torch.float32, device=dev) if want_max else None)
    if workspace is None:
        workspace = torch.empty((max(256, int(lib().etv_lm_head_argmax_workspace_bytes(B, T, V))),), dtype=torch.uint8,
                                device=dev)
    rc = lib().etv_lm_head_argmax(_ptr(hidden), _ptr(weight), int(packed), _ptr(n_nodes), B, T, D, V,
                                  _ptr(g) if finish else None, _ptr(mx) if finish else None,
                                  _ptr(workspace), workspace.numel(), _stream())
    _check("etv_lm_head_argmax", rc)
    return dict(argmax=g, maxval=mx) if finish else dict(workspace=workspace)


def _commit_desc(kt, k_cache, block_table, W: int, B: Optional[int] = None, T_max: Optional[int] = None) -> CommitDesc:
    if kt is not None:
        Lyr, B, T, Hkv, d = kt.shape
    else:   # in-place branch cache: shapes from the cache, B and T_max from the caller
        Lyr, T = k_cache.shape[0], int(T_max)
        Hkv, d = (k_cache.shape[2], k_cache.shape[4]) if block_table is not None else (k_cache.shape[3], k_cache.shape[4])
    assert k_cache.shape[0] == Lyr
    dsc = CommitDesc(B=B, T_max=T, Hkv=Hkv, d=d, elem_bytes=k_cache.element_size(), n_layers=Lyr, W=W, block_size=0,
                     max_blocks=0, num_blocks=0, P_cap=0, reserved=0,
                     cache_layer_stride=k_cache.stride(0) if Lyr > 1 else k_cache[0].numel())
    if block_table is not None:
        dsc.block_size, dsc.max_blocks, dsc.num_blocks = k_cache.shape[3], block_table.shape[1], k_cache.shape[1]
    else:
        dsc.P_cap = k_cache.shape[2]
    return dsc


def verify_epilogue(logits, tokens, retrieve, n_nodes, kt, vt, k_cache, v_cache, prefix_len, capacity, *,
                    block_table=None, dummy: int = 0, src: Optional[torch.Tensor] = None, workspace=None,
                    gather_out: Optional[Dict[str, torch.Tensor]] = None,
                    post_out: Optional[Dict[str, torch.Tensor]] = None,
                    commit_out: Optional[Dict[str, torch.Tensor]] = None, head_V: int = 0):
    """safe_gather_paths + evaluate_posterior + commit_accepted_kv in three launches; same tensors and results.
    With logits=None, post_out["argmax"] is an input, or, with head_V > 0, `workspace` is the one
    lm_head_argmax(..., finish=False) returned.  Returns (gather dict, posterior dict, commit dict)."""
    if logits is None:
        (B, T), V = tokens.shape, int(head_V)
        assert workspace is not None if V else (post_out is not None and post_out.get("argmax") is not None)
    else:
        B, T, V = logits.shape
    _, L, W = retrieve.shape
    dev = tokens.device
    i32 = dict(dtype=torch.int32, device=dev)
    go, po, co = gather_out or {}, post_out or {}, commit_out or {}

    def get(d, name, shape, dtype=torch.int32):
        t = d.get(name)
        return t if t is not None else torch.empty(shape, dtype=dtype, device=dev)
    safe, pvalid = get(go, "safe", (B, L, W)), get(go, "pvalid", (B, L, W), torch.uint8)
    gathered, row_bytes = None, 0
    if src is not None:
        row_bytes = src[0, 0].numel() * src.element_size()
        gathered = get(go, "gathered", (B, L, W) + tuple(src.shape[2:]), src.dtype)
    g, ln, best = get(po, "argmax", (B, T)), get(po, "len", (B, L)), get(po, "best", (B,))
    A, acc, bonus = get(po, "accept_len", (B,)), get(po, "acc_nodes", (B, W)), get(po, "bonus", (B,))
    plo, slot, status = get(co, "prefix_len_out", (B,)), get(co, "slot_map", (B, W)), get(co, "status", (B,))
    if workspace is None and logits is not None:
        workspace = torch.empty((max(256, evaluate_posterior_workspace_bytes(B, T, V)),), dtype=torch.uint8, device=dev)
    dsc = _commit_desc(kt, k_cache, block_table, W, B, T)
    rc = lib().etv_verify_epilogue(C.byref(dsc), _ptr(logits), V, _ptr(tokens), _ptr(retrieve), L, dummy, _ptr(src),
                                   row_bytes, _ptr(safe), _ptr(pvalid), _ptr(gathered), _ptr(g), _ptr(ln), _ptr(best),
                                   _ptr(A), _ptr(acc), _ptr(bonus), _ptr(kt), _ptr(vt), _ptr(k_cache), _ptr(v_cache),
                                   _ptr(block_table), _ptr(prefix_len), _ptr(capacity), _ptr(n_nodes), _ptr(plo),
                                   _ptr(slot), _ptr(status), _ptr(workspace),
                                   workspace.numel() if workspace is not None else 0, _stream())
    _check("etv_verify_epilogue", rc)
    return (dict(safe=safe, pvalid=pvalid, gathered=gathered),
            dict(argmax=g, len=ln, best=best, accept_len=A, acc_nodes=acc, bonus=bonus),
            dict(prefix_len_out=plo, slot_map=slot, status=status))


def commit_accepted_kv(kt, vt, k_cache, v_cache, prefix_len, capacity, n_nodes, acc_nodes, accept_len, *,
                       block_table=None, prefix_len_out=None, out: Optional[Dict[str, torch.Tensor]] = None,
                       T_max: Optional[int] = None):
    """kt/vt [Lyr,B,T,Hkv,d]; caches [Lyr,B,P_cap,Hkv,d] or [Lyr,nb,Hkv,bs,d] updated in place.
    kt = vt = None (with T_max): in-place branch cache, the tree rows are in the caches behind the prefix.
    Returns prefix_len_out, slot_map, status."""
    B, W = acc_nodes.shape
    dev = k_cache.device
    dsc = _commit_desc(kt, k_cache, block_table, W, B, T_max)
    o = out or {}
    if prefix_len_out is None:
        prefix_len_out = o.get("prefix_len_out")
    if prefix_len_out is None:
        prefix_len_out = torch.empty((B,), dtype=torch.int32, device=dev)
    slot = o.get("slot_map") if out else torch.empty((B, W), dtype=torch.int32, device=dev)
    status = o.get("status") if out else torch.empty((B,), dtype=torch.int32, device=dev)
    rc = lib().etv_commit_accepted_kv(C.byref(dsc), _ptr(kt), _ptr(vt), _ptr(k_cache), _ptr(v_cache),
                                      _ptr(block_table), _ptr(prefix_len), _ptr(capacity), _ptr(n_nodes),
                                      _ptr(acc_nodes), _ptr(accept_len), _ptr(prefix_len_out), _ptr(slot),
                                      _ptr(status), _stream())
    _check("etv_commit_accepted_kv", rc)
    return dict(prefix_len_out=prefix_len_out, slot_map=slot, status=status)


def _cache_desc(cache: torch.Tensor, B: int, table: Optional[torch.Tensor]) -> CacheDesc:
    Lyr = cache.shape[0]
    dsc = CacheDesc(B=B, Hkv=0, d=cache.shape[4], elem_bytes=cache.element_size(), n_layers=Lyr, block_size=0,
                    max_blocks=0, num_blocks=0, P_cap=0, reserved=0,
                    cache_layer_stride=cache.stride(0) if Lyr > 1 else cache[0].numel())
    if table is not None:
        dsc.Hkv, dsc.block_size, dsc.max_blocks, dsc.num_blocks = cache.shape[2], cache.shape[3], table.shape[-1], cache.shape[1]
    else:
        dsc.Hkv, dsc.P_cap = cache.shape[3], cache.shape[2]
    return dsc


def replicate_branches(k_cache, v_cache, block_table, prefix_len, tail_len, N: int, free_blocks):
    """Paged caches [Lyr, nb, Hkv, bs, d]; block_table [B, max_blocks]; free_blocks int32 [n_free].
    Returns branch_table [B, N, max_blocks], block_base [B], n_taken [1], status [B] (device tensors)."""
    B, dev = block_table.shape[0], k_cache.device
    dsc = _cache_desc(k_cache, B, block_table)
    bt = torch.empty((B, N, block_table.shape[1]), dtype=torch.int32, device=dev)
    base = torch.empty((B,), dtype=torch.int32, device=dev)
    taken = torch.empty((1,), dtype=torch.int32, device=dev)
    status = torch.empty((B,), dtype=torch.int32, device=dev)
    rc = lib().etv_replicate_branches(C.byref(dsc), _ptr(k_cache), _ptr(v_cache), _ptr(block_table), _ptr(prefix_len),
                                      _ptr(tail_len), N, _ptr(free_blocks), free_blocks.numel(), _ptr(bt), _ptr(base),
                                      _ptr(taken), _ptr(status), _stream())
    _check("etv_replicate_branches", rc)
    return dict(branch_table=bt, block_base=base, n_taken=taken, status=status)


def commit_path_indices(src_k, src_v, dst_k, dst_v, path_indices, src_len, new_len, *, src_table=None, dst_table=None,
                        fast: bool = False):
    """Caches [Lyr, B, P_cap, Hkv, d] (two buffers) or [Lyr, nb, Hkv, bs, d] with two block tables (dst_table is
    updated in place with the shared blocks).  Returns kept_len, status."""
    B, L_cap = path_indices.shape
    dev = src_k.device
    dsc = _cache_desc(src_k, B, src_table)
    kept = torch.empty((B,), dtype=torch.int32, device=dev)
    status = torch.empty((B,), dtype=torch.int32, device=dev)
    rc = lib().etv_commit_path_indices(C.byref(dsc), _ptr(src_k), _ptr(src_v), _ptr(dst_k), _ptr(dst_v), _ptr(src_table),
                                       _ptr(dst_table), _ptr(path_indices), L_cap, _ptr(src_len), _ptr(new_len),
                                       int(fast), _ptr(kept), _ptr(status), _stream())
    _check("etv_commit_path_indices", rc)
    return dict(kept_len=kept, status=status)
