"""Pins for the oracle's tree-masked attention against library float64 attention on
the cases that reduce to it, closed forms, and invariances."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_08088_amd import synth
from helpers import as_f64, path_to, random_tree


def _inputs(rng, B, T, Hq, Hkv, d, P, dtype="f32", paged=False, n_nodes=None, q_scale=1.0):
    parents = [random_tree(rng, T) for _ in range(B)]
    if n_nodes is not None:
        parents = [p[:n] for p, n in zip(parents, n_nodes)]
    wl = synth.assemble("t", rng, parents, [P] * B if np.isscalar(P) else P, Hq=Hq, Hkv=Hkv, d=d, dtype=dtype,
                        V=512, W=T, paged=paged, T_max=T, with_logits=False, q_scale=q_scale, spare_blocks=3)
    return wl


def _run(wl, dense=None, **kw):
    if dense is None:
        dense = oracle.build_tree_mask(wl.parent, wl.n_nodes)["dense"]
    return oracle.tree_verify_attention(wl.q, wl.k_cache, wl.v_cache, wl.prefix_len, wl.kt, wl.vt, dense,
                                        wl.n_nodes, dtype=wl.dtype, block_table=wl.block_table, **kw)


def _prefix_rows(wl, b, kvh, which):
    """Logical prefix rows [P, d] of one KV head as float64, read straight from the generator's layout."""
    cache = as_f64(wl.k_cache if which == "k" else wl.v_cache, wl.dtype)
    P = int(wl.prefix_len[b])
    if wl.paged:
        rows = [cache[wl.block_table[b, j // synth.BLOCK], kvh, j % synth.BLOCK] for j in range(P)]
        return np.stack(rows) if rows else np.zeros((0, wl.d))
    return cache[b, :P, kvh]


def _lib_attention(q, K, V):
    """float64 library softmax attention of one query vector over rows K, V."""
    qt, Kt, Vt = (torch.from_numpy(np.ascontiguousarray(x)) for x in (q, K, V))
    s = (Kt @ qt) / np.sqrt(q.shape[0])
    return (torch.softmax(s, dim=0) @ Vt).numpy(), float(torch.logsumexp(s, dim=0))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_node_tree_is_plain_decode_attention(dtype):
    rng = np.random.default_rng(11)
    wl = _inputs(rng, 2, 1, 8, 2, 32, 37, dtype=dtype)
    out, lse = _run(wl)
    G = wl.Hq // wl.Hkv
    q, kt, vt = as_f64(wl.q, dtype), as_f64(wl.kt, dtype), as_f64(wl.vt, dtype)
    for b in range(2):
        for h in range(wl.Hq):
            K = np.concatenate([_prefix_rows(wl, b, h // G, "k"), kt[b, :1, h // G]])
            V = np.concatenate([_prefix_rows(wl, b, h // G, "v"), vt[b, :1, h // G]])
            ref, ref_lse = _lib_attention(q[b, 0, h], K, V)
            assert np.abs(out[b, 0, h] - ref).max() < 1e-12
            assert abs(lse[b, h, 0] - ref_lse) < 1e-12


def test_chain_tree_is_causal_attention_library_sdpa():
    rng = np.random.default_rng(12)
    B, T, Hq, Hkv, d, P = 1, 9, 4, 2, 16, 21
    wl = synth.assemble("t", rng, [synth.tree_chain(T)], [P], Hq=Hq, Hkv=Hkv, d=d, dtype="f32", V=512, W=T,
                        paged=False, with_logits=False)
    out, _ = _run(wl)
    G = Hq // Hkv
    q = torch.from_numpy(as_f64(wl.q, "f32")[0]).permute(1, 0, 2)                       # [Hq,T,d]
    K = np.concatenate([as_f64(wl.k_cache, "f32")[0, :P], as_f64(wl.kt, "f32")[0]])      # [P+T,Hkv,d]
    V = np.concatenate([as_f64(wl.v_cache, "f32")[0, :P], as_f64(wl.vt, "f32")[0]])
    Kh = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)               # [Hq,P+T,d]
    Vh = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)
    mask = torch.ones(T, P + T, dtype=torch.bool).tril(diagonal=P)                      # causal, offset by prefix
    ref = torch.nn.functional.scaled_dot_product_attention(q[None], Kh[None], Vh[None], attn_mask=mask)[0]
    assert np.abs(out[0].transpose(1, 0, 2) - ref.numpy()).max() < 1e-12


@pytest.mark.parametrize("paged,dtype", [(False, "f32"), (True, "bf16")])
def test_every_node_equals_sequential_decode_over_its_own_path(paged, dtype):
    """Context correctness (Section 3.3): row k depends only on the prefix and k's ancestor chain."""
    rng = np.random.default_rng(13)
    wl = _inputs(rng, 2, 14, 8, 2, 32, [40, 23], dtype=dtype, paged=paged)
    out, lse = _run(wl)
    G = wl.Hq // wl.Hkv
    q, kt, vt = as_f64(wl.q, dtype), as_f64(wl.kt, dtype), as_f64(wl.vt, dtype)
    for b in range(wl.B):
        for k in range(int(wl.n_nodes[b])):
            path = path_to(wl.parent[b], k)
            for h in range(wl.Hq):
                K = np.concatenate([_prefix_rows(wl, b, h // G, "k"), kt[b, path, h // G]])
                V = np.concatenate([_prefix_rows(wl, b, h // G, "v"), vt[b, path, h // G]])
                ref, ref_lse = _lib_attention(q[b, k, h], K, V)
                assert np.abs(out[b, k, h] - ref).max() < 1e-12
                assert abs(lse[b, h, k] - ref_lse) < 1e-12


def test_closed_forms_equal_keys_and_dominant_key():
    rng = np.random.default_rng(14)
    wl = _inputs(rng, 1, 6, 2, 2, 16, 30)
    # all visible keys identical => uniform weights => output = mean of the visible V rows
    wl.k_cache[...] = wl.k_cache[0, 0, 0]
    for hh in range(2):
        wl.k_cache[0, :, hh] = wl.k_cache[0, 0, 0]
        wl.kt[0, :, hh] = wl.k_cache[0, 0, 0]
    out, _ = _run(wl)
    dense = oracle.build_tree_mask(wl.parent, wl.n_nodes)["dense"][0, 0]
    for k in range(6):
        vis = np.flatnonzero(dense[k])
        for h in range(2):
            V = np.concatenate([wl.v_cache[0, :30, h], wl.vt[0, vis, h]]).astype(np.float64)
            assert np.abs(out[0, k, h] - V.mean(axis=0)).max() < 1e-12
    # one prefix key aligned with q and scaled up dominates the softmax => output ~ its V row
    wl2 = _inputs(rng, 1, 3, 1, 1, 16, 12)
    wl2.k_cache[0, 5, 0] = wl2.q[0, 2, 0] * 400.0 / np.dot(wl2.q[0, 2, 0], wl2.q[0, 2, 0])   # score = 100
    out2, _ = _run(wl2)
    assert np.abs(out2[0, 2, 0] - wl2.v_cache[0, 5, 0]).max() < 1e-15


def test_relabeling_nodes_permutes_outputs():
    rng = np.random.default_rng(15)
    wl = _inputs(rng, 1, 10, 4, 2, 16, 17)
    out, _ = _run(wl)
    # swap labels 4 and 7 (any permutation that fixes the root is a valid relabeling for the mask definition)
    perm = np.arange(10); perm[4], perm[7] = 7, 4
    inv = np.argsort(perm)
    par2 = np.zeros_like(wl.parent)
    for k in range(10):
        par2[0, perm[k]] = perm[wl.parent[0, k]]
    dense2 = oracle.build_tree_mask(par2, wl.n_nodes)
    assert dense2["status"][0] == 0
    out2, _ = oracle.tree_verify_attention(wl.q[:, inv], wl.k_cache, wl.v_cache, wl.prefix_len, wl.kt[:, inv],
                                           wl.vt[:, inv], dense2["dense"], wl.n_nodes, dtype="f32")
    assert np.abs(out2[:, perm] - out).max() < 1e-12


def test_paged_equals_contiguous_under_any_block_table():
    rng = np.random.default_rng(16)
    wl = _inputs(rng, 3, 7, 4, 2, 16, [33, 16, 5], dtype="bf16", paged=True)
    out_p, lse_p = _run(wl)
    P_cap = 40
    kc = np.zeros((3, P_cap, 2, 16), dtype=np.uint16)
    vc = np.zeros_like(kc)
    for b in range(3):
        for j in range(int(wl.prefix_len[b])):
            kc[b, j] = wl.k_cache[wl.block_table[b, j // synth.BLOCK], :, j % synth.BLOCK]
            vc[b, j] = wl.v_cache[wl.block_table[b, j // synth.BLOCK], :, j % synth.BLOCK]
    dense = oracle.build_tree_mask(wl.parent, wl.n_nodes)["dense"]
    out_c, lse_c = oracle.tree_verify_attention(wl.q, kc, vc, wl.prefix_len, wl.kt, wl.vt, dense, wl.n_nodes,
                                                dtype="bf16")
    assert np.array_equal(out_p, out_c) and np.array_equal(lse_p, lse_c)


def test_no_leak_from_non_ancestors_padded_rows_and_stale_cache():
    rng = np.random.default_rng(17)
    T_max, n, P = 12, 9, 20
    wl = _inputs(rng, 1, T_max, 4, 2, 16, P, n_nodes=[n])
    assert wl.n_nodes[0] == n and wl.q.shape[1] == T_max
    out, lse = _run(wl)
    dense = oracle.build_tree_mask(wl.parent, wl.n_nodes)["dense"][0, 0]
    k = 8
    hidden = [j for j in range(T_max) if not dense[k, j]]
    wl.vt[0, hidden] = 1e4
    wl.kt[0, hidden] = 1e4
    wl.k_cache[0, P:] = 1e4          # rows past prefix_len are not part of the committed prefix
    wl.v_cache[0, P:] = 1e4
    wl.q[0, n:] = 1e4                # padded query rows
    out2, lse2 = _run(wl)
    assert np.array_equal(out2[0, k], out[0, k]) and np.array_equal(lse2[0, :, k], lse[0, :, k])
    assert np.all(out2[0, n:] == 0) and np.all(np.isneginf(lse2[0, :, n:]))


def test_empty_prefix_and_scale_argument():
    rng = np.random.default_rng(18)
    wl = _inputs(rng, 1, 5, 2, 1, 8, 0)
    out, _ = _run(wl)
    assert np.abs(out[0, 0, 0] - wl.vt[0, 0, 0]).max() < 1e-15     # the root sees only itself
    o1, _ = _run(wl, scale=1.0 / np.sqrt(8))
    assert np.array_equal(o1, out)
    o2, _ = _run(wl, scale=0.5)
    assert not np.array_equal(o2, out)
