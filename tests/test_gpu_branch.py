"""GPU parity (bit-exact) for the branch-cache calls: replicate_branches and commit_path_indices against the oracle,
and the flow replicate -> teacher pass writes the tails -> tree attention over all branches -> commit of the
selected branch."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_08088_amd import api, synth
from gpu_helpers import attention_errors, bits_of, to_dev
from helpers import random_tree

pytestmark = pytest.mark.gpu
BS = synth.BLOCK


def _pool(rng, B, lens, Lyr, dtype, Hkv, d, spare):
    need = [(n + BS - 1) // BS for n in lens]
    nb = sum(need) + spare
    perm = rng.permutation(nb).astype(np.int32)
    table = np.full((B, max(max(need), 1)), -1, dtype=np.int32)
    at = 0
    for b in range(B):
        table[b, :need[b]] = perm[at:at + need[b]]
        at += need[b]
    kc = synth._values(rng, (Lyr, nb, Hkv, BS, d), dtype)
    vc = synth._values(rng, (Lyr, nb, Hkv, BS, d), dtype)
    return kc, vc, table, perm[at:].copy()


def _replicate_case(kc, vc, table, P, tail, N, free):
    okc, ovc = kc.copy(), vc.copy()
    ref = oracle.replicate_branches(okc, ovc, table, P, tail, N, free)
    dkc, dvc = to_dev(kc), to_dev(vc)
    got = api.replicate_branches(dkc, dvc, to_dev(table), to_dev(np.asarray(P, dtype=np.int32)),
                                 to_dev(np.asarray(tail, dtype=np.int32)), N, to_dev(free))
    torch.cuda.synchronize()
    for name in ("branch_table", "block_base", "status"):
        assert np.array_equal(bits_of(got[name]), ref[name]), name
    assert int(got["n_taken"].item()) == ref["n_taken"]
    assert np.array_equal(bits_of(dkc), okc) and np.array_equal(bits_of(dvc), ovc)
    return ref, dkc, dvc, got


@pytest.mark.parametrize("dtype,Hkv,d,Lyr", [("bf16", 8, 128, 3), ("f32", 2, 64, 2), ("bf16", 1, 8, 1)])
def test_replicate_matches_the_oracle(dtype, Hkv, d, Lyr):
    rng = np.random.default_rng(500 + d)
    P = [1000, 37, 32, 5, 0, 511, 16]
    tail = [60, 20, 16, 0, 7, 1, 0]
    B, N = len(P), 4
    kc, vc, table, free = _pool(rng, B, [p + t for p, t in zip(P, tail)], Lyr, dtype, Hkv, d, spare=4 * 40)
    ref, *_ = _replicate_case(kc, vc, table, P, tail, N, free)
    assert np.all(ref["status"] == 0) and ref["n_taken"] > 0


def test_replicate_many_sequences_and_one_branch():
    """More sequences than the scan's 256 lanes, and N = 1 (a single branch is still a private tail)."""
    rng = np.random.default_rng(510)
    B = 600
    P = rng.integers(0, 90, size=B).tolist()
    tail = rng.integers(0, 40, size=B).tolist()
    kc, vc, table, free = _pool(rng, B, [p + t for p, t in zip(P, tail)], 1, "bf16", 1, 8, spare=3 * 2000)
    for N in (1, 3):
        ref, *_ = _replicate_case(kc, vc, table, P, tail, N, free)
        assert np.all(ref["status"] == 0)


def test_replicate_failures():
    rng = np.random.default_rng(520)
    P, tail = [20, 30, 40, 50], [10, 10, 10, 10]
    kc, vc, table, free = _pool(rng, 4, [60] * 4, 2, "bf16", 2, 8, spare=40)
    ref, *_ = _replicate_case(kc, vc, table, P, tail, 4, free[:15])         # 16 needed
    assert ref["n_taken"] == 0 and np.all(ref["status"] == oracle.BRANCH_NO_BLOCKS)
    bad = table.copy()
    bad[1, 0] = kc.shape[1]
    ref, *_ = _replicate_case(kc, vc, bad, [20, 30, -1, 50], [10, 10, 10, 4000], 2, free)
    assert ref["status"].tolist() == [0, oracle.COMMIT_BAD_BLOCK, oracle.COMMIT_BAD_LEN, oracle.COMMIT_CAPACITY]
    f2 = free.copy()
    f2[1] = -3
    f2[5] = kc.shape[1]
    ref, *_ = _replicate_case(kc, vc, table, P, tail, 2, f2)
    assert ref["status"].tolist() == [oracle.BRANCH_BAD_FREE, oracle.BRANCH_BAD_FREE, 0, 0]   # blocks 0-1 and 2-5
    ref, *_ = _replicate_case(kc, vc, table[:0], [], [], 2, free)            # empty batch
    assert ref["n_taken"] == 0


def _two_tables(rng, B, Ls, Ln, Lyr, dtype, Hkv, d):
    kc, vc, table, free = _pool(rng, B, Ls, Lyr, dtype, Hkv, d, spare=sum((n + BS - 1) // BS for n in Ln) + 7)
    width = max(table.shape[1], max((n + BS - 1) // BS for n in Ln))
    src, dst = np.full((B, width), -1, dtype=np.int32), np.full((B, width), -1, dtype=np.int32)
    src[:, :table.shape[1]] = table
    at = 0
    for b in range(B):
        nb = (Ln[b] + BS - 1) // BS
        dst[b, :nb] = free[at:at + nb]
        at += nb
    return kc, vc, src, dst


def _path_case(kc, vc, src, dst, idx, Ls, Ln, fast):
    okc, ovc, odst = kc.copy(), vc.copy(), dst.copy()
    ref = oracle.commit_path_indices(okc, ovc, okc, ovc, idx, Ls, Ln, src_table=src, dst_table=odst, fast=fast)
    dkc, dvc, ddst = to_dev(kc), to_dev(vc), to_dev(dst)
    got = api.commit_path_indices(dkc, dvc, dkc, dvc, to_dev(idx), to_dev(np.asarray(Ls, dtype=np.int32)),
                                  to_dev(np.asarray(Ln, dtype=np.int32)), src_table=to_dev(src), dst_table=ddst, fast=fast)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(got["status"]), ref["status"])
    assert np.array_equal(bits_of(got["kept_len"]), ref["kept_len"])
    assert np.array_equal(bits_of(ddst), odst)
    assert np.array_equal(bits_of(dkc), okc) and np.array_equal(bits_of(dvc), ovc)
    return ref


@pytest.mark.parametrize("fast", [False, True])
@pytest.mark.parametrize("dtype,Hkv,d,Lyr", [("bf16", 8, 128, 2), ("f32", 2, 64, 2), ("bf16", 1, 8, 1)])
def test_path_index_commit_paged(fast, dtype, Hkv, d, Lyr):
    rng = np.random.default_rng(530 + d)
    Ls = [300, 33, 16, 7, 200, 129, 90]
    Ln = [280, 60, 0, 7, 190, 140, 90]
    B, L_cap = len(Ls), 304
    kc, vc, src, dst = _two_tables(rng, B, Ls, Ln, Lyr, dtype, Hkv, d)
    idx = rng.integers(-9, 400, size=(B, L_cap)).astype(np.int32)          # garbage behind new_len
    idx[0, :280] = rng.permutation(300)[:280]                              # nothing preserved
    idx[1, :60] = rng.integers(0, 33, size=60)                             # repeats, longer than the source
    idx[3, :7] = np.arange(7)[::-1]
    idx[4, :190] = np.r_[np.arange(170), 170 + rng.permutation(30)[:20]]   # an accepted path behind a kept prefix
    idx[5, :140] = np.r_[np.arange(129), rng.integers(0, 129, size=11)]
    idx[6, :90] = np.arange(90); idx[6, [40, 41]] = [41, 40]               # order breaks in the third block
    ref = _path_case(kc, vc, src, dst, idx, Ls, Ln, fast)
    assert np.all(ref["status"] == 0)
    assert ref["kept_len"].tolist() == ([0, 0, 0, 0, 160, 128, 32] if fast else [0] * 7)


def test_path_index_commit_contiguous_and_failures():
    rng = np.random.default_rng(540)
    B, cap, Lyr = 4, 70, 2
    sk, sv = synth._values(rng, (Lyr, B, cap, 4, 64), "bf16"), synth._values(rng, (Lyr, B, cap, 4, 64), "bf16")
    dk, dv = synth._values(rng, sk.shape, "bf16"), synth._values(rng, sk.shape, "bf16")
    idx = rng.integers(0, 50, size=(B, 70)).astype(np.int32)
    idx[2, 3] = 50                                                         # one past the branch cache
    Ls, Ln = [50, 50, 50, 50], [70, 11, 20, 0]
    odk, odv = dk.copy(), dv.copy()
    ref = oracle.commit_path_indices(sk, sv, odk, odv, idx, Ls, Ln, fast=True)
    ddk, ddv = to_dev(dk), to_dev(dv)
    got = api.commit_path_indices(to_dev(sk), to_dev(sv), ddk, ddv, to_dev(idx), to_dev(np.asarray(Ls, dtype=np.int32)),
                                  to_dev(np.asarray(Ln, dtype=np.int32)), fast=True)
    torch.cuda.synchronize()
    assert ref["status"].tolist() == [0, 0, oracle.COMMIT_BAD_NODE, 0]
    assert np.array_equal(bits_of(got["status"]), ref["status"]) and np.all(bits_of(got["kept_len"]) == 0)
    assert np.array_equal(bits_of(ddk), odk) and np.array_equal(bits_of(ddv), odv)
    with pytest.raises(api.EtvError):                                      # a contiguous cache is rebuilt elsewhere
        api.commit_path_indices(ddk, ddv, ddk, ddv, to_dev(idx), to_dev(np.asarray(Ls, dtype=np.int32)),
                                to_dev(np.asarray(Ln, dtype=np.int32)))
    # paged: both tables index one pool, and they are two tables
    kc, vc, src, dst = _two_tables(rng, 2, [20, 20], [20, 20], 1, "bf16", 2, 8)
    dk_, dv_, dsrc, ddst = to_dev(kc), to_dev(vc), to_dev(src), to_dev(dst)
    lens = to_dev(np.asarray([20, 20], dtype=np.int32))
    ident = to_dev(np.tile(np.arange(20, dtype=np.int32), (2, 1)))
    with pytest.raises(api.EtvError):
        api.commit_path_indices(dk_, dv_, to_dev(kc), dv_, ident, lens, lens, src_table=dsrc, dst_table=ddst)
    with pytest.raises(api.EtvError):
        api.commit_path_indices(dk_, dv_, dk_, dv_, ident, lens, lens, src_table=dsrc, dst_table=dsrc)
    # paged failures: bad lengths, capacity, a hole in the destination table
    kc, vc, src, dst = _two_tables(rng, 4, [30] * 4, [30] * 4, 1, "bf16", 2, 8)
    ids = np.tile(np.arange(40, dtype=np.int32), (4, 1))
    ids[:, 30:] = 0
    bad = dst.copy()
    bad[3, 1] = -1
    ref = _path_case(kc, vc, src, bad, ids, [30, 33, 30, 30], [41, 30, 33, 30], True)
    assert ref["status"].tolist() == [oracle.COMMIT_BAD_LEN, oracle.COMMIT_BAD_LEN, oracle.COMMIT_CAPACITY,
                                      oracle.COMMIT_BAD_BLOCK]


def test_branches_through_attention_and_commit():
    """Replicate the committed cache into N branches per sequence, let every branch hold a different tree behind
    the prefix (as the teacher pass would write it), run tree attention over all B*N branch caches in one launch,
    commit the selected branch by path indices into fresh blocks and, separately, compact it in place.  Every
    stage is compared with the oracle working on the same pool."""
    rng = np.random.default_rng(550)
    B, N, T, Hq, Hkv, d = 3, 2, 24, 8, 2, 128
    P = [200, 64, 37]
    kc, vc, table, free = _pool(rng, B, [p + T for p in P], 1, "bf16", Hkv, d, spare=60)
    ref, dkc, dvc, got = _replicate_case(kc, vc, table, P, [T] * B, N, free)
    bt = ref["branch_table"]
    okc, ovc = kc.copy(), vc.copy()
    oracle.replicate_branches(okc, ovc, table, P, [T] * B, N, free)
    # branch (b, i) is sequence b*N + i of the attention batch
    parents = [random_tree(rng, T) for _ in range(B * N)]
    wl = synth.assemble("branches", rng, parents, [P[s // N] for s in range(B * N)], Hq=Hq, Hkv=Hkv, d=d, dtype="bf16",
                        V=512, W=T, paged=True, with_cache=False, with_logits=False)
    flat = bt.reshape(B * N, -1)
    for s in range(B * N):
        for j in range(T):
            pos = P[s // N] + j
            okc[0, flat[s, pos // BS], :, pos % BS] = wl.kt[s, j]
            ovc[0, flat[s, pos // BS], :, pos % BS] = wl.vt[s, j]
    dkc.copy_(to_dev(okc)); dvc.copy_(to_dev(ovc))
    par, n = to_dev(wl.parent), to_dev(wl.n_nodes)
    m = api.build_tree_mask(par, n)
    dflat = got["branch_table"].view(B * N, -1)
    out, _ = api.tree_verify_attention(to_dev(wl.q), dkc[0], dvc[0], to_dev(wl.prefix_len), None, None, m["bitmask"], n,
                                       P_max=max(P), block_table=dflat)
    torch.cuda.synchronize()
    rm = oracle.build_tree_mask(wl.parent, wl.n_nodes)
    want, _ = oracle.tree_verify_attention(wl.q, okc[0], ovc[0], wl.prefix_len, wl.kt, wl.vt, rm["dense"], wl.n_nodes,
                                           dtype="bf16", block_table=flat)
    err, rel, padded_zero = attention_errors(out, want, wl.n_nodes)
    assert padded_zero and err <= 2e-2 and rel <= 2e-2, (err, rel)
    # the selected branch of every sequence, committed by path indices into fresh blocks (fast: prefix shared)
    sel = [1, 0, 1]
    acc = [[int(x) for x in wl.retrieve[b * N + sel[b], 0] if x >= 0] for b in range(B)]
    Ln = [P[b] + len(acc[b]) for b in range(B)]
    idx = np.zeros((B, max(Ln)), dtype=np.int32)
    for b in range(B):
        idx[b, :Ln[b]] = np.r_[np.arange(P[b]), P[b] + np.asarray(acc[b])]
    src = np.stack([bt[b, sel[b]] for b in range(B)])
    dst = np.full_like(src, -1)
    at = ref["n_taken"]
    for b in range(B):
        nb = (Ln[b] + BS - 1) // BS
        dst[b, :nb] = free[at:at + nb]
        at += nb
    r2 = _path_case(okc, ovc, src, dst, idx, [P[b] + T for b in range(B)], Ln, True)
    assert r2["kept_len"].tolist() == [p // BS * BS for p in P]
    # and the in-place compaction of the same branch gives the same logical rows (oracle-side pin); here: parity
    accw = np.zeros((B, T), dtype=np.int32)
    A = np.zeros(B, dtype=np.int32)
    for b in range(B):
        accw[b, :len(acc[b])] = acc[b]
        A[b] = len(acc[b]) - 1
    cap = np.asarray([src.shape[1] * BS] * B, dtype=np.int32)
    ck, cv = okc.copy(), ovc.copy()
    rc = oracle.commit_accepted_kv(None, None, ck, cv, P, cap, [T] * B, accw, A, block_table=src, T_max=T)
    dk2, dv2 = to_dev(okc), to_dev(ovc)
    c = api.commit_accepted_kv(None, None, dk2, dv2, to_dev(np.asarray(P, dtype=np.int32)), to_dev(cap),
                               to_dev(np.full(B, T, dtype=np.int32)), to_dev(accw), to_dev(A), block_table=to_dev(src),
                               T_max=T)
    torch.cuda.synchronize()
    assert np.all(rc["status"] == 0) and np.array_equal(bits_of(c["status"]), rc["status"])
    assert np.array_equal(bits_of(dk2), ck) and np.array_equal(bits_of(dv2), cv)


def test_branch_calls_at_the_benchmark_shape():
    """The shape bench.py times (B=8 sequences, N=4 branches, P=2040, T=60, 8 KV heads, d=128, bf16, 16-row blocks),
    on two layers: replication, then the selected branch committed by path indices with the prefix kept and as a
    full reorder, every byte of the pool compared with the oracle."""
    rng = np.random.default_rng(560)
    B, N, P, T, Hkv, d, Lyr = 8, 4, 2040, 60, 8, 128, 2
    kc, vc, table, free = _pool(rng, B, [P + T] * B, Lyr, "bf16", Hkv, d, spare=B * N * 5 + B * 132 + 9)
    ref, dkc, dvc, got = _replicate_case(kc, vc, table, [P] * B, [T] * B, N, free)
    assert np.all(ref["status"] == 0) and ref["n_taken"] == B * N * ((P + T + BS - 1) // BS - P // BS)
    okc, ovc = bits_of(dkc), bits_of(dvc)                      # the pool after replication (equal to the oracle's)
    src = np.ascontiguousarray(ref["branch_table"][:, 1])
    Ln = P + 6
    idx = np.tile(np.arange(Ln, dtype=np.int32), (B, 1))
    idx[:, P:] = P + np.asarray([0, 2, 7, 19, 33, 51], dtype=np.int32)
    dst = np.full_like(src, -1)
    nb = (Ln + BS - 1) // BS
    dst[:, :nb] = free[ref["n_taken"]: ref["n_taken"] + B * nb].reshape(B, nb)
    for fast in (True, False):
        r = _path_case(okc, ovc, src, dst, idx, [P + T] * B, [Ln] * B, fast)
        assert np.all(r["status"] == 0) and np.all(r["kept_len"] == (P // BS * BS if fast else 0))
    perm = np.stack([rng.permutation(P + T)[:Ln] for _ in range(B)]).astype(np.int32)
    r = _path_case(okc, ovc, src, dst, perm, [P + T] * B, [Ln] * B, True)   # nothing to keep: the fall-back
    assert np.all(r["status"] == 0) and np.all(r["kept_len"] == 0)


def test_branch_calls_replayed_from_a_hip_graph():
    """Replication and the commit by path indices captured once in a HIP graph and replayed with eager work in
    between: every replay reproduces the oracle's tables and pool."""
    rng = np.random.default_rng(570)
    B, N, T, Hkv, d = 3, 2, 20, 2, 64
    P = [70, 33, 16]
    kc, vc, table, free = _pool(rng, B, [p + T for p in P], 2, "bf16", Hkv, d, spare=64)
    okc, ovc = kc.copy(), vc.copy()
    ref = oracle.replicate_branches(okc, ovc, table, P, [T] * B, N, free)
    src = np.ascontiguousarray(ref["branch_table"][:, 0])
    Ln = [p + 4 for p in P]
    idx = np.zeros((B, max(Ln)), dtype=np.int32)
    for b in range(B):
        idx[b, :Ln[b]] = np.r_[np.arange(P[b]), P[b] + np.asarray([0, 3, 9, 17])]
    dst = np.full_like(src, -1)
    at = ref["n_taken"]
    for b in range(B):
        nb = (Ln[b] + BS - 1) // BS
        dst[b, :nb] = free[at:at + nb]
        at += nb
    odst = dst.copy()
    r2 = oracle.commit_path_indices(okc, ovc, okc, ovc, idx, [p + T for p in P], Ln, src_table=src, dst_table=odst,
                                    fast=True)
    dkc, dvc = to_dev(kc), to_dev(vc)
    dtab, dP, dT, dfree = to_dev(table), to_dev(np.asarray(P, dtype=np.int32)), to_dev(np.full(B, T, dtype=np.int32)), to_dev(free)
    didx, dLs, dLn = to_dev(idx), to_dev(np.asarray([p + T for p in P], dtype=np.int32)), to_dev(np.asarray(Ln, dtype=np.int32))
    ddst = to_dev(dst)
    res = {}

    def calls():
        res["rep"] = api.replicate_branches(dkc, dvc, dtab, dP, dT, N, dfree)
        res["src"] = res["rep"]["branch_table"][:, 0].contiguous()
        res["com"] = api.commit_path_indices(dkc, dvc, dkc, dvc, didx, dLs, dLn, src_table=res["src"], dst_table=ddst,
                                             fast=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        calls()
    for rep in range(3):
        dkc.copy_(to_dev(kc)); dvc.copy_(to_dev(vc)); ddst.copy_(to_dev(dst))     # eager work between the replays
        res["rep"]["branch_table"].fill_(-9); res["com"]["kept_len"].fill_(-9)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bits_of(res["rep"]["branch_table"]), ref["branch_table"]), rep
        assert int(res["rep"]["n_taken"].item()) == ref["n_taken"]
        assert np.array_equal(bits_of(res["com"]["kept_len"]), r2["kept_len"]) and np.all(bits_of(res["com"]["status"]) == 0)
        assert np.array_equal(bits_of(ddst), odst)
        assert np.array_equal(bits_of(dkc), okc) and np.array_equal(bits_of(dvc), ovc)
