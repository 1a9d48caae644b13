"""Pins for the oracle's branch-cache calls (Section 3.1): copy-on-write replication against the deep copy it
stands for (content, isolation, block accounting), and the path-index commit against the gather that defines it
(numpy fancy indexing of the logical rows), against the pinned length-based commit, and with the fast path
falling back when the indices do not preserve the prefix."""
import numpy as np
import pytest

import oracle
from paper_2603_08088_amd import synth

BS = synth.BLOCK


def logical(cache, table_row, L):
    """Rows 0..L-1 of one sequence of a paged cache [Lyr, nb, Hkv, bs, d] -> [Lyr, L, Hkv, d]."""
    pos = np.arange(L)
    return cache[:, np.asarray(table_row)[pos // BS], :, pos % BS].transpose(1, 0, 2, 3)


def _pool(rng, B, P, tail, Lyr=2, dtype="bf16", Hkv=2, d=8, spare=40):
    need = [(p + tail + BS - 1) // BS for p in P]
    nb = sum(need) + spare
    perm = rng.permutation(nb).astype(np.int32)
    table = np.full((B, max(need)), -1, dtype=np.int32)
    at = 0
    for b in range(B):
        table[b, :need[b]] = perm[at:at + need[b]]
        at += need[b]
    kc = synth._values(rng, (Lyr, nb, Hkv, BS, d), dtype)
    vc = synth._values(rng, (Lyr, nb, Hkv, BS, d), dtype)
    return kc, vc, table, perm[at:].copy()


# ----------------------------------------------------------------------------------------------------------------
# replication
# ----------------------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_replicas_hold_the_committed_rows_and_are_isolated(dtype):
    rng = np.random.default_rng(71)
    B, N, tail = 4, 3, 20
    P = [37, 32, 5, 0]                                   # mid-block, block-aligned, inside the first block, empty
    kc, vc, table, free = _pool(rng, B, P, tail, dtype=dtype)
    k0, v0 = kc.copy(), vc.copy()
    r = oracle.replicate_branches(kc, vc, table, P, [tail] * B, N, free)
    assert np.all(r["status"] == 0)
    bt = r["branch_table"]
    need = [(p + tail + BS - 1) // BS - p // BS for p in P]
    assert r["n_taken"] == N * sum(need)
    assert r["block_base"].tolist() == [N * sum(need[:b]) for b in range(B)]
    # the deep copy the replica stands for: every branch reads the committed rows of the main cache
    for b in range(B):
        want_k, want_v = logical(k0, table[b], P[b]), logical(v0, table[b], P[b])
        for i in range(N):
            assert np.array_equal(logical(kc, bt[b, i], P[b]), want_k)
            assert np.array_equal(logical(vc, bt[b, i], P[b]), want_v)
            assert np.array_equal(bt[b, i, :P[b] // BS], table[b, :P[b] // BS])        # whole blocks are shared
            assert np.all(bt[b, i, P[b] // BS + need[b]:] == -1)
    # the main cache reads as before, and nothing outside the taken blocks changed
    taken = free[:r["n_taken"]]
    rest = np.setdiff1d(np.arange(kc.shape[1]), taken)
    assert np.array_equal(kc[:, rest], k0[:, rest]) and np.array_equal(vc[:, rest], v0[:, rest])
    # private blocks: each taken block appears exactly once over all branches, none is a block of a main table
    priv = np.concatenate([bt[b, i, P[b] // BS: P[b] // BS + need[b]] for b in range(B) for i in range(N)])
    assert sorted(priv.tolist()) == sorted(taken.tolist()) and len(set(priv.tolist())) == len(priv)
    assert not set(priv.tolist()) & set(table[table >= 0].tolist())
    # isolation: extend every branch in place with its own rows; main and the other branches read as before
    for b in range(B):
        for i in range(N):
            for j in range(P[b], P[b] + tail):
                kc[:, bt[b, i, j // BS], :, j % BS] = synth._values(rng, kc[:, 0, :, 0].shape, dtype)
    for b in range(B):
        assert np.array_equal(logical(kc, table[b], P[b]), logical(k0, table[b], P[b]))
        for i in range(N):
            assert np.array_equal(logical(kc, bt[b, i], P[b]), logical(k0, table[b], P[b]))
        tails = [logical(kc, bt[b, i], P[b] + tail)[:, P[b]:] for i in range(N)]
        assert not np.array_equal(tails[0], tails[1])


def test_block_aligned_prefix_copies_nothing_and_zero_tail_takes_only_the_partial_block():
    rng = np.random.default_rng(72)
    kc, vc, table, free = _pool(rng, 3, [48, 48, 50], 16)
    k0 = kc.copy()
    r = oracle.replicate_branches(kc, vc, table, [48, 48, 50], [16, 0, 0], 2, free)
    assert np.all(r["status"] == 0)
    moved = r["branch_table"][2, :, 3]                    # aligned prefixes: no row moves; 50: two rows per branch
    rest = np.setdiff1d(np.arange(kc.shape[1]), moved)
    assert np.array_equal(kc[:, rest], k0[:, rest]) and np.array_equal(kc[:, moved][:, :, :, 2:], k0[:, moved][:, :, :, 2:])
    assert r["n_taken"] == 2 * (1 + 0 + 1)
    assert np.all(r["branch_table"][1, :, 3:] == -1) and np.array_equal(r["branch_table"][1, 0, :3], table[1, :3])
    blk = r["branch_table"][2, 1, 3]
    assert blk == free[3] and np.array_equal(kc[:, blk, :, :2], k0[:, table[2, 3], :, :2])


def test_replication_failures_take_nothing():
    rng = np.random.default_rng(73)
    kc, vc, table, free = _pool(rng, 3, [20, 30, 40], 10)
    k0 = kc.copy()
    r = oracle.replicate_branches(kc, vc, table, [20, 30, 40], [10, 10, 10], 4, free[:11])   # needs 4 * 3 blocks
    assert r["n_taken"] == 0 and r["status"].tolist() == [oracle.BRANCH_NO_BLOCKS] * 3
    assert np.all(r["branch_table"] == -1) and np.array_equal(kc, k0)
    bad = table.copy()
    bad[1, 0] = kc.shape[1]                               # a committed block outside the pool
    r = oracle.replicate_branches(kc, vc, bad, [20, 30, 40], [10, 400, 10], 2, free)
    assert r["status"].tolist() == [0, oracle.COMMIT_CAPACITY, 0]
    r = oracle.replicate_branches(kc, vc, bad, [20, 30, -1], [10, 10, 10], 2, free)
    assert r["status"].tolist() == [0, oracle.COMMIT_BAD_BLOCK, oracle.COMMIT_BAD_LEN]
    # the accounting follows the lengths alone: the sequence refused for its table keeps its share (2 x 2 blocks),
    # the one refused for its length has none
    assert r["n_taken"] == 2 + 4 and r["block_base"].tolist() == [0, 2, 6] and np.all(r["branch_table"][1:] == -1)
    good = oracle.replicate_branches(kc.copy(), vc.copy(), table, [20, 30, 40], [10, 10, 10], 2, free)
    worse = oracle.replicate_branches(kc.copy(), vc.copy(), bad, [20, 30, 40], [10, 10, 10], 2, free)
    assert np.array_equal(good["block_base"], worse["block_base"]) and good["n_taken"] == worse["n_taken"]
    assert np.array_equal(good["branch_table"][[0, 2]], worse["branch_table"][[0, 2]])
    f2 = free.copy()
    f2[1] = -3
    r = oracle.replicate_branches(kc.copy(), vc, table, [20, 30, 40], [10, 10, 10], 2, f2)
    assert r["status"].tolist() == [oracle.BRANCH_BAD_FREE, 0, 0] and np.all(r["branch_table"][0] == -1)


def test_commit_on_a_replica_equals_commit_on_a_deep_copy():
    """Replicate, let the teacher pass write the tree rows into branch i's tail, compact in place: the branch then
    reads exactly like a deep copy of the main cache that went through the same steps (commit equivalence)."""
    rng = np.random.default_rng(74)
    B, N, T = 3, 2, 9
    P = [21, 16, 40]
    kc, vc, table, free = _pool(rng, B, P, T)
    deep_k, deep_v = kc.copy(), vc.copy()
    r = oracle.replicate_branches(kc, vc, table, P, [T] * B, N, free)
    bt = r["branch_table"]
    kt = synth._values(rng, (2, B, T, 2, 8), "bf16")
    vt = synth._values(rng, (2, B, T, 2, 8), "bf16")
    acc = np.asarray([[0, 2, 5, 8] + [0] * 5, [0, 1, 2, 3] + [0] * 5, [0, 7, 8, 0] + [0] * 5], dtype=np.int32)
    A = [3, 3, 2]
    sel = 1
    for b in range(B):
        for j in range(T):
            pos = P[b] + j
            for cache, tree in ((kc, kt), (vc, vt)):
                cache[:, bt[b, sel, pos // BS], :, pos % BS] = tree[:, b, j]
    cap = [(p + T + BS - 1) // BS * BS for p in P]
    oracle.commit_accepted_kv(None, None, kc, vc, P, cap, [T] * B, acc, A, block_table=bt[:, sel].copy(), T_max=T)
    oracle.commit_accepted_kv(kt, vt, deep_k, deep_v, P, cap, [T] * B, acc, A, block_table=table)
    for b in range(B):
        L = P[b] + A[b] + 1
        assert np.array_equal(logical(kc, bt[b, sel], L), logical(deep_k, table[b], L))
        assert np.array_equal(logical(vc, bt[b, sel], L), logical(deep_v, table[b], L))


# ----------------------------------------------------------------------------------------------------------------
# commit by path indices
# ----------------------------------------------------------------------------------------------------------------
def _two_tables(rng, B, Ls, Ln, **kw):
    """One pool; the source tables hold Ls rows, the destination tables own other blocks for Ln rows."""
    kc, vc, table, free = _pool(rng, B, Ls, 0, spare=sum((n + BS - 1) // BS for n in Ln) + 7, **kw)
    dst = np.full((B, max(table.shape[1], max((n + BS - 1) // BS for n in Ln))), -1, dtype=np.int32)
    src = np.full_like(dst, -1)
    src[:, :table.shape[1]] = table
    at = 0
    for b in range(B):
        nb = (Ln[b] + BS - 1) // BS
        dst[b, :nb] = free[at:at + nb]
        at += nb
    return kc, vc, src, dst


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("fast", [False, True])
def test_full_reorder_is_the_gather_along_the_sequence_axis(dtype, fast):
    rng = np.random.default_rng(75)
    B, Ls, Ln = 4, [50, 33, 16, 7], [40, 60, 0, 7]
    kc, vc, src, dst = _two_tables(rng, B, Ls, Ln, dtype=dtype)
    k0, v0, dst0 = kc.copy(), vc.copy(), dst.copy()
    idx = np.zeros((B, 64), dtype=np.int32)
    idx[0, :40] = rng.permutation(50)[:40]               # a permutation: nothing of the prefix is preserved
    idx[1, :60] = rng.integers(0, 33, size=60)           # repeats, longer than the source
    idx[3, :7] = np.arange(7)[::-1]
    r = oracle.commit_path_indices(kc, vc, kc, vc, idx, Ls, Ln, src_table=src, dst_table=dst, fast=fast)
    assert np.all(r["status"] == 0)
    for b in range(B):
        keep = int(r["kept_len"][b])
        assert keep % BS == 0 and np.array_equal(idx[b, :keep], np.arange(keep))
        assert np.array_equal(logical(kc, dst[b], Ln[b]), logical(k0, src[b], Ls[b])[:, idx[b, :Ln[b]]])
        assert np.array_equal(logical(vc, dst[b], Ln[b]), logical(v0, src[b], Ls[b])[:, idx[b, :Ln[b]]])
        assert np.array_equal(logical(kc, src[b], Ls[b]), logical(k0, src[b], Ls[b]))   # the branch is not mutated
    if not fast:
        assert np.all(r["kept_len"] == 0) and np.array_equal(dst, dst0)
    own = np.unique(dst0[dst0 >= 0])
    rest = np.setdiff1d(np.arange(kc.shape[1]), own)
    assert np.array_equal(kc[:, rest], k0[:, rest]) and np.array_equal(vc[:, rest], v0[:, rest])


def test_contiguous_full_reorder():
    rng = np.random.default_rng(76)
    B, cap = 3, 40
    sk, sv = synth._values(rng, (2, B, cap, 2, 8), "bf16"), synth._values(rng, (2, B, cap, 2, 8), "bf16")
    dk, dv = synth._values(rng, sk.shape, "bf16"), synth._values(rng, sk.shape, "bf16")
    d0 = dk.copy()
    idx = rng.integers(0, 30, size=(B, 40)).astype(np.int32)
    Ln = [40, 11, 0]
    r = oracle.commit_path_indices(sk, sv, dk, dv, idx, [30, 30, 30], Ln, fast=True)
    assert np.all(r["status"] == 0) and np.all(r["kept_len"] == 0)
    for b in range(B):
        assert np.array_equal(dk[:, b, :Ln[b]], sk[:, b, idx[b, :Ln[b]]])
        assert np.array_equal(dv[:, b, :Ln[b]], sv[:, b, idx[b, :Ln[b]]])
        assert np.array_equal(dk[:, b, Ln[b]:], d0[:, b, Ln[b]:])


@pytest.mark.parametrize("fast", [False, True])
def test_path_index_commit_of_an_accepted_path_equals_the_length_based_commit(fast):
    """path_indices = [0..P) then P + accepted nodes: the rebuilt cache reads like the in-place compaction of the
    same branch (itself pinned to sequential appends), and the fast path shares every whole block of the prefix."""
    rng = np.random.default_rng(77)
    B, T = 3, 10
    P = [37, 32, 9]
    Ls = [p + T for p in P]
    acc = np.asarray([[0, 3, 4, 9], [0, 1, 5, 0], [0, 2, 0, 0]], dtype=np.int32)
    A = [3, 2, 1]
    Ln = [P[b] + A[b] + 1 for b in range(B)]
    kc, vc, src, dst = _two_tables(rng, B, Ls, Ln)
    k0, dst0 = kc.copy(), dst.copy()
    idx = np.zeros((B, 64), dtype=np.int32)
    for b in range(B):
        idx[b, :P[b]] = np.arange(P[b])
        idx[b, P[b]:Ln[b]] = P[b] + acc[b, :A[b] + 1]
    r = oracle.commit_path_indices(kc, vc, kc, vc, idx, Ls, Ln, src_table=src, dst_table=dst, fast=fast)
    ref_k, ref_v = k0.copy(), vc.copy()
    cap = [src.shape[1] * BS] * B
    accw = np.zeros((B, T), dtype=np.int32)
    accw[:, :4] = acc
    rr = oracle.commit_accepted_kv(None, None, ref_k, ref_v, P, cap, [T] * B, accw, A, block_table=src.copy(), T_max=T)
    assert np.all(rr["status"] == 0) and np.all(r["status"] == 0)
    for b in range(B):
        assert np.array_equal(logical(kc, dst[b], Ln[b]), logical(ref_k, src[b], Ln[b]))
        assert np.array_equal(logical(vc, dst[b], Ln[b]), logical(ref_v, src[b], Ln[b]))
        nshared = P[b] // BS if fast else 0
        assert int(r["kept_len"][b]) == nshared * BS
        assert np.array_equal(dst[b, :nshared], src[b, :nshared])
        assert np.array_equal(dst[b, nshared:], dst0[b, nshared:])
        for blk in dst0[b, :nshared]:                     # blocks the fast path did not need stay untouched
            assert np.array_equal(kc[:, blk], k0[:, blk])


def test_fast_path_falls_back_where_the_prefix_order_breaks():
    rng = np.random.default_rng(78)
    Ls = [70, 70, 70]
    kc, vc, src, dst = _two_tables(rng, 3, Ls, Ls)
    k0 = kc.copy()
    idx = np.tile(np.arange(70, dtype=np.int32), (3, 1))
    idx[0, [40, 41]] = [41, 40]                           # order breaks in the third block: two blocks kept
    idx[1, 0] = 1                                         # breaks at once: full reorder
    r = oracle.commit_path_indices(kc, vc, kc, vc, idx, Ls, Ls, src_table=src, dst_table=dst, fast=True)
    assert r["kept_len"].tolist() == [32, 0, 64] and np.all(r["status"] == 0)
    for b in range(3):
        assert np.array_equal(logical(kc, dst[b], 70), logical(k0, src[b], 70)[:, idx[b]])


def test_path_index_failures_write_nothing():
    rng = np.random.default_rng(79)
    Ls = [30, 30, 30, 30]
    kc, vc, src, dst = _two_tables(rng, 4, Ls, [30, 30, 30, 30])
    k0, dst0 = kc.copy(), dst.copy()
    idx = np.tile(np.arange(32, dtype=np.int32), (4, 1))
    idx[0, 5] = 30                                        # one past the branch cache
    idx[1, 0] = -1
    bad = dst.copy()
    bad[3, 1] = -1                                        # the destination has no second block
    r = oracle.commit_path_indices(kc, vc, kc, vc, idx, Ls, [30, 30, 33, 30], src_table=src, dst_table=bad, fast=True)
    assert r["status"].tolist() == [oracle.COMMIT_BAD_NODE, oracle.COMMIT_BAD_NODE, oracle.COMMIT_BAD_LEN,
                                    oracle.COMMIT_BAD_BLOCK]
    assert np.array_equal(kc, k0) and np.array_equal(bad[:3], dst0[:3]) and np.all(r["kept_len"] == 0)
    wide = np.zeros((4, 40), dtype=np.int32)              # indices fit, the destination's two blocks do not
    r = oracle.commit_path_indices(kc, vc, kc, vc, wide, Ls, [33] * 4, src_table=src, dst_table=dst)
    assert r["status"].tolist() == [oracle.COMMIT_CAPACITY] * 4 and np.array_equal(kc, k0)
