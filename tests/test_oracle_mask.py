"""Pins for the oracle's tree mask: brute-force ancestor walk, closed-form shapes,
popcount = depth + 1, the hand-worked example, and the structural invariants."""
import numpy as np
import pytest

import oracle
from paper_2603_08088_amd import synth
from helpers import brute_mask, golden, random_tree


def _unpack(bitmask, T):
    B, Tm, words = bitmask.shape
    out = np.zeros((B, Tm, T), dtype=np.uint8)
    for j in range(T):
        out[:, :, j] = ((bitmask[:, :, j // 64] >> np.uint64(j % 64)) & np.uint64(1)).astype(np.uint8)
    return out


@pytest.mark.parametrize("T", [1, 2, 7, 15, 60, 64, 65, 128])
def test_mask_equals_brute_force_walk(T):
    rng = np.random.default_rng(T)
    B = 5
    parents = np.stack([random_tree(rng, T) for _ in range(B)])
    n = np.full(B, T, dtype=np.int32)
    r = oracle.build_tree_mask(parents, n)
    for b in range(B):
        bm = brute_mask(parents[b], T)
        assert np.array_equal(r["dense"][b, 0], bm)
        assert np.array_equal(r["depth"][b], synth.node_depths(parents[b]))
        assert np.array_equal(r["dense"][b, 0].sum(axis=1), r["depth"][b] + 1)      # popcount = depth+1
        assert np.all(r["dense"][b, 0][:, 0] == 1)                                   # root visible to all
    assert np.array_equal(_unpack(r["bitmask"], T), r["dense"][:, 0])
    assert np.all(r["status"] == 0)


def test_chain_is_lower_triangular_and_star_is_col0_plus_diag():
    T = 33
    r = oracle.build_tree_mask(np.stack([synth.tree_chain(T), synth.tree_star(T)]), [T, T])
    assert np.array_equal(r["dense"][0, 0], np.tril(np.ones((T, T), dtype=np.uint8)))
    star = np.eye(T, dtype=np.uint8)
    star[:, 0] = 1
    assert np.array_equal(r["dense"][1, 0], star)
    assert np.array_equal(r["depth"][0], np.arange(T))


def test_worked_example():
    ex = golden("worked_example.json")
    par = np.asarray([ex["parent"]], dtype=np.int32)
    r = oracle.build_tree_mask(par, [7])
    assert r["depth"][0].tolist() == ex["depth"]
    assert r["bitmask"][0, :, 0].tolist() == ex["bitmask_words"]
    for k, vis in enumerate(ex["visible"]):
        assert np.flatnonzero(r["dense"][0, 0, k]).tolist() == vis
    # the ancestor table of the example, retyped from the recursion by hand, gives the same visible sets
    A = np.asarray(ex["ancestor_table"])
    for k in range(7):
        assert sorted(set(A[:, k].tolist())) == ex["visible"][k]


def test_padding_rows_and_columns_are_zero():
    rng = np.random.default_rng(3)
    T_max, n = 20, 11
    par = np.zeros((1, T_max), dtype=np.int32)
    par[0, :n] = random_tree(rng, n)
    par[0, n:] = 0
    r = oracle.build_tree_mask(par, [n])
    assert r["dense"][0, 0, n:, :].sum() == 0 and r["dense"][0, 0, :, n:].sum() == 0
    assert np.array_equal(r["dense"][0, 0, :n, :n], brute_mask(par[0, :n], n))
    assert r["status"][0] == 0


def test_invariant_violations_are_flagged_and_mask_stays_defined():
    T = 8
    good = np.asarray([0, 0, 1, 1, 2, 2, 3, 3], dtype=np.int32)
    # out-of-range parent
    bad = good.copy(); bad[5] = 99
    r = oracle.build_tree_mask(bad[None], [T])
    assert r["status"][0] & oracle.TREE_RANGE
    fixed = good.copy(); fixed[5] = 0
    assert np.array_equal(r["dense"][0, 0], brute_mask(fixed, T))
    bad = good.copy(); bad[5] = -1
    assert oracle.build_tree_mask(bad[None], [T])["status"][0] & oracle.TREE_RANGE
    # cycle 4 -> 6 -> 4, node 7 hangs off the cycle
    bad = good.copy(); bad[4] = 6; bad[6] = 4; bad[7] = 6
    r = oracle.build_tree_mask(bad[None], [T])
    assert r["status"][0] & oracle.TREE_CYCLE
    fixed = good.copy(); fixed[4] = 0; fixed[6] = 0; fixed[7] = 0
    assert np.array_equal(r["dense"][0, 0], brute_mask(fixed, T))
    assert r["depth"][0].tolist() == [0, 1, 2, 2, 1, 3, 1, 1]
    # self loop
    bad = good.copy(); bad[3] = 3
    assert oracle.build_tree_mask(bad[None], [T])["status"][0] & oracle.TREE_CYCLE
    # valid child of an invalid (padded) parent slot
    par = np.zeros((1, 10), dtype=np.int32); par[0, :T] = good; par[0, 4] = 9
    r = oracle.build_tree_mask(par, [T])
    assert r["status"][0] == oracle.TREE_CLOSURE
    # non-topological but valid order is accepted (only depth consistency is required)
    perm = np.asarray([0, 2, 0, 1], dtype=np.int32)   # 2 child of root, 1 child of 2, 3 child of 1
    r = oracle.build_tree_mask(perm[None], [4])
    assert r["status"][0] == 0 and r["depth"][0].tolist() == [0, 2, 1, 3]
    assert np.array_equal(r["dense"][0, 0], brute_mask(perm, 4))


def test_generated_workload_trees_satisfy_invariants():
    for wl in (synth.config1(), synth.config2(with_cache=False, with_logits=False),
               synth.config4(with_cache=False, with_logits=False),
               synth.config5(64, 10, B=2, with_cache=False, with_logits=False)):
        r = oracle.build_tree_mask(wl.parent, wl.n_nodes)
        assert np.all(r["status"] == 0)
        for b in range(wl.B):
            n = int(wl.n_nodes[b])
            assert np.all(wl.parent[b, 1:n] < np.arange(1, n))
            assert r["depth"][b].max() <= wl.W - 1
