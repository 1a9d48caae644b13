"""Pins for the oracle's tree tensorization (depth, position ids, root-to-leaf path table): the hand-worked
example, closed-form shapes (chain, star, complete binary tree), brute-force parent walks on random trees,
structural properties that hold for any tree, the overflow bits, and agreement with the mask builder on
trees that break an invariant."""
import numpy as np
import pytest

import oracle
from paper_2603_08088_amd import synth
from helpers import golden, path_to, random_tree


def test_worked_example():
    ex = golden("worked_example.json")
    par = np.asarray([ex["parent"]], dtype=np.int32)
    r = oracle.tensorize_tree(par, [7], [100], L_max=4, W=4)
    assert r["depth"][0].tolist() == ex["depth"]
    assert r["position_ids"][0].tolist() == [100 + d for d in ex["depth"]]
    assert r["n_paths"][0] == 3 and r["status"][0] == 0
    assert r["retrieve"][0, :3].tolist() == ex["retrieve"]
    assert r["retrieve"][0, 3].tolist() == [-1] * 4
    # the rows are columns of the hand-written ancestor table read bottom-up: entry i = A[depth - i][leaf]
    A = np.asarray(ex["ancestor_table"])
    for row in r["retrieve"][0, :3]:
        nodes = [x for x in row.tolist() if x >= 0]
        leaf, d = nodes[-1], len(nodes) - 1
        assert nodes == [int(A[d - i, leaf]) for i in range(d + 1)]


def test_chain_star_and_complete_binary_tree():
    T = 17
    r = oracle.tensorize_tree(np.stack([synth.tree_chain(T), synth.tree_star(T)]), [T, T], [5, 9], L_max=T, W=T)
    # chain: one path 0..T-1, depth k, position P + k
    assert r["n_paths"].tolist() == [1, T - 1]
    assert r["retrieve"][0, 0].tolist() == list(range(T))
    assert np.all(r["retrieve"][0, 1:] == -1)
    assert r["position_ids"][0].tolist() == [5 + k for k in range(T)]
    # star: T-1 paths [0, k], every non-root node at depth 1
    for k in range(1, T):
        assert r["retrieve"][1, k - 1].tolist() == [0, k] + [-1] * (T - 2)
    assert r["position_ids"][1].tolist() == [9] + [10] * (T - 1)
    # complete binary tree in heap order: 2^D leaves, leaf k's path is its heap ancestors
    D = 4
    n = 2 ** (D + 1) - 1
    heap = np.asarray([0] + [(k - 1) // 2 for k in range(1, n)], dtype=np.int32)
    r = oracle.tensorize_tree(heap[None], [n], [0], L_max=2 ** D, W=D + 1)
    assert r["n_paths"][0] == 2 ** D and r["status"][0] == 0
    for i, leaf in enumerate(range(2 ** D - 1, n)):
        want, k = [], leaf
        while True:
            want.append(k)
            if k == 0:
                break
            k = (k - 1) // 2
        assert r["retrieve"][0, i].tolist() == want[::-1]
    assert r["depth"][0].tolist() == [int(np.floor(np.log2(k + 1))) for k in range(n)]


@pytest.mark.parametrize("T", [1, 2, 3, 8, 31, 60, 64, 65, 128])
def test_random_trees_against_parent_walks_and_properties(T):
    rng = np.random.default_rng(40 + T)
    B = 6
    parents = np.stack([random_tree(rng, T) for _ in range(B)])
    n = np.asarray([T, max(1, T // 2), 1, T, max(1, T - 1), 0], dtype=np.int32)
    P = rng.integers(0, 5000, size=B).astype(np.int32)
    # a padded tree must behave like the tree cut to its valid rows; make the cut closed under `parent`
    for b in range(B):
        for k in range(1, T):
            if parents[b, k] >= max(1, n[b]):
                parents[b, k] = 0
    r = oracle.tensorize_tree(parents, n, P, L_max=T, W=T)
    assert np.all(r["status"] == 0)
    for b in range(B):
        nb = int(n[b])
        par = parents[b]
        leaves = [k for k in range(nb) if not any(par[j] == k for j in range(1, nb))]
        assert r["n_paths"][b] == len(leaves)
        for i, leaf in enumerate(leaves):                       # ascending leaf order, brute-force walk
            want = path_to(par, leaf)
            assert r["retrieve"][b, i, :len(want)].tolist() == want
            assert np.all(r["retrieve"][b, i, len(want):] == -1)
        assert np.all(r["retrieve"][b, len(leaves):] == -1)
        seen = set()
        for i in range(len(leaves)):                            # properties that hold for any tree
            row = [x for x in r["retrieve"][b, i].tolist() if x >= 0]
            assert row[0] == 0
            assert all(par[row[j]] == row[j - 1] for j in range(1, len(row)))
            assert [int(r["depth"][b, x]) for x in row] == list(range(len(row)))
            seen.update(row)
        assert seen == set(range(nb))                           # every valid node lies on some path
        assert r["depth"][b, nb:].tolist() == [0] * (T - nb)
        assert r["position_ids"][b].tolist() == [int(P[b]) + int(d) for d in r["depth"][b]]
        if nb:
            assert np.array_equal(r["retrieve"][b, :len(leaves)], synth.build_retrieve(par[:nb], T)[:, :T])


def test_overflow_bits_keep_the_first_rows_and_columns():
    par = np.asarray([[0, 0, 1, 2, 3, 0, 0, 0]], dtype=np.int32)   # chain 0-1-2-3-4 plus leaves 5, 6, 7
    full = oracle.tensorize_tree(par, [8], [0], L_max=8, W=8)
    assert full["n_paths"][0] == 4 and full["status"][0] == 0
    few = oracle.tensorize_tree(par, [8], [0], L_max=2, W=8)
    assert few["status"][0] == 8 and few["n_paths"][0] == 2
    assert np.array_equal(few["retrieve"][0], full["retrieve"][0, :2])
    narrow = oracle.tensorize_tree(par, [8], [0], L_max=8, W=3)
    assert narrow["status"][0] == 16 and narrow["n_paths"][0] == 4
    assert np.array_equal(narrow["retrieve"][0], full["retrieve"][0, :, :3])
    exact = oracle.tensorize_tree(par, [8], [0], L_max=4, W=5)
    assert exact["status"][0] == 0


def test_broken_trees_agree_with_the_mask_builder():
    # parent out of range, parent in the padding, a 2-cycle, a self-loop, a bad root entry
    par = np.asarray([[0, 0, 9, 1, 5, 4, 7, 6, 8],
                      [3, 0, 1, 1, 2, 2, 2, 2, 2]], dtype=np.int32)
    n = [9, 6]
    r = oracle.tensorize_tree(par, n, [0, 0], L_max=9, W=9)
    m = oracle.build_tree_mask(par, n)
    assert np.array_equal(r["depth"], m["depth"])
    assert np.array_equal(r["status"] & 7, m["status"])
    assert np.all(m["status"] != 0)
    for b in range(2):                                          # the paths follow the repaired tree: the mask says the same
        for i in range(int(r["n_paths"][b])):
            row = [x for x in r["retrieve"][b, i].tolist() if x >= 0]
            assert np.flatnonzero(m["dense"][b, 0, row[-1]]).tolist() == sorted(row)
