"""Pins for the ancestor mask: brute-force walk in the oracle vs. an
independent bitmask recurrence, on every tree of up to 6 nodes and on random
trees up to 128 nodes; plus the shapes the mask must have on special trees."""
import json
import os

import numpy as np

from paper_2505_23219_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def mask_by_recurrence(parent):
    M = len(parent)
    anc = [0] * M
    for i in range(M):
        anc[i] = (anc[parent[i]] if parent[i] >= 0 else 0) | (1 << i)
    return np.array([[(anc[i] >> j) & 1 for j in range(M)] for i in range(M)], dtype=np.uint8)


def test_mask_all_small_trees(orc32):
    count = 0
    for M in range(1, 7):
        for parent in wl.all_trees(M):
            assert orc32.tree_validate(parent)
            assert np.array_equal(orc32.tree_mask(parent), mask_by_recurrence(parent)), parent
            count += 1
    assert count == 1 + 1 + 2 + 6 + 24 + 120


def test_mask_random_trees_and_counts(orc32):
    for M, depth, seed in ((8, 3, 0), (16, 4, 1), (64, 5, 2), (128, 5, 3), (128, 127, 4)):
        parent = wl.tree_random(M, depth, seed)
        mask = orc32.tree_mask(parent)
        assert np.array_equal(mask, mask_by_recurrence(parent))
        d = orc32.tree_depth(parent)
        assert d.max() <= depth
        assert np.array_equal(mask.sum(axis=1), d + 1)       # row i has depth+1 ones
        assert np.all(np.triu(mask, 1) == 0)                 # nothing above the diagonal
        assert np.all(mask[:, 0] == 1) and np.all(np.diag(mask) == 1)


def test_mask_special_shapes(orc32):
    M = 9
    assert np.array_equal(orc32.tree_mask(wl.tree_chain(M)), np.tril(np.ones((M, M), np.uint8)))
    star = orc32.tree_mask(wl.tree_star(M))
    want = np.eye(M, dtype=np.uint8)
    want[:, 0] = 1
    assert np.array_equal(star, want)
    assert np.array_equal(orc32.tree_mask([-1]), [[1]])


def test_validate_rejects_bad_trees(orc32):
    assert not orc32.tree_validate([0])
    assert not orc32.tree_validate([-1, 1])          # self / forward reference
    assert not orc32.tree_validate([-1, 0, 3, 1])
    assert not orc32.tree_validate([-1, -1])
    assert orc32.tree_validate([-1, 0, 0, 2])


def test_paper_worked_example_width(orc32):
    """Section 2.3: with two candidates from the first head and three from the
    second, the paper's verification tree has width 8 (drafted nodes)."""
    with open(os.path.join(GOLDEN, "medusa_example_width.json")) as f:
        gold = json.load(f)
    parent = wl.tree_product(gold["candidates_per_head"])
    assert len(parent) - 1 == gold["verification_width"]
    mask = orc32.tree_mask(parent)
    # every drafted node sees the root and itself; second-level nodes also their parent
    assert int(mask[1:, 1:].sum()) == 2 * 1 + 6 * 2


def test_workload_trees_match_their_recipes(orc32):
    w = wl.workload("layer7b")
    assert len(w.parent) == 16 and orc32.tree_validate(w.parent)
    assert orc32.tree_depth(w.parent).max() <= 4
    w = wl.workload("stack7b")
    assert len(w.parent) == 64 and orc32.tree_depth(w.parent).max() <= 5
    w = wl.workload("stack13b")
    d = orc32.tree_depth(w.parent)
    assert len(w.parent) == 64 and d.max() == 2 and (d == 1).sum() == 32
    assert int(orc32.tree_mask(w.parent).sum()) == 1 + 2 * 32 + 3 * 31
    w = wl.workload("tiny")
    assert len(w.parent) == 8 and orc32.tree_depth(w.parent).max() <= 3
    # the committed fixtures pin the tree shapes independently of the RNG library
    with open(os.path.join(GOLDEN, "workload_trees.json")) as f:
        gold = json.load(f)
    for name, parent in gold.items():
        assert list(map(int, wl.workload(name).parent)) == parent, name
