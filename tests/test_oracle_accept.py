"""Pins for greedy acceptance: the oracle's validity propagation vs. a brute
force that enumerates every node's root path and tests every edge on it."""
import itertools

import numpy as np

from paper_2505_23219_amd import workloads as wl


def brute_force_accept(logits, tokens, parent):
    M = len(parent)
    amax = [int(np.flatnonzero(row == row.max())[0]) for row in logits]
    best = [0]
    for node in range(M):
        path = []
        j = node
        while j >= 0:
            path.append(j)
            j = int(parent[j])
        path = path[::-1]
        ok = all(tokens[c] == amax[p] for p, c in zip(path[:-1], path[1:]))
        if ok and len(path) > len(best):
            best = path
    return len(best), amax[best[-1]], best, amax


def test_width_one_accepts_one(orc32):
    """Table 1: at verification width 1 the acceptance length is 1."""
    logits = np.array([[0.1, 0.7, 0.3]], dtype=np.float32)
    n, nxt, path, amax = orc32.accept_greedy(logits, [2], [-1])
    assert (n, nxt, list(path), list(amax)) == (1, 1, [0], [1])


def test_all_small_trees_all_edge_patterns(orc32):
    rng = np.random.default_rng(0)
    V = 7
    checked = 0
    for M in range(1, 6):
        for parent in wl.all_trees(M):
            logits = rng.standard_normal((M, V)).astype(np.float32)
            amax = logits.argmax(axis=1)
            for pattern in itertools.product((0, 1), repeat=M - 1):
                tokens = np.zeros(M, dtype=np.int32)
                for c in range(1, M):
                    good = int(amax[parent[c]])
                    tokens[c] = good if pattern[c - 1] else (good + 1 + c) % V
                    if tokens[c] == good and not pattern[c - 1]:
                        tokens[c] = (good + 1) % V
                n, nxt, path, am = orc32.accept_greedy(logits, tokens, parent)
                bn, bnxt, bpath, bam = brute_force_accept(logits, tokens, parent)
                assert (n, nxt, list(path), list(am)) == (bn, bnxt, bpath, bam)
                checked += 1
    assert checked == 1 + 2 + 2 * 4 + 6 * 8 + 24 * 16


def test_planted_paths_of_every_length(orc32):
    rng = np.random.default_rng(1)
    M, V = 40, 300
    parent = wl.tree_random(M, 6, 11)
    depth = orc32.tree_depth(parent)
    logits = rng.standard_normal((M, V)).astype(np.float32)
    amax = logits.argmax(axis=1)
    for target in range(M):
        tokens = np.full(M, -1, dtype=np.int32)           # -1 never matches
        j = target
        while parent[j] >= 0:
            tokens[j] = amax[parent[j]]
            j = parent[j]
        n, nxt, path, _ = orc32.accept_greedy(logits, tokens, parent)
        assert n == depth[target] + 1 and path[-1] == target and nxt == amax[target]
        assert list(path) == brute_force_accept(logits, tokens, parent)[2]


def test_duplicate_siblings_and_ties(orc32):
    # two children of the root carry the same (matching) token; only the second
    # one has a matching child: the deeper path through the second must win.
    parent = np.array([-1, 0, 0, 2], dtype=np.int32)
    logits = np.zeros((4, 5), dtype=np.float32)
    logits[0, 3] = 1.0      # root predicts 3
    logits[1, 1] = 1.0      # node 1 predicts 1 (no child)
    logits[2, 4] = 1.0      # node 2 predicts 4
    logits[3, 2] = 1.0
    tokens = np.array([0, 3, 3, 4], dtype=np.int32)
    n, nxt, path, _ = orc32.accept_greedy(logits, tokens, parent)
    assert (n, nxt, list(path)) == (3, 2, [0, 2, 3])
    # equal depth: lowest node index wins
    tokens = np.array([0, 3, 3, 0], dtype=np.int32)
    n, nxt, path, _ = orc32.accept_greedy(logits, tokens, parent)
    assert (n, nxt, list(path)) == (2, 1, [0, 1])
    # argmax ties resolve to the lowest index
    logits = np.zeros((1, 6), dtype=np.float32)
    logits[0, [2, 4]] = 5.0
    assert orc32.accept_greedy(logits, [0], [-1])[1] == 2
    # a valid child under an invalid parent is not accepted
    parent = np.array([-1, 0, 1], dtype=np.int32)
    logits = np.zeros((3, 4), dtype=np.float32)
    logits[0, 1] = logits[1, 2] = logits[2, 3] = 1.0
    n, _, path, _ = orc32.accept_greedy(logits, [0, 0, 2], parent)
    assert (n, list(path)) == (1, [0])
