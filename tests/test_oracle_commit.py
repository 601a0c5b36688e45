"""Pins for the oracle's commit of the accepted path.

After a verification pass the cache holds one K/V row per tree node (row
kv_len + i for node i); committing the accepted root path must leave the cache in
exactly the state that feeding the accepted tokens one after the other would have
produced.  That state is computed here without the commit routine: the same stack run
on a chain made of the accepted nodes' inputs.
"""
import numpy as np
import pytest

from paper_2505_23219_amd import workloads as wl

SHAPE = wl.ModelShape("mini", H=64, nh=4, d=16, F=88, V=50, L=2)


def model(seed):
    layers = [{k: v.numpy() for k, v in wl.layer_weights(SHAPE, seed, l).items()} for l in range(SHAPE.L)]
    return layers


def caches(cap, kv_len, seed):
    ks, vs = [], []
    for l in range(SHAPE.L):
        k, v = wl.kv_cache(SHAPE, cap, kv_len, seed, l)
        ks.append(k.numpy().copy())
        vs.append(v.numpy().copy())
    return ks, vs


def root_path(parent, node):
    path = []
    while node >= 0:
        path.append(node)
        node = int(parent[node])
    return np.array(path[::-1], dtype=np.int32)


@pytest.mark.parametrize("seed,M,leaf", [(1, 8, 7), (2, 12, 5), (3, 12, 11), (4, 6, 0)])
def test_commit_equals_feeding_the_accepted_tokens_in_sequence(orc32, seed, M, leaf):
    kv_len, cap = 21, 64
    parent = wl.tree_random(M, 4, seed)
    layers = model(seed)
    x16 = wl.activations(M, SHAPE.H, seed).numpy()
    path = root_path(parent, leaf)
    # tree pass, then commit
    kt, vt = caches(cap, kv_len, seed)
    orc32.verify_stack(SHAPE, layers, kt, vt, None, x16, parent, kv_len, True)
    for l in range(SHAPE.L):
        orc32.commit_path(kt[l], vt[l], kv_len, path)
    # the accepted tokens alone, as a chain, on a fresh copy of the cache
    kc, vc = caches(cap, kv_len, seed)
    orc32.verify_stack(SHAPE, layers, kc, vc, None, x16[path], wl.tree_chain(len(path)), kv_len, True)
    n = kv_len + len(path)
    for l in range(SHAPE.L):
        assert np.array_equal(kt[l].view(np.uint16)[:, :n], kc[l].view(np.uint16)[:, :n]), l
        assert np.array_equal(vt[l].view(np.uint16)[:, :n], vc[l].view(np.uint16)[:, :n]), l


def test_commit_of_a_fully_accepted_chain_changes_nothing(orc32):
    kv_len, cap, M = 10, 64, 9
    rng = np.random.default_rng(0)
    k = rng.integers(0, 0x7bff, size=(SHAPE.nh, cap, SHAPE.d)).astype(np.uint16)
    v = rng.integers(0, 0x7bff, size=(SHAPE.nh, cap, SHAPE.d)).astype(np.uint16)
    k0, v0 = k.copy(), v.copy()
    orc32.commit_path(k, v, kv_len, np.arange(M, dtype=np.int32))
    assert np.array_equal(k, k0) and np.array_equal(v, v0)


def test_commit_moves_exactly_the_path_rows(orc32):
    """Row kv_len + j takes the old row kv_len + path[j]; committed rows and rows past the
    accepted length stay."""
    kv_len, cap = 5, 32
    rng = np.random.default_rng(1)
    k = rng.integers(0, 0x7bff, size=(2, cap, 8)).astype(np.uint16)
    v = rng.integers(0, 0x7bff, size=(2, cap, 8)).astype(np.uint16)
    k0, v0 = k.copy(), v.copy()
    path = np.array([0, 2, 3, 9], dtype=np.int32)
    orc32.commit_path(k, v, kv_len, path)
    for j, node in enumerate(path):
        assert np.array_equal(k[:, kv_len + j], k0[:, kv_len + node])
        assert np.array_equal(v[:, kv_len + j], v0[:, kv_len + node])
    assert np.array_equal(k[:, :kv_len], k0[:, :kv_len])
    assert np.array_equal(k[:, kv_len + len(path):], k0[:, kv_len + len(path):])
    assert np.array_equal(v[:, kv_len + len(path):], v0[:, kv_len + len(path):])
