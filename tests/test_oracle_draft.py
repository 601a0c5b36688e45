"""Pins for the oracle's drafting side: top-R, drafting-head logits, embedding, tree tokens,
tree design, and the decoding loop (drafting and verification never change the output).
"""
import itertools

import numpy as np
import pytest

from paper_2505_23219_amd import workloads as wl

SHAPE = wl.ModelShape("mini", H=64, nh=4, d=16, F=88, V=50, L=2)
EPS = 1e-5


# ---- top-R ---------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(4))
def test_topk_equals_a_stable_full_sort(orc32, seed):
    rng = np.random.default_rng(seed)
    v = rng.integers(-5, 6, size=(3, 40)).astype(np.float32)      # many ties
    got = orc32.topk(v, 7)
    for row in range(3):
        want = np.argsort(-v[row], kind="stable")[:7]              # ties: lowest index first
        assert np.array_equal(got[row], want)


def test_topk_of_distinct_values(orc32):
    rng = np.random.default_rng(9)
    v = rng.permutation(1000).astype(np.float32).reshape(2, 500)
    got = orc32.topk(v, 10)
    for row in range(2):
        assert np.array_equal(v[row][got[row]], np.sort(v[row])[::-1][:10])


# ---- head logits ------------------------------------------------------------------------------
def test_head_logits_are_rmsnorm_then_matmul(orc64):
    rng = np.random.default_rng(3)
    H, V, K = 32, 17, 3
    x = rng.standard_normal(H)
    g = (1 + 0.1 * rng.standard_normal(H)).astype(np.float16)
    W = (0.1 * rng.standard_normal((K * V, H))).astype(np.float16)
    got = orc64.draft_logits(x, g, W, K, EPS, False)
    n = x / np.sqrt(np.mean(x * x) + EPS) * g.astype(np.float64)
    want = (W.astype(np.float64) @ n).reshape(K, V)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_each_head_is_an_lm_head_of_its_own(orc32):
    """Head k of the stacked matrix gives exactly what the LM-head routine gives for rows
    k*V .. (k+1)*V (same normalisation, same rounding point)."""
    rng = np.random.default_rng(4)
    K = 2
    x = rng.standard_normal((1, SHAPE.H)).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(SHAPE.H)).astype(np.float16)
    W = (0.1 * rng.standard_normal((K * SHAPE.V, SHAPE.H))).astype(np.float16)
    got = orc32.draft_logits(x[0], g, W, K, SHAPE.rms_eps, True)
    for k in range(K):
        want = orc32.lm_head(SHAPE, g, W[k * SHAPE.V:(k + 1) * SHAPE.V], x, True)
        assert np.array_equal(got[k], want[0])


# ---- embedding, tree tokens ---------------------------------------------------------------------
def test_embed_is_a_row_gather(orc32):
    rng = np.random.default_rng(5)
    table = rng.integers(0, 0x7bff, size=(30, 16)).astype(np.uint16)
    tokens = rng.integers(0, 30, size=9)
    assert np.array_equal(orc32.embed(table, tokens), table[tokens])


def test_tree_tokens_worked_example(orc32):
    # root; 1, 2 children of the root (candidates 0, 1 of head 0); 3, 4 children of 1
    # (candidates 0, 1 of head 1); 5 child of 2 (candidate 0 of head 1); 6 child of 3 (head 2)
    parent = [-1, 0, 0, 1, 1, 2, 3]
    rank = [0, 0, 1, 0, 1, 0, 1]
    topk = np.array([[10, 11], [20, 21], [30, 31]])
    assert orc32.tree_tokens(parent, rank, topk, 7).tolist() == [7, 10, 11, 20, 21, 20, 31]


# ---- tree design (section 3.3.1) --------------------------------------------------------------
def expected_length(acc, nodes):
    """1 + sum of sequence accuracies; a node is the tuple of candidate ranks along its path."""
    return 1.0 + sum(np.prod([acc[t][r] for t, r in enumerate(seq)]) for seq in nodes)


def best_tree_by_enumeration(acc, M):
    K, R = acc.shape
    universe = [seq for t in range(1, K + 1) for seq in itertools.product(range(R), repeat=t)]
    best = -1.0
    for sub in itertools.combinations(universe, M - 1):
        s = set(sub)
        if all(len(seq) == 1 or seq[:-1] in s for seq in sub):       # closed under "parent"
            best = max(best, expected_length(acc, sub))
    return best


@pytest.mark.parametrize("K,R,M,seed", [(3, 2, 5, 0), (2, 3, 6, 1), (3, 2, 7, 2), (2, 3, 4, 3), (4, 2, 5, 4)])
def test_tree_design_reaches_the_best_expected_length(orc32, K, R, M, seed):
    rng = np.random.default_rng(seed)
    acc = np.sort(rng.uniform(0.05, 0.9, size=(K, R)), axis=1)[:, ::-1].copy()
    parent, rank, e = orc32.tree_build(acc, M)
    assert len(parent) == M and orc32.tree_validate(parent)
    # the tree as rank sequences; siblings have distinct ranks; depth never exceeds K
    seqs = [()]
    for i in range(1, M):
        seqs.append(seqs[parent[i]] + (int(rank[i]),))
    assert len(set(seqs)) == M and max(len(s) for s in seqs) <= K
    assert abs(e - expected_length(acc, seqs[1:])) < 1e-12
    assert abs(e - best_tree_by_enumeration(acc, M)) < 1e-12


def test_tree_design_with_one_candidate_per_head_is_a_chain(orc32):
    acc = np.array([[0.8], [0.5], [0.25]])
    parent, rank, e = orc32.tree_build(acc, 4)
    assert parent.tolist() == [-1, 0, 1, 2] and rank.tolist() == [0, 0, 0, 0]
    assert abs(e - (1 + 0.8 + 0.4 + 0.1)) < 1e-12
    # no candidates left after K levels: the tree stops at K + 1 nodes
    parent, rank, e = orc32.tree_build(acc, 9)
    assert len(parent) == 4


# ---- the loop: drafting and verification never change the produced tokens ------------------------
def model(seed):
    layers = [{k: v.numpy() for k, v in wl.layer_weights(SHAPE, seed, l).items()} for l in range(SHAPE.L)]
    head = {k: v.numpy() for k, v in wl.head_weights(SHAPE, seed).items()}
    table = wl.activations(SHAPE.V, SHAPE.H, seed, tag="embed").numpy()
    return layers, head, table


def caches(cap, kv_len, seed):
    ks, vs = [], []
    for l in range(SHAPE.L):
        k, v = wl.kv_cache(SHAPE, cap, kv_len, seed, l)
        ks.append(k.numpy().copy())
        vs.append(v.numpy().copy())
    return ks, vs


def sequential(orc, layers, head, table, kv_len, cap, seed, first_token, count):
    """Plain greedy decoding: one token per step."""
    kc, vc = caches(cap, kv_len, seed)
    out, tok = [], first_token
    for _ in range(count):
        st = orc.spec_step(SHAPE, layers, kc, vc, head, table, [tok], [-1], kv_len, True)
        assert st["n"] == 1
        tok = st["next_token"]
        out.append(tok)
        kv_len += 1
    return out


@pytest.mark.parametrize("seed", [1, 2])
def test_tree_decoding_with_head_drafts_equals_sequential_decoding(orc32, seed):
    layers, head, table = model(seed)
    K, R, M = 2, 3, 7
    Wheads = wl.activations(K * SHAPE.V, SHAPE.H, seed, tag="heads", std=0.1).numpy()
    acc = np.array([[0.6, 0.3, 0.1], [0.5, 0.2, 0.1]])
    parent, rank, _ = orc32.tree_build(acc, M)
    kv_len, cap = 9, 64
    want = sequential(orc32, layers, head, table, kv_len, cap, seed, 3, 12)
    kc, vc = caches(cap, kv_len, seed)
    rng = np.random.default_rng(seed)
    tokens = np.concatenate([[3], rng.integers(0, SHAPE.V, size=M - 1)]).astype(np.int32)
    got = []
    while len(got) < 12:
        st = orc32.spec_step(SHAPE, layers, kc, vc, head, table, tokens, parent, kv_len, True)
        got += st["produced"]
        kv_len += st["n"]
        tokens, _, _ = orc32.draft(st["x_last"], head["g_final"], Wheads, K, R, SHAPE.rms_eps, parent, rank,
                                   st["next_token"], True)
    assert got[:12] == want


@pytest.mark.parametrize("seed,planted", [(1, 3), (2, 2), (3, 4)])
def test_tree_decoding_with_planted_drafts_accepts_them_and_equals_sequential(orc32, seed, planted):
    """Drafts that are right along one root path are accepted to exactly that depth, and the
    output is still the sequential one."""
    layers, head, table = model(seed)
    M = 8
    parent = np.array([-1, 0, 0, 1, 1, 3, 5, 6], dtype=np.int32)      # path 0-1-3-5-6-7 and side nodes
    chain = [0, 1, 3, 5, 6, 7]
    kv_len, cap = 5, 64
    want = sequential(orc32, layers, head, table, kv_len, cap, seed, 11, 16 + M)
    kc, vc = caches(cap, kv_len, seed)
    got, tok = [], 11
    while len(got) < 16:
        tokens = np.full(M, -1, dtype=np.int32)
        tokens[0] = tok
        future = want[len(got):]
        for j in range(1, planted + 1):
            tokens[chain[j]] = future[j - 1]                       # the right continuation
        wrong = (np.array(future[:M]) + 1) % SHAPE.V               # never the right token
        for i in range(1, M):
            if tokens[i] < 0:
                tokens[i] = wrong[orc32.tree_depth(parent)[i] - 1]
        st = orc32.spec_step(SHAPE, layers, kc, vc, head, table, tokens, parent, kv_len, True)
        assert st["n"] == planted + 1 and st["path"].tolist() == chain[:planted + 1]
        got += st["produced"]
        kv_len += st["n"]
        tok = st["next_token"]
    assert got == want[:len(got)]


# ---- choice of the width (sections 3.3.1, 3.3.2) -------------------------------------------------
def test_width_choice_closed_forms(orc32):
    acc = np.array([[0.8], [0.5], [0.25]])          # one candidate per head: chains
    widths = [1, 2, 3, 4]
    expect = np.array([1.0, 1.8, 2.2, 2.3])
    # the same step time at every width: the widest tree wins
    i, rate = orc32.choose_width(acc, widths, [2.0] * 4)
    assert i == 3 and np.allclose(rate, expect / 2.0, rtol=0, atol=1e-15)
    # step time proportional to the width: one token at a time wins
    i, rate = orc32.choose_width(acc, widths, [1.0, 2.0, 3.0, 4.0])
    assert i == 0 and np.allclose(rate, expect / np.arange(1, 5), rtol=0, atol=1e-15)
    # a step that gets 10% slower per extra node: rates 1, 1.636, 1.833, 1.769
    i, rate = orc32.choose_width(acc, widths, [1.0, 1.1, 1.2, 1.3])
    assert i == 2


def test_width_choice_takes_the_first_of_equal_rates(orc32):
    acc = np.array([[1.0]])                         # expected lengths 1, 2
    i, _ = orc32.choose_width(acc, [1, 2], [1.0, 2.0])
    assert i == 0
