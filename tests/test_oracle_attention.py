"""Pins for the oracle's tree attention.

Independent checks: a textbook dense masked softmax written with fp64 matrix
products, torch's scaled_dot_product_attention with an explicit boolean mask,
the causal special case, path decomposition (verifying a tree means scoring
each root path as if it were the only continuation), non-interference, the
online-softmax merge identity of section 3.2.2, and closed forms.
"""
import numpy as np
import pytest
import torch

from paper_2505_23219_amd import workloads as wl
from tests.test_oracle_tree import mask_by_recurrence


def make_case(M, nh, d, kv_len, seed, cap=None):
    shape = wl.ModelShape("t", H=nh * d, nh=nh, d=d, F=8, V=8, L=1)
    cap = cap or kv_len + M
    kc, vc = wl.kv_cache(shape, cap, kv_len, seed, 0)
    kc, vc = kc.numpy().copy(), vc.numpy().copy()
    tk = wl.activations(M, nh * d, seed, tag="tk").numpy().reshape(M, nh, d)
    tv = wl.activations(M, nh * d, seed, tag="tv").numpy().reshape(M, nh, d)
    kc[:, kv_len:kv_len + M] = tk.transpose(1, 0, 2)
    vc[:, kv_len:kv_len + M] = tv.transpose(1, 0, 2)
    q = wl.activations(M, nh * d, seed, tag="q").numpy().astype(np.float64).reshape(M, nh, d)
    return q, kc, vc


def dense_masked_attention(q, kc, vc, vis, scale):
    """Textbook softmax(QK^T * scale + mask) V in fp64; vis [M, T] boolean."""
    M, nh, d = q.shape
    T = vis.shape[1]
    out = np.zeros_like(q)
    for h in range(nh):
        K = kc[h, :T].astype(np.float64)
        Vv = vc[h, :T].astype(np.float64)
        X = (q[:, h] @ K.T) * scale
        X = np.where(vis, X, -np.inf)
        A = np.exp(X - X.max(axis=1, keepdims=True))
        A /= A.sum(axis=1, keepdims=True)
        out[:, h] = A @ Vv
    return out


def visibility(parent, kv_len):
    M = len(parent)
    return np.concatenate([np.ones((M, kv_len), bool), mask_by_recurrence(parent).astype(bool)], 1)


@pytest.mark.parametrize("M,depth,kv_len,seed", [(1, 1, 5, 0), (8, 3, 37, 1), (16, 4, 0, 2),
                                                  (33, 5, 70, 3)])
def test_tree_attention_matches_dense_masked_softmax(orc32, orc64, M, depth, kv_len, seed):
    nh, d = 3, 16
    parent = wl.tree_random(M, depth, seed)
    q, kc, vc = make_case(M, nh, d, kv_len, seed)
    scale = 1.0 / np.sqrt(d)
    ref = dense_masked_attention(q, kc, vc, visibility(parent, kv_len), scale)
    np.testing.assert_allclose(orc64.tree_attention(q, kc, vc, parent, kv_len), ref, atol=1e-12)
    np.testing.assert_allclose(orc32.tree_attention(q, kc, vc, parent, kv_len), ref, atol=5e-6)


def test_tree_attention_matches_torch_sdpa(orc64):
    M, nh, d, kv_len = 12, 2, 32, 19
    parent = wl.tree_random(M, 4, 9)
    q, kc, vc = make_case(M, nh, d, kv_len, 9)
    vis = torch.from_numpy(visibility(parent, kv_len))
    T = kv_len + M
    tq = torch.from_numpy(q).permute(1, 0, 2)                      # [nh, M, d]
    tk = torch.from_numpy(kc[:, :T].astype(np.float64))
    tv = torch.from_numpy(vc[:, :T].astype(np.float64))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=vis)
    got = orc64.tree_attention(q, kc, vc, parent, kv_len)
    np.testing.assert_allclose(got, ref.permute(1, 0, 2).numpy(), atol=1e-12)


def test_chain_tree_is_causal_attention(orc64):
    M, nh, d, kv_len = 10, 2, 16, 23
    q, kc, vc = make_case(M, nh, d, kv_len, 4)
    T = kv_len + M
    tq = torch.zeros(nh, T, d, dtype=torch.float64)
    tq[:, kv_len:] = torch.from_numpy(q).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq, torch.from_numpy(kc[:, :T].astype(np.float64)),
        torch.from_numpy(vc[:, :T].astype(np.float64)), is_causal=True)[:, kv_len:]
    got = orc64.tree_attention(q, kc, vc, wl.tree_chain(M), kv_len)
    np.testing.assert_allclose(got, ref.permute(1, 0, 2).numpy(), atol=1e-12)


def test_path_decomposition(orc32):
    """Each root path, attended alone as a chain, reproduces its nodes' rows."""
    M, nh, d, kv_len = 14, 2, 16, 9
    parent = wl.tree_random(M, 4, 5)
    q, kc, vc = make_case(M, nh, d, kv_len, 5)
    full = orc32.tree_attention(q, kc, vc, parent, kv_len)
    for leaf in range(M):
        path = []
        j = leaf
        while j >= 0:
            path.append(j)
            j = int(parent[j])
        path = path[::-1]
        n = len(path)
        kc2 = np.zeros((nh, kv_len + n, d), np.float16)
        vc2 = np.zeros_like(kc2)
        kc2[:, :kv_len], vc2[:, :kv_len] = kc[:, :kv_len], vc[:, :kv_len]
        for r, node in enumerate(path):
            kc2[:, kv_len + r], vc2[:, kv_len + r] = kc[:, kv_len + node], vc[:, kv_len + node]
        sub = orc32.tree_attention(q[path], kc2, vc2, wl.tree_chain(n), kv_len)
        # same keys in the same ascending order: bit-identical
        assert np.array_equal(sub, full[path])


def test_non_interference(orc32):
    M, nh, d, kv_len = 12, 2, 16, 7
    parent = wl.tree_random(M, 3, 6)
    q, kc, vc = make_case(M, nh, d, kv_len, 6)
    base = orc32.tree_attention(q, kc, vc, parent, kv_len)
    mask = mask_by_recurrence(parent)
    for j in range(1, M):
        kc2, vc2, q2 = kc.copy(), vc.copy(), q.copy()
        kc2[:, kv_len + j] += np.float16(3.0)
        vc2[:, kv_len + j] -= np.float16(2.0)
        q2[j] += 1.0
        out = orc32.tree_attention(q2, kc2, vc2, parent, kv_len)
        for i in range(M):
            if i != j and not mask[i, j]:
                assert np.array_equal(out[i], base[i]), (i, j)
            elif mask[i, j]:
                assert not np.array_equal(out[i], base[i]), (i, j)


def test_online_softmax_merge_identity(orc64):
    """Section 3.2.2: parts run their own softmax and are aligned by a scaling
    factor at the end.  Attention over the whole visible set equals the rescaled
    merge of attention over the committed rows and over the tree rows."""
    M, nh, d, kv_len = 9, 2, 16, 21
    parent = wl.tree_random(M, 3, 8)
    q, kc, vc = make_case(M, nh, d, kv_len, 8)
    scale = 1.0 / np.sqrt(d)
    full = orc64.tree_attention(q, kc, vc, parent, kv_len)
    # part 1: committed rows only == star-free single-node trees over the cache
    star_cache_k = np.zeros((nh, kv_len, d), np.float16)
    o1 = np.zeros_like(q)
    o2 = np.zeros_like(q)
    m1 = np.zeros((M, nh)); l1 = np.zeros((M, nh)); m2 = np.zeros((M, nh)); l2 = np.zeros((M, nh))
    vis = mask_by_recurrence(parent).astype(bool)
    for i in range(M):
        # dense part: node i alone against the first kv_len-1 rows plus row kv_len-1 as "self"
        kd = kc[:, :kv_len].copy(); vd = vc[:, :kv_len].copy()
        o1[i] = orc64.tree_attention(q[i:i + 1], kd, vd, [-1], kv_len - 1)[0]
        # sparse part: node i against its root path only (no committed rows)
        path = [j for j in range(M) if vis[i, j]]
        ks = np.ascontiguousarray(kc[:, [kv_len + j for j in path]])
        vs = np.ascontiguousarray(vc[:, [kv_len + j for j in path]])
        o2[i] = orc64.tree_attention(q[i:i + 1], ks, vs, [-1], len(path) - 1)[0]
        for h in range(nh):
            s1 = (kc[h, :kv_len].astype(np.float64) @ q[i, h]) * scale
            s2 = (ks[h].astype(np.float64) @ q[i, h]) * scale
            m1[i, h], m2[i, h] = s1.max(), s2.max()
            l1[i, h], l2[i, h] = np.exp(s1 - m1[i, h]).sum(), np.exp(s2 - m2[i, h]).sum()
    m = np.maximum(m1, m2)
    a1, a2 = np.exp(m1 - m) * l1, np.exp(m2 - m) * l2
    merged = (a1[..., None] * o1 + a2[..., None] * o2) / (a1 + a2)[..., None]
    np.testing.assert_allclose(merged, full, atol=1e-12)


def test_closed_forms(orc64):
    M, nh, d, kv_len = 6, 2, 16, 11
    parent = wl.tree_random(M, 2, 10)
    q, kc, vc = make_case(M, nh, d, kv_len, 10)
    vis = visibility(parent, kv_len)
    # q = 0: uniform weights, output = mean of the visible V rows
    out = orc64.tree_attention(np.zeros_like(q), kc, vc, parent, kv_len)
    for i in range(M):
        for h in range(nh):
            want = vc[h, :kv_len + M][vis[i]].astype(np.float64).mean(axis=0)
            np.testing.assert_allclose(out[i, h], want, atol=1e-13)
    # one key far ahead of the rest: output is that key's V row
    kc2 = np.zeros_like(kc)
    kc2[:, 4, 0] = 60.0
    q2 = np.zeros_like(q)
    q2[:, :, 0] = 4.0                        # score 4*60/sqrt(16) = 60 for row 4, 0 elsewhere
    out = orc64.tree_attention(q2, kc2, vc, parent, kv_len)
    for i in range(M):
        np.testing.assert_allclose(out[i], vc[:, 4].astype(np.float64), atol=1e-12)
    # kv_len = 0: the root sees only itself
    q, kc, vc = make_case(M, nh, d, 0, 12)
    out = orc64.tree_attention(q, kc, vc, parent, 0)
    np.testing.assert_allclose(out[0], vc[:, 0].astype(np.float64), atol=1e-15)


def test_strided_cache_capacity_is_respected(orc64):
    # rows beyond kv_len + M hold garbage and must never be read into the result
    M, nh, d, kv_len = 5, 2, 16, 6
    parent = wl.tree_random(M, 2, 13)
    q, kc, vc = make_case(M, nh, d, kv_len, 13, cap=kv_len + M + 9)
    a = orc64.tree_attention(q, kc, vc, parent, kv_len)
    kc[:, kv_len + M:] = np.float16(100.0)
    vc[:, kv_len + M:] = np.float16(-100.0)
    b = orc64.tree_attention(q, kc, vc, parent, kv_len)
    assert np.array_equal(a, b)


# ---- attention under a given mask (the other verification patterns of section 2.3) -------------
def random_mask(M, seed, density=0.4):
    rng = np.random.default_rng(seed)
    m = rng.random((M, M)) < density
    m[np.arange(M), np.arange(M)] = True
    return m.astype(np.uint8)


def draft_model_mask(n_seq, length):
    """Several drafted sequences verified side by side: a token sees the earlier tokens of
    its own sequence and itself."""
    M = n_seq * length
    m = np.zeros((M, M), np.uint8)
    for s in range(n_seq):
        for a in range(length):
            m[s * length + a, s * length:s * length + a + 1] = 1
    return m


def test_masked_attention_with_the_tree_mask_is_tree_attention(orc32):
    M, nh, d, kv_len = 21, 2, 16, 30
    parent = wl.tree_random(M, 4, 6)
    q, kc, vc = make_case(M, nh, d, kv_len, 6)
    got = orc32.masked_attention(q, kc, vc, orc32.tree_mask(parent), kv_len)
    assert np.array_equal(got, orc32.tree_attention(q, kc, vc, parent, kv_len))


@pytest.mark.parametrize("kind,kv_len", [("random", 17), ("random", 0), ("sequences", 40), ("full", 5)])
def test_masked_attention_matches_torch_sdpa(orc64, kind, kv_len):
    M, nh, d = 12, 2, 32
    mask = {"random": random_mask(M, 3), "sequences": draft_model_mask(3, 4),
            "full": np.ones((M, M), np.uint8)}[kind]
    q, kc, vc = make_case(M, nh, d, kv_len, 11)
    T = kv_len + M
    vis = torch.from_numpy(np.concatenate([np.ones((M, kv_len), bool), mask.astype(bool)], 1))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).permute(1, 0, 2), torch.from_numpy(kc[:, :T].astype(np.float64)),
        torch.from_numpy(vc[:, :T].astype(np.float64)), attn_mask=vis)
    got = orc64.masked_attention(q, kc, vc, mask, kv_len)
    np.testing.assert_allclose(got, ref.permute(1, 0, 2).numpy(), atol=1e-12)
    np.testing.assert_allclose(got, dense_masked_attention(q, kc, vc, vis.numpy(), 1 / np.sqrt(d)), atol=1e-12)


def test_masked_attention_row_without_keys_gives_zeros(orc32):
    M, nh, d = 5, 2, 16
    mask = random_mask(M, 1)
    mask[3] = 0
    q, kc, vc = make_case(M, nh, d, 0, 2)
    got = orc32.masked_attention(q, kc, vc, mask, 0)
    assert np.all(got[3] == 0) and np.all(np.isfinite(got))
    # one visible key: the output is that key's value row
    mask[2] = 0
    mask[2, 4] = 1
    got = orc32.masked_attention(q, kc, vc, mask, 0)
    assert np.allclose(got[2], vc[:, 4].astype(np.float32), atol=1e-6)
