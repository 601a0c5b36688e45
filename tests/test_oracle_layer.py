"""Pins for the oracle's decoder layer, stack and LM head.

The layer is checked against a second implementation assembled only from torch
library routines in fp64 (rms_norm, linear, scaled_dot_product_attention with a
boolean mask, silu; the rotation done as a complex multiplication), against the
sequential-decode special case, and for structural invariants.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

from paper_2505_23219_amd import workloads as wl
from tests.test_oracle_tree import mask_by_recurrence

SHAPE = wl.ModelShape("mini", H=64, nh=4, d=16, F=88, V=50, L=2)


def np_weights(shape, seed, layer):
    return {k: v.numpy() for k, v in wl.layer_weights(shape, seed, layer).items()}


def np_cache(shape, cap, kv_len, seed, layer):
    k, v = wl.kv_cache(shape, cap, kv_len, seed, layer)
    return k.numpy().copy(), v.numpy().copy()


ROUNDING_POINTS = ("n_attn", "q", "o", "n_ffn", "a")
NOT_ROUNDED = ("wo_out", "gu", "down_out")     # places the oracle must not round at


def library_layer(shape, w, kc, vc, x, parent, kv_len, casts=()):
    """One layer from torch library routines in fp64.  `casts` names the intermediate
    results that are rounded to fp16 on the way (numpy's direct double -> half
    conversion): the normalised activations of the two blocks, the rotated queries, the
    attention output and the SwiGLU activation.  The rows appended to the cache are fp16
    in every variant, because the cache is."""
    H, nh, d, F = shape.H, shape.nh, shape.d, shape.F
    M = len(parent)
    t = lambda a: torch.from_numpy(np.asarray(a).astype(np.float64))
    assert set(casts) <= set(ROUNDING_POINTS + NOT_ROUNDED)

    def cast(name, v):
        return t(v.numpy().astype(np.float16)) if name in casts else v

    x = t(x)
    depth = [0] * M
    for i in range(1, M):
        depth[i] = depth[parent[i]] + 1
    pos = torch.tensor([kv_len + dd for dd in depth], dtype=torch.float64)

    def rot(v):                                   # [M, nh, d], half-split pairs as complex
        j = torch.arange(d // 2, dtype=torch.float64)
        ang = pos[:, None] * shape.rope_base ** (-2.0 * j / d)[None, :]
        z = torch.complex(v[..., :d // 2], v[..., d // 2:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    n = cast("n_attn", Fn.rms_norm(x, (H,), t(w["g_attn"]), shape.rms_eps))
    qkv = Fn.linear(n, t(w["Wqkv"]))
    q = cast("q", rot(qkv[:, :H].reshape(M, nh, d)))
    k = rot(qkv[:, H:2 * H].reshape(M, nh, d))
    v = qkv[:, 2 * H:].reshape(M, nh, d)
    # the cache holds fp16: the tree rows are attended as stored
    h16 = lambda a: a.to(torch.float16).to(torch.float64)
    K = torch.cat([t(kc[:, :kv_len]), h16(k).permute(1, 0, 2)], dim=1)
    V = torch.cat([t(vc[:, :kv_len]), h16(v).permute(1, 0, 2)], dim=1)
    vis = torch.cat([torch.ones(M, kv_len, dtype=torch.bool),
                     torch.from_numpy(mask_by_recurrence(parent).astype(bool))], dim=1)
    o = cast("o", Fn.scaled_dot_product_attention(q.permute(1, 0, 2), K, V, attn_mask=vis))
    x = x + cast("wo_out", Fn.linear(o.permute(1, 0, 2).reshape(M, H), t(w["Wo"])))
    n2 = cast("n_ffn", Fn.rms_norm(x, (H,), t(w["g_ffn"]), shape.rms_eps))
    gu = cast("gu", Fn.linear(n2, t(w["Wgu"])))
    a = cast("a", Fn.silu(gu[:, :F]) * gu[:, F:])
    x = x + cast("down_out", Fn.linear(a, t(w["Wdown"])))
    return x.numpy(), k.numpy(), v.numpy()


@pytest.mark.parametrize("M,depth,kv_len,seed", [(1, 1, 9, 0), (7, 3, 20, 1), (16, 4, 0, 2)])
def test_layer_matches_library_composition(orc32, orc64, M, depth, kv_len, seed):
    parent = wl.tree_random(M, depth, seed)
    w = np_weights(SHAPE, seed, 0)
    x = wl.activations(M, SHAPE.H, seed).numpy()
    kc, vc = np_cache(SHAPE, kv_len + M + 3, kv_len, seed, 0)
    ref, k_ref, v_ref = library_layer(SHAPE, w, kc, vc, x, parent, kv_len)
    kc64, vc64 = kc.copy(), vc.copy()
    got = orc64.verify_layer(SHAPE, w, kc64, vc64, x, parent, kv_len, round16=False)
    np.testing.assert_allclose(got, ref, atol=1e-10)
    # tree rows appended to the cache are the rotated keys and plain values, as fp16
    np.testing.assert_array_equal(kc64[:, kv_len:kv_len + M],
                                  k_ref.transpose(1, 0, 2).astype(np.float16))
    np.testing.assert_array_equal(vc64[:, kv_len:kv_len + M],
                                  v_ref.transpose(1, 0, 2).astype(np.float16))
    assert np.array_equal(kc64[:, :kv_len], kc[:, :kv_len])
    assert np.all(kc64[:, kv_len + M:] == 0)
    # the fp32 build differs from fp64 only by accumulation noise
    got32 = orc32.verify_layer(SHAPE, w, kc.copy(), vc.copy(), x, parent, kv_len, round16=False)
    np.testing.assert_allclose(got32, ref, atol=2e-5)
    # the fp16 rounding points move the result by fp16-sized amounts only
    got16 = orc32.verify_layer(SHAPE, w, kc.copy(), vc.copy(), x, parent, kv_len, round16=True)
    err = np.abs(got16 - ref).max()
    assert 0 < err < 5e-3


@pytest.mark.parametrize("M,depth,kv_len,seed", [(1, 1, 9, 0), (7, 3, 20, 1), (16, 4, 0, 2)])
def test_rounded_layer_rounds_at_exactly_the_documented_points(orc32, orc64, M, depth, kv_len, seed):
    """The variant with fp16 rounding points (the truth of every GPU layer and stack
    comparison) is the library composition with casts at exactly five places.  In the fp64
    build the casts are then the only difference, so the two agree to accumulation noise;
    with any one cast left out, or with none, they do not."""
    parent = wl.tree_random(M, depth, seed)
    w = np_weights(SHAPE, seed, 0)
    x = wl.activations(M, SHAPE.H, seed).numpy()
    kc, vc = np_cache(SHAPE, kv_len + M + 3, kv_len, seed, 0)
    ref, k_ref, v_ref = library_layer(SHAPE, w, kc, vc, x, parent, kv_len, ROUNDING_POINTS)
    kc64, vc64 = kc.copy(), vc.copy()
    got = orc64.verify_layer(SHAPE, w, kc64, vc64, x, parent, kv_len, round16=True)
    np.testing.assert_allclose(got, ref, atol=1e-9, rtol=0)
    np.testing.assert_array_equal(kc64[:, kv_len:kv_len + M], k_ref.transpose(1, 0, 2).astype(np.float16))
    np.testing.assert_array_equal(vc64[:, kv_len:kv_len + M], v_ref.transpose(1, 0, 2).astype(np.float16))
    # the fp32 build of the same variant: accumulation noise, now and then carried across
    # a rounding boundary of one element (an fp16 ulp of an O(1) value times a weight)
    got32 = orc32.verify_layer(SHAPE, w, kc.copy(), vc.copy(), x, parent, kv_len, round16=True)
    np.testing.assert_allclose(got32, ref, atol=3e-4, rtol=0)
    assert np.abs(got32 - ref).mean() < 5e-6
    # negatives: a missing rounding point is seen
    for missing in ROUNDING_POINTS:
        fewer = tuple(p for p in ROUNDING_POINTS if p != missing)
        other, _, _ = library_layer(SHAPE, w, kc, vc, x, parent, kv_len, fewer)
        assert np.abs(got - other).max() > 1e-6, missing
    none, _, _ = library_layer(SHAPE, w, kc, vc, x, parent, kv_len)
    assert np.abs(got - none).max() > 1e-5
    # ... and so is a sixth one
    for extra in NOT_ROUNDED:
        other, _, _ = library_layer(SHAPE, w, kc, vc, x, parent, kv_len, ROUNDING_POINTS + (extra,))
        assert np.abs(got - other).max() > 1e-7, extra   # (the match above holds to 1e-9)


def test_rounded_lm_head_rounds_the_normalised_input_only(orc64):
    M, seed = 5, 6
    head = {k: v.numpy() for k, v in wl.head_weights(SHAPE, seed).items()}
    x = (3.0 * wl.activations(M, SHAPE.H, seed).numpy().astype(np.float64))
    t = lambda a: torch.from_numpy(np.asarray(a).astype(np.float64))
    n = Fn.rms_norm(t(x), (SHAPE.H,), t(head["g_final"]), SHAPE.rms_eps)
    n16 = t(n.numpy().astype(np.float16))
    ref = Fn.linear(n16, t(head["Wlm"])).numpy()
    got = orc64.lm_head(SHAPE, head["g_final"], head["Wlm"], x, True)
    np.testing.assert_allclose(got, ref, atol=1e-10, rtol=0)
    plain = Fn.linear(n, t(head["Wlm"])).numpy()
    assert np.abs(got - plain).max() > 1e-6
    # logits are not rounded to fp16
    assert np.abs(got - got.astype(np.float16)).max() > 1e-7


def test_width1_tree_equals_sequential_decode(orc32):
    """A depth-k path verified in one pass == k plain decode steps that each
    append one row to the cache (bit-identical in the oracle)."""
    k, kv_len = 6, 13
    w = np_weights(SHAPE, 3, 0)
    x = wl.activations(k, SHAPE.H, 3).numpy()
    kc, vc = np_cache(SHAPE, kv_len + k, kv_len, 3, 0)
    for r16 in (False, True):
        kc_a, vc_a = kc.copy(), vc.copy()
        tree = orc32.verify_layer(SHAPE, w, kc_a, vc_a, x, wl.tree_chain(k), kv_len, r16)
        kc_b, vc_b = kc.copy(), vc.copy()
        for s in range(k):
            row = orc32.verify_layer(SHAPE, w, kc_b, vc_b, x[s:s + 1], [-1], kv_len + s, r16)
            assert np.array_equal(row[0], tree[s]), s
        assert np.array_equal(kc_a, kc_b) and np.array_equal(vc_a, vc_b)


def test_siblings_with_equal_inputs_get_equal_outputs(orc32):
    parent = np.array([-1, 0, 0, 1, 1, 2], dtype=np.int32)
    w = np_weights(SHAPE, 4, 0)
    x = wl.activations(6, SHAPE.H, 4).numpy().copy()
    x[2] = x[1]
    x[4] = x[3]
    kc, vc = np_cache(SHAPE, 32, 10, 4, 0)
    out = orc32.verify_layer(SHAPE, w, kc, vc, x, parent, 10, True)
    assert np.array_equal(out[1], out[2])
    assert np.array_equal(out[3], out[4])
    assert not np.array_equal(out[3], out[5])


def test_stack_is_layers_then_head(orc32):
    M, kv_len = 5, 12
    parent = wl.tree_random(M, 2, 5)
    layers = [np_weights(SHAPE, 5, l) for l in range(SHAPE.L)]
    head = {k: v.numpy() for k, v in wl.head_weights(SHAPE, 5).items()}
    x16 = wl.activations(M, SHAPE.H, 5).numpy()
    caches = [np_cache(SHAPE, kv_len + M, kv_len, 5, l) for l in range(SHAPE.L)]
    kcs = [c[0].copy() for c in caches]
    vcs = [c[1].copy() for c in caches]
    logits, x_out = orc32.verify_stack(SHAPE, layers, kcs, vcs, head, x16, parent, kv_len, True)
    x = x16.astype(np.float32)
    for l in range(SHAPE.L):
        kc, vc = caches[l][0].copy(), caches[l][1].copy()
        x = orc32.verify_layer(SHAPE, layers[l], kc, vc, x, parent, kv_len, True)
        assert np.array_equal(kc, kcs[l]) and np.array_equal(vc, vcs[l])
    assert np.array_equal(x, x_out)
    assert np.array_equal(orc32.lm_head(SHAPE, head["g_final"], head["Wlm"], x, True), logits)
    # the head is norm then linear (library routines, fp64)
    n = Fn.rms_norm(torch.from_numpy(x.astype(np.float64)), (SHAPE.H,),
                    torch.from_numpy(head["g_final"].astype(np.float64)), SHAPE.rms_eps)
    ref = Fn.linear(n, torch.from_numpy(head["Wlm"].astype(np.float64))).numpy()
    np.testing.assert_allclose(orc32.lm_head(SHAPE, head["g_final"], head["Wlm"], x, False), ref,
                               atol=1e-5)


def test_tiny_workload_runs_and_is_finite(orc32):
    w = wl.workload("tiny")
    s = w.shape
    layers = [np_weights(s, w.seed, 0)]
    head = {k: v.numpy() for k, v in wl.head_weights(s, w.seed).items()}
    kc, vc = np_cache(s, w.capacity, w.kv_len, w.seed, 0)
    x16 = wl.activations(w.M, s.H, w.seed).numpy()
    logits, _ = orc32.verify_stack(s, layers, [kc], [vc], head, x16, w.parent, w.kv_len, True)
    assert logits.shape == (8, 1000) and np.isfinite(logits).all()
    n, nxt, path, amax = orc32.accept_greedy(logits, wl.draft_tokens(w.M, s.V, w.seed), w.parent)
    assert n >= 1 and path[0] == 0 and nxt == amax[path[-1]]
