"""GPU-vs-oracle parity through the C ABI, on the same seeded inputs.

Integer results (packed bytes, masks, argmax, accepted paths) must be
bit-identical.  Floating-point tolerances:
  * fp32 outputs of a single linear layer: both sides add exact fp16 x fp16
    products in fp32 in different orders, so the gap is accumulation noise;
    bound used: 2e-4 + 2e-4*|ref| (K <= 11008, |terms| ~ 0.02).
  * fp16 activations / residual stream / logits after whole layers:
    |gpu - ref| <= 2e-2 + 1e-2*|ref| against the fp32 oracle with the fp16
    rounding points switched on.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2505_23219_amd import workloads as wl

pytestmark = pytest.mark.gpu


_capman = None


@pytest.fixture(autouse=True, scope="module")
def _capture_manager(request):
    global _capman
    _capman = request.config.pluginmanager.getplugin("capturemanager")


def say(*a):
    """Progress line that reaches the terminal even under output capture: names the case
    before each GPU step."""
    if _capman is not None:
        with _capman.global_and_fixture_disabled():
            print(*a, flush=True)
    else:
        print(*a, flush=True)


@pytest.fixture(scope="module")
def B():
    from paper_2505_23219_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.lib()          # fails loudly when libghd.so is missing
    return binding


@pytest.fixture(scope="module")
def model():
    from paper_2505_23219_amd import model
    return model


def close(got, ref, atol, rtol):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    worst = float((err - bound).max())
    return worst <= 0, float(err.max()), float((err / np.maximum(np.abs(ref), 1e-3)).max())


def reference_pack(W, kind=0, d=0):
    """The packed layout written out from its definition (include/ghd.h)."""
    N, K = W.shape
    ntiles = (N + 15) // 16
    rb = 8 if ntiles >= 640 else 4              # tiles per storage block
    nitems = (ntiles + rb - 1) // rb
    Np, Kp = nitems * rb * 16, (K + 31) // 32 * 32
    src = np.full(Np, -1, dtype=np.int64)
    for p in range(N):
        if kind == 0:
            src[p] = p
        elif kind == 1:
            H = N // 3
            nh = H // d
            if nh % 8 == 0:                     # heads grouped by XCD: q, k, v rows of nh/8 heads each
                hpx = nh // 8
                x, q = divmod(p, 3 * hpx * d)
                part, hn = divmod(q, hpx * d)
                head, ph = x * hpx + hn // d, hn % d
            else:
                part, hn = divmod(p, H)
                head, ph = divmod(hn, d)
            i, r = divmod(ph, 4)
            src[p] = part * H + head * d + 2 * i + (r & 1) + (d // 2 if r >= 2 else 0)
        else:
            F = N // 2
            t, q = divmod(p, 16)
            i, r = divmod(q, 4)
            f = 8 * t + 2 * i + (r & 1)
            src[p] = (F if r >= 2 else 0) + f
    Wp = np.zeros((Np, Kp), dtype=np.uint16)
    rows = src >= 0
    Wp[rows, :K] = W.view(np.uint16)[src[rows]]
    # [block, tile, row, kstep, kgroup, 8] -> [block, kstep, tile, kgroup, row, 8]
    out = Wp.reshape(nitems, rb, 16, Kp // 32, 4, 8).transpose(0, 3, 1, 4, 2, 5)
    return np.ascontiguousarray(out).reshape(-1)


@pytest.mark.parametrize("N,K,kind,d", [(16, 32, 0, 0), (40, 72, 0, 0), (1000, 256, 0, 0),
                                        (256, 688, 0, 0), (768, 256, 1, 64), (3 * 512, 136, 1, 128),
                                        (2 * 688, 256, 2, 0), (2 * 1376, 128, 2, 0),
                                        (10240, 64, 0, 0), (10300, 40, 0, 0), (3 * 3584, 32, 1, 128),
                                        (3 * 1024, 64, 1, 128), (3 * 512, 40, 1, 64), (3 * 4096, 32, 1, 128),
                                        (2 * 5504, 64, 2, 0)])
def test_pack_weight_bytes(B, N, K, kind, d):
    say("pack", N, K, kind, d)
    W = wl.activations(N, K, 21, tag="w", std=0.02)
    got = B.ghd_pack_weight(W.cuda(), kind, d).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, reference_pack(W.numpy(), kind, d))


def test_tree_mask_bit_exact(B, orc32):
    cases = [p for M in range(1, 6) for p in wl.all_trees(M)]
    cases += [wl.tree_random(M, dep, s) for M, dep, s in ((8, 3, 0), (64, 5, 2), (65, 9, 5),
                                                          (128, 5, 3), (128, 127, 4))]
    cases += [wl.tree_chain(128), wl.tree_star(128), wl.tree_wide_shallow(64, 32, 4)]
    for parent in cases:
        M = len(parent)
        got = B.ghd_tree_mask(torch.from_numpy(parent).cuda()).cpu().numpy().view(np.uint64)
        ref = orc32.tree_mask(parent)
        bits = np.zeros((M, 2), dtype=np.uint64)
        for i in range(M):
            for j in range(M):
                if ref[i, j]:
                    bits[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
        assert np.array_equal(got, bits), list(parent)


LINEAR_CASES = [(1, 64, 64), (3, 130, 688), (8, 1000, 256), (16, 256, 256), (17, 48, 96),
                (33, 688 * 2, 256), (64, 256, 688), (100, 130, 520), (128, 512, 1024),
                (16, 12288, 4096), (64, 4096, 11008), (1, 4096, 4096),
                # narrow matrices at few rows: whole tiles where they spread evenly over the workgroups
                # (256 tiles), k ranges of row blocks where they do not (320 tiles); a wide one with
                # shares of unequal tile counts and a ragged last tile
                (16, 4096, 11008), (1, 5120, 5120), (8, 5120, 13824), (4, 22016, 4096), (64, 11000, 1000)]


@pytest.mark.parametrize("M,N,K", LINEAR_CASES)
def test_linear_skinny(B, orc32, M, N, K):
    say("linear", M, N, K)
    x = wl.activations(M, K, 31)
    W = wl.activations(N, K, 32, tag="w", std=0.02)
    Wp = B.ghd_pack_weight(W.cuda())
    ref = orc32.linear(x.numpy().astype(np.float32), W.numpy())
    ws = B.workspace(B.lib().ghd_linear_workspace_bytes(M, N, K))
    y = B.ghd_linear_skinny(x.cuda(), Wp, N, ws=ws)
    assert B.ghd_step_status(ws) == 0
    y = y.cpu().numpy()
    ok, ma, mr = close(y, ref, 2e-4, 2e-4)
    assert ok, (ma, mr)
    # fp16 output = the fp32 result rounded once
    y16 = B.ghd_linear_skinny(x.cuda(), Wp, N, out_dtype=torch.float16).cpu().numpy()
    ok, ma, mr = close(y16, ref, 1e-3, 1e-3)
    assert ok, (ma, mr)


@pytest.mark.parametrize("M,N,K,padx,pady", [(5, 130, 688, 24, 6), (64, 4096, 1024, 8, 64), (33, 10300, 264, 40, 4)])
def test_linear_skinny_with_padded_leading_dimensions(B, orc32, M, N, K, padx, pady):
    """x and y given as views of wider arrays (ldx > K, ldy > N): the columns beside them
    are neither read into the result nor written."""
    say("linear padded", M, N, K, padx, pady)
    x = wl.activations(M, K, 33)
    W = wl.activations(N, K, 34, tag="w", std=0.02)
    ref = orc32.linear(x.numpy().astype(np.float32), W.numpy())
    bigx = torch.full((M, K + padx), float("nan"), dtype=torch.float16)
    bigx[:, :K] = x
    bigx = bigx.cuda()
    for dt, tol in ((torch.float32, 2e-4), (torch.float16, 1e-3)):
        bigy = torch.full((M, N + pady), -77.0, dtype=dt, device="cuda")
        ws = B.workspace(B.lib().ghd_linear_workspace_bytes(M, N, K))
        B.ghd_linear_skinny(bigx[:, :K], B.ghd_pack_weight(W.cuda()), N, ws=ws, y=bigy[:, :N])
        assert B.ghd_step_status(ws) == 0
        got = bigy.cpu().float().numpy()
        ok, ma, mr = close(got[:, :N], ref, tol, tol)
        assert ok, (ma, mr)
        assert (got[:, N:] == -77.0).all()


def test_step_status_is_sticky_until_reset(B, orc32):
    """A status an earlier call left (planted here from the host, no kernel is made to give
    up) survives the set-up of later calls and is reported until the caller resets it; a
    workspace used for the first time reports nothing, whatever its bytes were."""
    say("sticky status")
    M, N, K = 8, 130, 256
    x = wl.activations(M, K, 35).cuda()
    Wp = B.ghd_pack_weight(wl.activations(N, K, 36, tag="w", std=0.02).cuda())
    ws = torch.full((B.lib().ghd_linear_workspace_bytes(M, N, K),), 0xAB, dtype=torch.uint8, device="cuda")
    B.ghd_linear_skinny(x, Wp, N, ws=ws)
    assert B.ghd_step_status(ws) == 0                     # first use: the garbage is not a status
    words = ws[:16].view(torch.int32)
    words[1] = 1004                                       # as if a wait of the last call had given up
    torch.cuda.synchronize()
    assert B.ghd_step_status(ws) == 1004
    y1 = B.ghd_linear_skinny(x, Wp, N, ws=ws)             # a later, clean call
    assert B.ghd_step_status(ws) == 1004                  # still reported
    B._check(B.lib().ghd_step_status_reset(B._ptr(ws), B._stream()), "ghd_step_status_reset")
    assert B.ghd_step_status(ws) == 0
    y2 = B.ghd_linear_skinny(x, Wp, N, ws=ws)
    assert B.ghd_step_status(ws) == 0 and torch.equal(y1, y2)


def attention_case(M, nh, d, kv_len, parent, seed, cap=None):
    shape = wl.ModelShape("t", H=nh * d, nh=nh, d=d, F=8, V=8, L=1)
    cap = cap or ((kv_len + M + 63) // 64) * 64
    kc, vc = wl.kv_cache(shape, cap, kv_len, seed, 0)
    tk = wl.activations(M, nh * d, seed, tag="tk").reshape(M, nh, d)
    tv = wl.activations(M, nh * d, seed, tag="tv").reshape(M, nh, d)
    kc[:, kv_len:kv_len + M] = tk.permute(1, 0, 2)
    vc[:, kv_len:kv_len + M] = tv.permute(1, 0, 2)
    q = wl.activations(M, nh * d, seed, tag="q").reshape(M, nh, d).contiguous()
    return q, kc.contiguous(), vc.contiguous()


ATTN_CASES = [
    # M, nh, d, kv_len, tree
    (1, 4, 64, 128, "chain"), (8, 4, 64, 128, "rand3"), (8, 4, 64, 0, "rand3"),
    (16, 2, 128, 1024, "medusa"), (16, 3, 128, 100, "chain"), (16, 3, 128, 63, "star"),
    (17, 2, 128, 65, "rand5"), (64, 32, 128, 2048, "rand5"), (64, 4, 128, 2048, "chain"),
    (64, 5, 128, 8192, "wide"), (100, 2, 64, 300, "rand5"), (128, 2, 128, 257, "rand5"),
    (128, 2, 128, 1000, "chain"), (128, 2, 64, 0, "star"), (1, 2, 128, 0, "chain"),
]


def make_tree(kind, M):
    if kind == "chain":
        return wl.tree_chain(M)
    if kind == "star":
        return wl.tree_star(M)
    if kind == "medusa":
        return wl.tree_medusa(M, (4, 2, 1, 1), 1)
    if kind == "wide":
        return wl.tree_wide_shallow(M, 32, 4)
    return wl.tree_random(M, int(kind[4:]), 7)


@pytest.mark.parametrize("M,nh,d,kv_len,tree", ATTN_CASES)
def test_tree_attention(B, model, orc32, M, nh, d, kv_len, tree):
    say("attention", M, nh, d, kv_len, tree)
    parent = make_tree(tree, M)
    q, kc, vc = attention_case(M, nh, d, kv_len, parent, 41)
    ref = orc32.tree_attention(q.numpy().astype(np.float32), kc.numpy(), vc.numpy(), parent, kv_len)
    ws = B.workspace(B.lib().ghd_attention_workspace_bytes(M, kv_len, nh, d))
    got = B.ghd_tree_attention(q.cuda(), *model.upload_cache(kc, vc), torch.from_numpy(parent).cuda(),
                               kv_len, ws=ws)
    assert B.ghd_step_status(ws) == 0
    got = got.cpu().numpy()
    ok, ma, mr = close(got, ref, 5e-3, 5e-3)
    assert ok, (ma, mr)


@pytest.mark.parametrize("M,nh,d,kv_len,tree", [(8, 4, 64, 128, "rand3"), (40, 3, 128, 333, "rand5"),
                                                (64, 8, 128, 1000, "chain")])
def test_tree_attention_token_major_keys(B, model, orc32, M, nh, d, kv_len, tree):
    """K cache kept [capacity][nh][d] (k_stride_tok = nh * d, k_stride_head = d), the layout
    the strides of the call exist for."""
    say("attention, token-major K", M, nh, d, kv_len, tree)
    parent = make_tree(tree, M)
    q, kc, vc = attention_case(M, nh, d, kv_len, parent, 45)
    ref = orc32.tree_attention(q.numpy().astype(np.float32), kc.numpy(), vc.numpy(), parent, kv_len)
    kd, vd = model.upload_cache(kc, vc)
    k_tok = kd.permute(1, 0, 2).contiguous()          # [cap, nh, d] in memory
    view = k_tok.permute(1, 0, 2)                     # indexed [nh, cap, d] with strides (d, nh * d, 1)
    assert view.stride() == (d, nh * d, 1)
    ws = B.workspace(B.lib().ghd_attention_workspace_bytes(M, kv_len, nh, d))
    got = B.ghd_tree_attention(q.cuda(), view, vd, torch.from_numpy(parent).cuda(), kv_len, ws=ws)
    assert B.ghd_step_status(ws) == 0
    ok, ma, mr = close(got.cpu().numpy(), ref, 5e-3, 5e-3)
    assert ok, (ma, mr)


def test_tree_attention_with_256_heads(B, model, orc32):
    """More heads than workgroups per XCD: every workgroup takes whole heads."""
    M, nh, d, kv_len = 8, 256, 64, 130
    say("attention, 256 heads")
    parent = make_tree("rand3", M)
    q, kc, vc = attention_case(M, nh, d, kv_len, parent, 46)
    ref = orc32.tree_attention(q.numpy().astype(np.float32), kc.numpy(), vc.numpy(), parent, kv_len)
    ws = B.workspace(B.lib().ghd_attention_workspace_bytes(M, kv_len, nh, d))
    got = B.ghd_tree_attention(q.cuda(), *model.upload_cache(kc, vc), torch.from_numpy(parent).cuda(),
                               kv_len, ws=ws)
    assert B.ghd_step_status(ws) == 0
    ok, ma, mr = close(got.cpu().numpy(), ref, 5e-3, 5e-3)
    assert ok, (ma, mr)


@pytest.mark.parametrize("M,nh,d,kv_len,tree", [(8, 4, 64, 128, "rand3"), (64, 4, 128, 200, "rand5"),
                                                (64, 2, 128, 0, "chain"), (128, 2, 64, 77, "chain"),
                                                (128, 3, 128, 333, "rand5"), (64, 2, 128, 2048, "wide"),
                                                (1, 2, 128, 9, "chain"), (100, 2, 64, 40, "star")])
def test_tree_part_attention_from_the_mask_nonzeros(B, model, orc32, M, nh, d, kv_len, tree):
    """The sparse component alone (one dot product per (token, ancestor) pair): equals the
    oracle's tree attention on a cache that holds the tree rows only, and the attention
    kernel's masked tile on that cache."""
    say("tree part coo", M, nh, d, kv_len, tree)
    parent = make_tree(tree, M)
    q, kc, vc = attention_case(M, nh, d, kv_len, parent, 43)
    rows_k = kc[:, kv_len:kv_len + M].contiguous()
    rows_v = vc[:, kv_len:kv_len + M].contiguous()
    ref = orc32.tree_attention(q.numpy().astype(np.float32), rows_k.numpy(), rows_v.numpy(), parent, 0)
    kd, vd = model.upload_cache(kc, vc)
    pd = torch.from_numpy(parent).cuda()
    got = B.ghd_tree_part_attention_coo(q.cuda(), kd, vd, pd, kv_len).cpu().numpy()
    ok, ma, mr = close(got, ref, 5e-3, 5e-3)
    assert ok, (ma, mr)
    cap = ((M + 63) // 64) * 64
    pk = torch.zeros((nh, cap, d), dtype=torch.float16)
    pv = torch.zeros((nh, cap, d), dtype=torch.float16)
    pk[:, :M], pv[:, :M] = rows_k, rows_v
    dense = B.ghd_tree_attention(q.cuda(), *model.upload_cache(pk, pv), pd, 0).cpu().numpy()
    ok, ma, mr = close(got, dense, 5e-3, 5e-3)
    assert ok, (ma, mr)


@pytest.mark.parametrize("M,kv_len,cap", [(6, 64, 72), (1, 7, 8), (10, 118, 128), (9, 190, 200)])
def test_tree_attention_tight_capacity(B, model, orc32, M, kv_len, cap):
    """Capacity not a multiple of the 64-key tile: the last tile's V pieces past the
    capacity are never read (every piece there is replaced by the last valid one and
    zeroed), and rows between the tree and the capacity hold NaN."""
    say("attention tight", M, kv_len, cap)
    nh, d = 2, 128
    parent = wl.tree_random(M, 3, 5)
    q, kc, vc = attention_case(M, nh, d, kv_len, parent, 47, cap=cap)
    ref = orc32.tree_attention(q.numpy().astype(np.float32), kc.numpy(), vc.numpy(), parent, kv_len)
    kc[:, kv_len + M:] = float("nan")
    vc[:, kv_len + M:] = float("nan")
    ws = B.workspace(B.lib().ghd_attention_workspace_bytes(M, kv_len, nh, d))
    got = B.ghd_tree_attention(q.cuda(), *model.upload_cache(kc, vc), torch.from_numpy(parent).cuda(),
                               kv_len, ws=ws)
    assert B.ghd_step_status(ws) == 0
    ok, ma, mr = close(got.cpu().numpy(), ref, 5e-3, 5e-3)
    assert ok, (ma, mr)


def test_tree_attention_ignores_rows_past_the_tree(B, model):
    M, nh, d, kv_len = 9, 2, 128, 70
    parent = wl.tree_random(M, 3, 1)
    q, kc, vc = attention_case(M, nh, d, kv_len, parent, 43, cap=256)
    a = B.ghd_tree_attention(q.cuda(), *model.upload_cache(kc, vc), torch.from_numpy(parent).cuda(), kv_len)
    kc[:, kv_len + M:] = 100.0
    vc[:, kv_len + M:] = -100.0
    b = B.ghd_tree_attention(q.cuda(), *model.upload_cache(kc, vc), torch.from_numpy(parent).cuda(), kv_len)
    assert torch.equal(a, b)
    # not even a NaN there may leak (a zero weight times NaN would be NaN)
    kc[:, kv_len + M:] = float("nan")
    vc[:, kv_len + M:] = float("nan")
    c = B.ghd_tree_attention(q.cuda(), *model.upload_cache(kc, vc), torch.from_numpy(parent).cuda(), kv_len)
    assert torch.equal(a, c)


def run_layer_case(B, model, orc32, shape, M, kv_len, parent, seed):
    cap = ((kv_len + M + 63) // 64) * 64
    w = wl.layer_weights(shape, seed, 0)
    kc, vc = wl.kv_cache(shape, cap, kv_len, seed, 0)
    x16 = wl.activations(M, shape.H, seed)
    # oracle
    kc_o, vc_o = kc.numpy().copy(), vc.numpy().copy()
    ref = orc32.verify_layer(shape, {k: v.numpy() for k, v in w.items()}, kc_o, vc_o,
                             x16.numpy().astype(np.float32), parent, kv_len, round16=True)
    # GPU
    wd = model.upload_layer(w, shape.d)
    kc_d, vc_d = model.upload_cache(kc, vc)
    x = x16.float().cuda()
    cfg = B.make_cfg(shape, cap)
    ws = B.workspace(B.ghd_workspace_bytes(cfg, M, kv_len))
    B.ghd_verify_layer(cfg, wd, kc_d, vc_d, x, torch.from_numpy(parent).cuda(), kv_len, ws=ws)
    assert B.ghd_step_status(ws) == 0
    ok, ma, mr = close(x.cpu().numpy(), ref, 2e-2, 1e-2)
    assert ok, ("residual stream", ma, mr)
    for name, got, want in (("k", kc_d, kc_o), ("v", model.rows_of_v(vc_d), vc_o)):
        got = got.cpu().numpy()
        # committed rows untouched, rows past the tree untouched
        assert np.array_equal(got[:, :kv_len], want[:, :kv_len]), name
        assert np.array_equal(got[:, kv_len + M:], want[:, kv_len + M:]), name
        ok, ma, mr = close(got[:, kv_len:kv_len + M], want[:, kv_len:kv_len + M], 2e-3, 2e-3)
        assert ok, (name, ma, mr)
    return ma


@pytest.mark.parametrize("x_std,gain", [(1e-2, 0.03), (1e3, 1.0), (30.0, 4.0)])
def test_verify_layer_small_and_large_magnitudes(B, model, orc32, x_std, gain):
    """The normalised linear layers stream fp16(x * gain) and apply the row factor after the
    contraction: a small residual stream with small gains (first-layer embeddings) and a
    large one must come out as precisely as the usual N(0, 1) one.  The tolerance of the
    other layer tests, taken relative to the size of the layer's own update."""
    shape = wl.ModelShape("mag", H=512, nh=4, d=128, F=1376, V=100, L=1)
    M, kv_len, seed = 40, 64, 12
    say("layer magnitudes", x_std, gain)
    parent = make_tree("rand5", M)
    cap = ((kv_len + M + 63) // 64) * 64
    w = wl.layer_weights(shape, seed, 0)
    for g in ("g_attn", "g_ffn"):
        w[g] = (w[g].float() * gain).to(torch.float16)
    kc, vc = wl.kv_cache(shape, cap, kv_len, seed, 0)
    x32 = (wl.activations(M, shape.H, seed).float() * x_std).contiguous()
    kc_o, vc_o = kc.numpy().copy(), vc.numpy().copy()
    ref = orc32.verify_layer(shape, {k: v.numpy() for k, v in w.items()}, kc_o, vc_o, x32.numpy().copy(),
                             parent, kv_len, round16=True)
    wd = model.upload_layer(w, shape.d)
    kc_d, vc_d = model.upload_cache(kc, vc)
    x = x32.cuda()
    cfg = B.make_cfg(shape, cap)
    ws = B.workspace(B.ghd_workspace_bytes(cfg, M, kv_len))
    B.ghd_verify_layer(cfg, wd, kc_d, vc_d, x, torch.from_numpy(parent).cuda(), kv_len, ws=ws)
    assert B.ghd_step_status(ws) == 0
    update = ref - x32.numpy()
    unit = float(np.sqrt((update.astype(np.float64) ** 2).mean()))
    err = np.abs(x.cpu().numpy() - ref)
    # fp32 spacing of the residual stream itself is part of what can be had at x ~ 1e3
    bound = 2e-2 * unit + 1e-2 * np.abs(update) + 4 * np.spacing(np.abs(ref).astype(np.float32))
    assert (err <= bound).all(), (float(err.max()), unit)
    ok, ma, mr = close(kc_d.cpu().numpy()[:, kv_len:kv_len + M], kc_o[:, kv_len:kv_len + M], 2e-3 * max(gain, 1e-3), 2e-3)
    assert ok, ("k", ma, mr)


def test_verify_layer_tiny(B, model, orc32):
    w = wl.workload("tiny")
    say("layer tiny")
    run_layer_case(B, model, orc32, w.shape, w.M, w.kv_len, w.parent, w.seed)


@pytest.mark.parametrize("M,kv_len,tree", [(1, 77, "chain"), (5, 0, "rand3"), (16, 130, "star"),
                                           (40, 64, "rand5"), (128, 200, "rand5")])
def test_verify_layer_small_shapes(B, model, orc32, M, kv_len, tree):
    say("layer small", M, kv_len, tree)
    shape = wl.ModelShape("small", H=512, nh=4, d=128, F=1376, V=100, L=1)
    run_layer_case(B, model, orc32, shape, M, kv_len, make_tree(tree, M), 5)


@pytest.mark.parametrize("M,kv_len,tree", [(1, 130, "chain"), (16, 77, "rand3"), (64, 200, "rand5"), (128, 64, "rand5")])
def test_verify_layer_with_eight_heads(B, model, orc32, M, kv_len, tree):
    """A head count that is a multiple of 8: the packed QKV rows are grouped by XCD (and, for
    a wide enough QKV matrix, the attention runs in the QKV launch)."""
    say("layer 8 heads", M, kv_len, tree)
    shape = wl.ModelShape("h8", H=1024, nh=8, d=128, F=1376, V=100, L=1)
    run_layer_case(B, model, orc32, shape, M, kv_len, make_tree(tree, M), 6)


def test_fused_and_split_qkv_attention_agree(B, model, orc32):
    """One 7B-shaped layer with the QKV layer and the attention in one launch and as two
    launches: identical results bit for bit (same kernels' code, same summation orders)."""
    w = wl.workload("layer7b")
    shape, M, kv_len = w.shape, 64, 300
    say("layer 7b fused vs split")
    parent = make_tree("rand5", M)
    cap = ((kv_len + M + 63) // 64) * 64
    wd = model.upload_layer(wl.layer_weights(shape, 3, 0, device="cuda"), shape.d)
    kc, vc = wl.kv_cache(shape, cap, kv_len, 3, 0, device="cuda")
    x0 = wl.activations(M, shape.H, 3).float().cuda()
    cfg = B.make_cfg(shape, cap)
    ws = B.workspace(B.ghd_workspace_bytes(cfg, M, kv_len))
    outs = []
    try:
        for split in (0, 1):
            B.lib().ghd_debug_split_qkv_attn(split)
            x = x0.clone()
            kd, vd = model.upload_cache(kc.clone(), vc.clone())
            B.ghd_verify_layer(cfg, wd, kd, vd, x, torch.from_numpy(parent).cuda(), kv_len, ws=ws)
            assert B.ghd_step_status(ws) == 0
            outs.append((x, kd, vd))
    finally:
        B.lib().ghd_debug_split_qkv_attn(0)
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)


def test_verify_layer_7b_shape(B, model, orc32):
    w = wl.workload("layer7b")
    say("layer 7b", w.M, w.kv_len)
    run_layer_case(B, model, orc32, w.shape, w.M, w.kv_len, w.parent, w.seed)


def run_stack_case(B, model, orc32, shape, M, kv_len, parent, seed):
    cap = ((kv_len + M + 63) // 64) * 64
    layers = [wl.layer_weights(shape, seed, l) for l in range(shape.L)]
    head = wl.head_weights(shape, seed)
    caches = [wl.kv_cache(shape, cap, kv_len, seed, l) for l in range(shape.L)]
    x16 = wl.activations(M, shape.H, seed)
    kcs = [c[0].numpy().copy() for c in caches]
    vcs = [c[1].numpy().copy() for c in caches]
    ref_logits, ref_x = orc32.verify_stack(
        shape, [{k: v.numpy() for k, v in w.items()} for w in layers], kcs, vcs,
        {k: v.numpy() for k, v in head.items()}, x16.numpy(), parent, kv_len, round16=True)
    stack = model.build_stack(shape, cap, [model.upload_layer(w, shape.d) for w in layers],
                              [model.upload_cache(k, v) for k, v in caches], model.upload_head(head))
    x_out = torch.empty((M, shape.H), dtype=torch.float32, device="cuda")
    pd = torch.from_numpy(parent).cuda()
    ws = B.workspace(B.ghd_workspace_bytes(stack.cfg, M, kv_len))
    logits = B.ghd_verify_stack(stack, x16.cuda(), pd, kv_len, x_out=x_out, ws=ws)
    assert B.ghd_step_status(ws) == 0
    ok, ma, mr = close(x_out.cpu().numpy(), ref_x, 2e-2, 1e-2)
    assert ok, ("final residual", ma, mr)
    ok, ma, mr = close(logits.cpu().numpy(), ref_logits, 2e-2, 1e-2)
    assert ok, ("logits", ma, mr)
    return stack, logits, ref_logits, pd


def check_accept(B, orc32, logits, ref_logits, parent, pd, V, seed):
    """argmax must agree wherever the oracle's top-2 margin exceeds 1e-3; then
    plant a path from the agreed argmaxes and compare the accepted paths."""
    M = len(parent)
    top2 = np.sort(ref_logits, axis=1)[:, -2:]
    safe = (top2[:, 1] - top2[:, 0]) > 1e-3
    tokens = wl.draft_tokens(M, V, seed)
    _, _, _, ref_amax = orc32.accept_greedy(ref_logits, tokens, parent)
    # plant: every node on the path to the deepest leaf carries its parent's argmax
    depth = orc32.tree_depth(parent)
    j = int(np.argmax(depth))
    while parent[j] >= 0:
        tokens[j] = ref_amax[parent[j]]
        j = int(parent[j])
    res, amax = B.ghd_accept_greedy(logits, torch.from_numpy(tokens).cuda(), pd)
    res, amax = res.cpu().numpy(), amax.cpu().numpy()
    assert np.array_equal(amax[safe], ref_amax[safe])
    n, nxt, path, _ = orc32.accept_greedy(ref_logits, tokens, parent)
    if safe.all():
        assert res[0] == n and res[1] == nxt and np.array_equal(res[2:2 + n], path)
        assert n == depth.max() + 1
    return int(safe.sum())


def test_verify_stack_tiny_with_acceptance(B, model, orc32):
    w = wl.workload("tiny")
    say("stack tiny")
    stack, logits, ref_logits, pd = run_stack_case(B, model, orc32, w.shape, w.M, w.kv_len,
                                                   w.parent, w.seed)
    check_accept(B, orc32, logits, ref_logits, w.parent, pd, w.shape.V, w.seed)


def test_verify_stack_small_multilayer(B, model, orc32):
    shape = wl.ModelShape("small3", H=512, nh=4, d=128, F=1376, V=3000, L=3)
    parent = wl.tree_random(48, 5, 9)
    say("stack small3")
    stack, logits, ref_logits, pd = run_stack_case(B, model, orc32, shape, 48, 333, parent, 9)
    check_accept(B, orc32, logits, ref_logits, parent, pd, shape.V, 9)


@pytest.mark.parametrize("M,V,L", [(48, 3000, 2), (1, 1000, 1), (64, 10300, 1), (100, 300, 1)])
def test_verify_stack_argmax_in_the_lm_head_finish(B, model, orc32, M, V, L):
    """The row argmaxes reduced in the LM-head finish (per 16-column tile, then merged) are
    exactly the argmax of the logits the same call writes, lowest index on ties (the
    vocabulary holds duplicated rows, so maxima are tied), with and without the logits
    written; the walk from them is the oracle's acceptance."""
    shape = wl.ModelShape("amax%d" % V, H=256, nh=2, d=128, F=688, V=V, L=L)
    say("stack argmax", M, V, L)
    parent = wl.tree_random(M, 5, M + V)
    kv_len = 70
    cap = ((kv_len + M + 63) // 64) * 64
    layers = [wl.layer_weights(shape, 5, l) for l in range(L)]
    head = wl.head_weights(shape, 5)
    half = V // 2
    head["Wlm"][half:2 * half] = head["Wlm"][:half]          # logits of v and v + half are equal
    caches = [wl.kv_cache(shape, cap, kv_len, 5, l) for l in range(L)]
    stack = model.build_stack(shape, cap, [model.upload_layer(w, shape.d) for w in layers],
                              [model.upload_cache(k, v) for k, v in caches], model.upload_head(head))
    x16 = wl.activations(M, shape.H, 5).cuda()
    pd = torch.from_numpy(parent).cuda()
    ws = B.workspace(B.ghd_workspace_bytes(stack.cfg, M, kv_len))
    logits = torch.empty((M, V), dtype=torch.float32, device="cuda")
    amax = B.ghd_verify_stack_argmax(stack, x16, pd, kv_len, logits=logits, ws=ws)
    assert B.ghd_step_status(ws) == 0
    plain = B.ghd_verify_stack(stack, x16, pd, kv_len, ws=ws)
    assert torch.equal(plain, logits)
    lg = logits.cpu().numpy()
    first = np.array([int(np.flatnonzero(row == row.max())[0]) for row in lg], dtype=np.int32)
    # (a duplicated row is bit-equal to its twin only where both tiles are cut the same way
    # between workgroups, so not every row's maximum is tied - but some are)
    tied = sum(int((row == row.max()).sum() > 1) for row in lg)
    assert M < 8 or tied > 0
    assert np.array_equal(amax.cpu().numpy(), first)
    only = B.ghd_verify_stack_argmax(stack, x16, pd, kv_len, ws=ws)     # no logits written at all
    assert np.array_equal(only.cpu().numpy(), first)
    # the walk from the argmaxes
    tokens = wl.draft_tokens(M, V, 5)
    depth = orc32.tree_depth(parent)
    j = int(np.argmax(depth))
    while parent[j] >= 0:
        tokens[j] = first[parent[j]]
        j = int(parent[j])
    td = torch.from_numpy(tokens).cuda()
    res = B.ghd_accept_path(only, td, pd).cpu().numpy()
    n, nxt, path, ref_amax = orc32.accept_greedy(lg, tokens, parent)
    assert np.array_equal(ref_amax, first)
    assert res[0] == n == depth.max() + 1 and res[1] == nxt and np.array_equal(res[2:2 + n], path)
    res2, _ = B.ghd_accept_greedy(logits, td, pd)
    assert np.array_equal(res2.cpu().numpy()[:2 + n], res[:2 + n])


def test_stack_is_deterministic(B, model, orc32):
    shape = wl.ModelShape("small2", H=512, nh=4, d=128, F=1376, V=3000, L=2)
    parent = wl.tree_random(33, 4, 10)
    say("stack determinism")
    stack, logits, _, pd = run_stack_case(B, model, orc32, shape, 33, 100, parent, 10)
    x16 = wl.activations(33, shape.H, 10).cuda()
    again = B.ghd_verify_stack(stack, x16, pd, 100)
    torch.cuda.synchronize()
    assert torch.equal(logits, again)


@pytest.mark.parametrize("M,V", [(1, 10), (8, 1000), (64, 32000), (128, 257)])
def test_accept_greedy_same_logits_bit_exact(B, orc32, M, V):
    say("accept", M, V)
    rng = np.random.default_rng(M * 1000 + V)
    parent = wl.tree_random(M, 6, M)
    logits = rng.standard_normal((M, V)).astype(np.float32)
    # exact ties: the lowest index must win on both sides
    logits[:, V // 2] = logits.max(axis=1)
    if V > 3:
        logits[0, 1] = logits[0, V // 2]
    pd = torch.from_numpy(parent).cuda()
    lg = torch.from_numpy(logits).cuda()
    ref_amax = orc32.accept_greedy(logits, np.zeros(M, np.int32), parent)[3]
    depth = orc32.tree_depth(parent)
    targets = sorted(set([0, M - 1, int(np.argmax(depth)), M // 2]))
    for target in targets:
        tokens = np.full(M, -1, dtype=np.int32)
        j = target
        while parent[j] >= 0:
            tokens[j] = ref_amax[parent[j]]
            j = int(parent[j])
        # a duplicate sibling of the first accepted node
        sib = [c for c in range(1, M) if parent[c] == 0 and tokens[c] == -1]
        if sib and target != 0:
            tokens[sib[0]] = ref_amax[0]
        n, nxt, path, amax = orc32.accept_greedy(logits, tokens, parent)
        res, amax_g = B.ghd_accept_greedy(lg, torch.from_numpy(tokens).cuda(), pd)
        res, amax_g = res.cpu().numpy(), amax_g.cpu().numpy()
        assert np.array_equal(amax_g, amax)
        assert res[0] == n and res[1] == nxt and np.array_equal(res[2:2 + n], path)


# ---- commit of the accepted path: a pure copy, bit-exact -----------------------------

@pytest.mark.parametrize("nh,d,L,M,kv_len,tree,seed", [(4, 64, 1, 8, 128, "rand3", 0), (2, 128, 3, 64, 70, "rand5", 1),
                                                      (3, 128, 2, 128, 0, "chain", 2), (2, 64, 2, 1, 5, "chain", 3),
                                                      (32, 128, 2, 64, 2048, "rand5", 4)])
def test_commit_path_bit_exact(B, model, orc32, nh, d, L, M, kv_len, tree, seed):
    say("commit", nh, d, L, M, kv_len, tree)
    shape = wl.ModelShape("c", H=nh * d, nh=nh, d=d, F=8 * d, V=16, L=L)
    cap = ((kv_len + M + 63) // 64) * 64
    parent = make_tree(tree, M)
    depth = orc32.tree_depth(parent)
    rng = np.random.default_rng(seed)
    for node in {0, M - 1, int(np.argmax(depth)), int(rng.integers(0, M))}:
        path = []
        j = node
        while j >= 0:
            path.append(j)
            j = int(parent[j])
        path = np.array(path[::-1], dtype=np.int32)
        # every cache row distinct and recognisable
        ks = [torch.from_numpy(rng.integers(0, 0x7bff, size=(nh, cap, d)).astype(np.int16)).view(torch.float16)
              for _ in range(L)]
        vs = [torch.from_numpy(rng.integers(0, 0x7bff, size=(nh, cap, d)).astype(np.int16)).view(torch.float16)
              for _ in range(L)]
        dev = [model.upload_cache(k, v) for k, v in zip(ks, vs)]
        stack = B.Stack(B.make_cfg(shape, cap), [dict(g_attn=ks[0], Wqkv=ks[0], Wo=ks[0], g_ffn=ks[0],
                                                      Wgu=ks[0], Wdown=ks[0])] * L, dev,
                        dict(g_final=ks[0], Wlm=ks[0]))
        res = np.zeros(2 + M, dtype=np.int32)
        res[0] = len(path)
        res[2:2 + len(path)] = path
        B.ghd_commit_path(stack, torch.from_numpy(res).cuda(), M, kv_len)
        torch.cuda.synchronize()
        for l in range(L):
            k_ref, v_ref = ks[l].numpy().copy(), vs[l].numpy().copy()
            orc32.commit_path(k_ref, v_ref, kv_len, path)
            assert np.array_equal(dev[l][0].cpu().numpy().view(np.uint16), k_ref.view(np.uint16)), (node, l)
            assert np.array_equal(model.rows_of_v(dev[l][1]).cpu().numpy().view(np.uint16),
                                  v_ref.view(np.uint16)), (node, l)


# ---- full-size cases: the benchmark's configuration and the large shapes -------------

def run_big_stack(B, model, orc32, w, L):
    """The stack at its real shape through the same ghd_verify_stack call bench.py times.

    The oracle goes layer by layer so that only one layer's fp16 weights are on the host,
    twice: with fp16 rounding at the GPU path's rounding points (x16) and in pure fp32
    (x32).  Three checks:
      * every layer on its own, fed the oracle's residual stream: stated tolerance;
      * the free-running stack's logits (normalised quantities): stated tolerance;
      * the free-running stack's final residual stream: it is not normalised (rms grows
        like sqrt(layers)) and rounding noise accumulates over the layers, so the two
        oracle variants themselves drift apart by more than the tolerance at depth 32;
        the GPU must be no further from the pure-fp32 result than 1.5x the rounded oracle
        is (max and rms), plus the stated tolerance, and no further from the rounded oracle
        than twice that distance (both are printed).
    """
    shape = wl.with_layers(w.shape, L)
    M, kv_len, parent = w.M, w.kv_len, w.parent
    cap = w.capacity
    x16 = wl.activations(M, shape.H, w.seed)
    xr = x16.numpy().astype(np.float32)     # rounded oracle
    xp = xr.copy()                          # pure fp32 oracle
    layers, caches = [], []
    cfg = B.make_cfg(shape, cap)
    ws = B.workspace(B.ghd_workspace_bytes(cfg, M, kv_len))
    pd = torch.from_numpy(parent).cuda()
    for l in range(L):
        # generated on the GPU (seconds for the whole model); the oracle gets host copies
        lw = wl.layer_weights(shape, w.seed, l, device="cuda")
        kc, vc = wl.kv_cache(shape, cap, kv_len, w.seed, l, device="cuda")
        lwh = {k: v.cpu().numpy() for k, v in lw.items()}
        x_in = xr.copy()
        xr = orc32.verify_layer(shape, lwh, kc.cpu().numpy(), vc.cpu().numpy(), xr, parent, kv_len,
                                round16=True)
        xp = orc32.verify_layer(shape, lwh, kc.cpu().numpy(), vc.cpu().numpy(), xp, parent, kv_len,
                                round16=False)
        wd = model.upload_layer(lw, shape.d)
        # this layer alone, on the oracle's input (scratch copies of the cache)
        xg = torch.from_numpy(x_in).cuda()
        kc_d, vc_d = model.upload_cache(kc, vc)
        B.ghd_verify_layer(cfg, wd, kc_d.clone(), vc_d, xg, pd, kv_len, ws=ws)
        assert B.ghd_step_status(ws) == 0
        ok, ma, mr = close(xg.cpu().numpy(), xr, 2e-2, 1e-2)
        assert ok, ("layer", l, ma, mr)
        layers.append(wd)
        # the free-running stack gets this layer's cache too: the tree rows the layer-alone
        # run just wrote are simply written again
        caches.append((kc, vc_d))
        del lw, lwh
        if l % 4 == 3:
            say("  layer", l + 1, "of", L, "max abs err (layer alone) %.4f" % ma)
    head = wl.head_weights(shape, w.seed, device="cuda")
    hh = {k: v.cpu().numpy() for k, v in head.items()}
    ref_logits = orc32.lm_head(shape, hh["g_final"], hh["Wlm"], xr, True)
    stack = model.build_stack(shape, cap, layers, caches, model.upload_head(head))
    x_out = torch.empty((M, shape.H), dtype=torch.float32, device="cuda")
    logits = B.ghd_verify_stack(stack, x16.cuda(), pd, kv_len, x_out=x_out, ws=ws)
    assert B.ghd_step_status(ws) == 0
    ok, ma, mr = close(logits.cpu().numpy(), ref_logits, 2e-2, 1e-2)
    assert ok, ("logits", ma, mr)
    e_gpu = np.abs(x_out.cpu().numpy() - xp)
    e_orc = np.abs(xr - xp)
    say("  final residual vs pure fp32: gpu max %.4f rms %.5f | rounded oracle max %.4f rms %.5f"
        % (e_gpu.max(), np.sqrt((e_gpu ** 2).mean()), e_orc.max(), np.sqrt((e_orc ** 2).mean())))
    assert e_gpu.max() <= 1.5 * e_orc.max() + 2e-2
    assert np.sqrt((e_gpu ** 2).mean()) <= 1.5 * np.sqrt((e_orc ** 2).mean()) + 2e-3
    # ... and the GPU against the rounded oracle directly: two paths with the same rounding
    # points and different summation orders, each about e_orc away from pure fp32 with noise
    # of its own, so their distance is bounded by twice that (the triangle inequality through
    # pure fp32 with the factors above would allow 2.5)
    e_gr = np.abs(x_out.cpu().numpy() - xr)
    say("  final residual, gpu vs rounded oracle: max %.4f rms %.5f" % (e_gr.max(), np.sqrt((e_gr ** 2).mean())))
    assert e_gr.max() <= 2.0 * e_orc.max() + 2e-2
    assert np.sqrt((e_gr ** 2).mean()) <= 2.0 * np.sqrt((e_orc ** 2).mean()) + 2e-3
    # the row argmaxes from the LM-head finish are those of the logits just written
    amax = B.ghd_verify_stack_argmax(stack, x16.cuda(), pd, kv_len, ws=ws).cpu().numpy()
    lg = logits.cpu().numpy()
    assert np.array_equal(amax, np.array([int(np.flatnonzero(r == r.max())[0]) for r in lg], dtype=np.int32))
    checked = check_accept(B, orc32, logits, ref_logits, parent, pd, shape.V, w.seed)
    say("  argmax compared on", checked, "of", M, "rows")
    return checked


@pytest.mark.timeout(900)
def test_verify_stack_7b_full_size(B, model, orc32):
    """configs: 32-layer 7B-shaped stack + LM head, 64-node tree, 2048-token cache."""
    w = wl.workload("stack7b")
    say("stack 7b full size", w.M, w.kv_len, w.shape.L)
    assert run_big_stack(B, model, orc32, w, w.shape.L) > w.M // 2


@pytest.mark.timeout(600)
def test_verify_stack_13b_shape_two_layers(B, model, orc32):
    """13B-shaped layers (H=5120, 40 heads, F=13824), 8192-token cache, wide shallow
    64-node tree; two of the 40 layers + LM head keep the oracle to seconds."""
    w = wl.workload("stack13b")
    say("stack 13b shape, 2 layers", w.M, w.kv_len)
    run_big_stack(B, model, orc32, w, 2)


@pytest.mark.parametrize("M,tree", [(1, "chain"), (4, "chain"), (32, "rand5"), (128, "chain"),
                                    (128, "rand5")])
def test_verify_layer_7b_shape_tree_sizes(B, model, orc32, M, tree):
    """Tree-size sweep shapes: one 7B-shaped layer, 2048-token cache."""
    say("layer 7b sweep", M, tree)
    shape = wl.with_layers(wl.LLAMA_7B, 1)
    run_layer_case(B, model, orc32, shape, M, 2048, make_tree(tree, M), 3)


# ---- attention under a caller's mask (the other verification patterns of section 2.3) -----------
def mask_words(mask, extra_bits=False):
    """0/1 matrix [M, M] -> int64 [M, 2] bit masks (bit j of row i: token i sees token j);
    with extra_bits every bit from M on is set as well (must be ignored)."""
    M = mask.shape[0]
    words = np.zeros((M, 2), dtype=np.uint64)
    for i in range(M):
        for j in range(128):
            if (j < M and mask[i, j]) or (j >= M and extra_bits):
                words[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return torch.from_numpy(words.view(np.int64))


def pattern(kind, M, seed):
    rng = np.random.default_rng(seed)
    if kind == "random":                 # any relation, self included
        m = rng.random((M, M)) < 0.3
        m[np.arange(M), np.arange(M)] = True
    elif kind == "sequences":            # draft-model style: independent sequences side by side
        m = np.zeros((M, M), bool)
        L = 8
        for i in range(M):
            m[i, (i // L) * L:i + 1] = True
    elif kind == "ngram":                # Lookahead style: a causal window plus a few n-gram rows
        m = np.zeros((M, M), bool)
        for i in range(M):
            m[i, max(0, i - 5):i + 1] = True
            m[i, 0] = True
    else:                                # "sparse": most rows see only themselves
        m = np.eye(M, dtype=bool)
        m[::7, :3] = True
    return m.astype(np.uint8)


@pytest.mark.parametrize("M,nh,d,kv_len,kind,extra", [
    (40, 3, 128, 333, "random", False), (64, 4, 128, 1000, "sequences", True), (64, 2, 64, 70, "ngram", False),
    (128, 2, 128, 257, "random", False), (100, 2, 64, 0, "sparse", True), (16, 2, 128, 2048, "random", True),
    (1, 2, 128, 5, "random", True)])
def test_masked_attention(B, model, orc32, M, nh, d, kv_len, kind, extra):
    say("masked attention", M, nh, d, kv_len, kind)
    mask = pattern(kind, M, 13)
    q, kc, vc = attention_case(M, nh, d, kv_len, wl.tree_chain(M), 43)
    ref = orc32.masked_attention(q.numpy().astype(np.float32), kc.numpy(), vc.numpy(), mask, kv_len)
    ws = B.workspace(B.lib().ghd_attention_workspace_bytes(M, kv_len, nh, d))
    got = B.ghd_masked_attention(q.cuda(), *model.upload_cache(kc, vc), mask_words(mask, extra).cuda(),
                                 kv_len, ws=ws)
    assert B.ghd_step_status(ws) == 0
    ok, ma, mr = close(got.cpu().numpy(), ref, 5e-3, 5e-3)
    assert ok, (ma, mr)


def test_masked_attention_rows_without_keys_give_zeros(B, model, orc32):
    M, nh, d = 70, 2, 128
    mask = pattern("random", M, 5)
    mask[[3, 64, 69]] = 0
    say("masked attention, empty rows")
    q, kc, vc = attention_case(M, nh, d, 0, wl.tree_chain(M), 44)
    ref = orc32.masked_attention(q.numpy().astype(np.float32), kc.numpy(), vc.numpy(), mask, 0)
    got = B.ghd_masked_attention(q.cuda(), *model.upload_cache(kc, vc), mask_words(mask).cuda(), 0)
    got = got.cpu().numpy()
    assert np.all(got[[3, 64, 69]] == 0)
    ok, ma, mr = close(got, ref, 5e-3, 5e-3)
    assert ok, (ma, mr)


def test_step_can_be_captured_in_a_graph(B, model, orc32):
    """The step allocates nothing and records no memset: captured in a HIP graph it gives,
    on every replay (with eager steps and synchronisations in between), exactly the eager
    result."""
    shape = wl.ModelShape("graph2", H=512, nh=4, d=128, F=1376, V=3000, L=2)
    M, kv_len, seed = 24, 200, 12
    parent = wl.tree_random(M, 4, seed)
    say("graph capture")
    stack, logits_eager, _, pd = run_stack_case(B, model, orc32, shape, M, kv_len, parent, seed)
    x16 = wl.activations(M, shape.H, seed).cuda()
    tokens = torch.from_numpy(wl.draft_tokens(M, shape.V, seed)).cuda()
    ws = B.workspace(B.ghd_workspace_bytes(stack.cfg, M, kv_len))
    aws = B.workspace(B.lib().ghd_accept_workspace_bytes(M))
    logits = torch.empty((M, shape.V), dtype=torch.float32, device="cuda")
    res = torch.zeros(2 + M, dtype=torch.int32, device="cuda")
    amax = torch.empty(M, dtype=torch.int32, device="cuda")

    def step():
        B.ghd_verify_stack(stack, x16, pd, kv_len, logits=logits, ws=ws)
        B.ghd_accept_greedy(logits, tokens, pd, res=res, amax=amax, ws=aws)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()
        torch.cuda.synchronize()
        want_logits, want_res = logits.clone(), res.clone()
        assert torch.equal(want_logits, logits_eager)            # the step is deterministic
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step()
        torch.cuda.synchronize()
        for rep in range(4):
            logits.fill_(float("nan"))
            res.zero_()
            if rep % 2:
                step()                                           # eager work between replays
                torch.cuda.synchronize()
                logits.fill_(float("nan"))
            g.replay()
            torch.cuda.synchronize()
            assert B.ghd_step_status(ws) == 0
            assert torch.equal(logits, want_logits) and torch.equal(res, want_res), rep
