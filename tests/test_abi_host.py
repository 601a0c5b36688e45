"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the header declares, and rejects bad arguments before touching
the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2505_23219_amd import binding as B
from paper_2505_23219_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # non-null, 16-byte aligned, never dereferenced on these paths


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2505_23219_amd.build import build
        build()
    return B.lib()


def test_header_functions_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "ghd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ghd_[a-z_0-9]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    seen = set()
    for code in range(0, -8, -1):
        s = B.status_str(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert B.status_str(-99) == "unknown status"


def test_tree_validate(lib):
    assert B.ghd_tree_validate([-1]) == B.GHD_OK
    assert B.ghd_tree_validate([-1, 0, 0, 2, 3]) == B.GHD_OK
    assert B.ghd_tree_validate([0]) == B.GHD_ERR_TREE
    assert B.ghd_tree_validate([-1, 1]) == B.GHD_ERR_TREE
    assert B.ghd_tree_validate([-1, 0, 2]) == B.GHD_ERR_TREE
    assert B.ghd_tree_validate([-1, -1]) == B.GHD_ERR_TREE
    assert B.ghd_tree_validate([-1] + [0] * 128) == B.GHD_ERR_SHAPE
    assert lib.ghd_tree_validate(None, 4) == B.GHD_ERR_NULL
    for M in (1, 2, 3, 4, 5):
        for parent in wl.all_trees(M):
            assert B.ghd_tree_validate(list(parent)) == B.GHD_OK
    for w in ("tiny", "layer7b", "stack7b", "stack13b"):
        assert B.ghd_tree_validate(list(wl.workload(w).parent)) == B.GHD_OK


def test_packed_size(lib):
    assert lib.ghd_packed_weight_bytes(16, 32) == 64 * 32 * 2          # one row block of four 16-row tiles
    assert lib.ghd_packed_weight_bytes(257, 129) == 320 * 160 * 2      # 17 tiles -> 5 row blocks, 5 k-steps
    assert lib.ghd_packed_weight_bytes(10241, 33) == 10368 * 64 * 2    # wide: 641 tiles -> 81 blocks of 8 tiles
    assert lib.ghd_packed_weight_bytes(32000, 4096) == 32000 * 4096 * 2
    assert lib.ghd_packed_weight_bytes(22016, 4096) == 22016 * 4096 * 2
    assert lib.ghd_packed_weight_bytes(12288, 4096) == 12288 * 4096 * 2   # same bytes as row-major
    assert lib.ghd_packed_weight_bytes(0, 32) == 0


def test_linear_rejects_bad_arguments(lib):
    f = lib.ghd_linear_skinny
    ok = dict(y=FAKE, x=FAKE, W=FAKE, M=16, N=64, K=64, ldx=64, ldy=64, flags=0, ws=FAKE,
              ws_bytes=1 << 30, stream=None)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["y"], a["x"], a["W"], a["M"], a["N"], a["K"], a["ldx"], a["ldy"], a["flags"],
                 a["ws"], a["ws_bytes"], a["stream"])

    assert call(y=None) == B.GHD_ERR_NULL
    assert call(x=None) == B.GHD_ERR_NULL
    assert call(W=None) == B.GHD_ERR_NULL
    assert call(M=0) == B.GHD_ERR_SHAPE
    assert call(M=129) == B.GHD_ERR_SHAPE
    assert call(K=60) == B.GHD_ERR_SHAPE
    assert call(ldx=56) == B.GHD_ERR_SHAPE
    assert call(ldy=8) == B.GHD_ERR_SHAPE
    assert call(flags=7) == B.GHD_ERR_SHAPE
    assert call(x=FAKE + 2) == B.GHD_ERR_ALIGN
    assert call(ldx=68) == B.GHD_ERR_ALIGN
    assert call(ws=None) == B.GHD_ERR_WORKSPACE
    assert call(ws_bytes=16) == B.GHD_ERR_WORKSPACE
    assert lib.ghd_linear_workspace_bytes(16, 64, 64) >= 16 * 256 * 4
    assert lib.ghd_linear_workspace_bytes(0, 64, 64) == 0


def test_attention_rejects_bad_arguments(lib):
    f = lib.ghd_tree_attention
    ok = dict(out=FAKE, q=FAKE, k=FAKE, v=FAKE, parent=FAKE, M=8, kv_len=100, nh=4, d=64,
              sh=64 * 256, st=64, vsh=64 * 256, vsc=256, scale=0.125, ws=FAKE, ws_bytes=1 << 30,
              stream=None)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["out"], a["q"], a["k"], a["v"], a["parent"], a["M"], a["kv_len"], a["nh"], a["d"],
                 a["sh"], a["st"], a["vsh"], a["vsc"], a["scale"], a["ws"], a["ws_bytes"], a["stream"])

    for name in ("out", "q", "k", "v", "parent"):
        assert call(**{name: None}) == B.GHD_ERR_NULL
    assert call(M=0) == B.GHD_ERR_SHAPE
    assert call(M=200) == B.GHD_ERR_SHAPE
    assert call(d=96) == B.GHD_ERR_SHAPE
    assert call(kv_len=-1) == B.GHD_ERR_SHAPE
    assert call(st=32) == B.GHD_ERR_SHAPE
    assert call(q=FAKE + 8) == B.GHD_ERR_ALIGN
    assert call(st=68) == B.GHD_ERR_ALIGN
    assert call(vsc=260) == B.GHD_ERR_ALIGN          # V rows must stay 16-byte aligned
    assert call(vsc=104) == B.GHD_ERR_CAPACITY       # fewer rows per channel than kv_len + M
    assert call(ws=None) == B.GHD_ERR_WORKSPACE
    assert call(ws_bytes=8) == B.GHD_ERR_WORKSPACE


def _cfg(shape, cap):
    return B.make_cfg(shape, cap)


def test_layer_and_stack_reject_bad_arguments(lib):
    cfg = _cfg(wl.TINY, 256)
    lw = B.LayerWeights(*([FAKE] * 6))
    kv = B.KV(FAKE, FAKE)
    need = lib.ghd_workspace_bytes(C.byref(cfg), 8, 128)
    assert need > 0

    def layer(cfgp=C.byref(cfg), lwp=C.byref(lw), kvp=C.byref(kv), x=FAKE, parent=FAKE, M=8,
              kv_len=128, ws=FAKE, ws_bytes=1 << 30):
        return lib.ghd_verify_layer(cfgp, lwp, kvp, x, parent, M, kv_len, ws, ws_bytes, None)

    assert layer(cfgp=None) == B.GHD_ERR_NULL
    assert layer(x=None) == B.GHD_ERR_NULL
    assert layer(parent=None) == B.GHD_ERR_NULL
    bad = B.LayerWeights(FAKE, None, FAKE, FAKE, FAKE, FAKE)
    assert layer(lwp=C.byref(bad)) == B.GHD_ERR_NULL
    assert layer(M=0) == B.GHD_ERR_SHAPE
    assert layer(M=129) == B.GHD_ERR_SHAPE
    assert layer(kv_len=250) == B.GHD_ERR_CAPACITY
    assert layer(x=FAKE + 4) == B.GHD_ERR_ALIGN
    assert layer(ws=None) == B.GHD_ERR_WORKSPACE
    assert layer(ws_bytes=need - 1) == B.GHD_ERR_WORKSPACE
    badcfg = _cfg(wl.ModelShape("bad", H=256, nh=4, d=32, F=64, V=10, L=1), 256)
    assert layer(cfgp=C.byref(badcfg)) == B.GHD_ERR_SHAPE
    badcfg = _cfg(wl.ModelShape("bad", H=250, nh=4, d=64, F=64, V=10, L=1), 256)
    assert layer(cfgp=C.byref(badcfg)) == B.GHD_ERR_SHAPE
    assert lib.ghd_workspace_bytes(C.byref(badcfg), 8, 128) == 0

    lws = (B.LayerWeights * 1)(lw)
    kvs = (B.KV * 1)(kv)

    def stack(g=FAKE, W=FAKE, x_in=FAKE, logits=FAKE, M=8, kv_len=128, ws=FAKE, ws_bytes=1 << 30):
        return lib.ghd_verify_stack(C.byref(cfg), lws, kvs, g, W, x_in, FAKE, M, kv_len, logits,
                                    None, ws, ws_bytes, None)

    assert stack(g=None) == B.GHD_ERR_NULL
    assert stack(logits=None) == B.GHD_ERR_NULL
    assert stack(M=130) == B.GHD_ERR_SHAPE
    assert stack(kv_len=249) == B.GHD_ERR_CAPACITY
    assert stack(x_in=FAKE + 2) == B.GHD_ERR_ALIGN
    assert stack(ws_bytes=100) == B.GHD_ERR_WORKSPACE

    def stack_argmax(amax=FAKE, logits=None, g=FAKE, M=8, ws=FAKE, ws_bytes=1 << 30):
        return lib.ghd_verify_stack_argmax(C.byref(cfg), lws, kvs, g, FAKE, FAKE, FAKE, M, 128, amax, logits,
                                           None, ws, ws_bytes, None)

    assert stack_argmax(amax=None) == B.GHD_ERR_NULL              # the argmaxes are what the call is for
    assert stack_argmax(g=None) == B.GHD_ERR_NULL
    assert stack_argmax(amax=FAKE + 2) == B.GHD_ERR_ALIGN
    assert stack_argmax(logits=FAKE + 4) == B.GHD_ERR_ALIGN
    assert stack_argmax(M=0) == B.GHD_ERR_SHAPE
    assert stack_argmax(ws=None) == B.GHD_ERR_WORKSPACE
    assert stack_argmax(ws_bytes=need - 1) == B.GHD_ERR_WORKSPACE


def test_pack_and_mask_reject_bad_arguments(lib):
    f = lib.ghd_pack_weight
    assert f(None, FAKE, 16, 32, 0, 0, None) == B.GHD_ERR_NULL
    assert f(FAKE, FAKE, 0, 32, 0, 0, None) == B.GHD_ERR_SHAPE
    assert f(FAKE, FAKE, 16, 32, 3, 0, None) == B.GHD_ERR_SHAPE
    assert f(FAKE, FAKE, 768, 32, B.GHD_PACK_QKV, 96, None) == B.GHD_ERR_SHAPE
    assert f(FAKE, FAKE, 100, 32, B.GHD_PACK_QKV, 64, None) == B.GHD_ERR_SHAPE
    assert f(FAKE, FAKE, 40, 32, B.GHD_PACK_GATE_UP, 0, None) == B.GHD_ERR_SHAPE
    assert f(FAKE + 4, FAKE, 16, 32, 0, 0, None) == B.GHD_ERR_ALIGN
    g = lib.ghd_tree_mask
    need = lib.ghd_tree_mask_workspace_bytes()
    assert need > 0
    assert g(None, 4, FAKE, FAKE, need, None) == B.GHD_ERR_NULL
    assert g(FAKE, 0, FAKE, FAKE, need, None) == B.GHD_ERR_SHAPE
    assert g(FAKE, 4, FAKE, None, need, None) == B.GHD_ERR_WORKSPACE
    assert g(FAKE, 4, FAKE, FAKE, 8, None) == B.GHD_ERR_WORKSPACE
    assert lib.ghd_step_status(None, None, None) == B.GHD_ERR_NULL


def test_accept_path_and_static_reject_bad_arguments(lib):
    p = lib.ghd_accept_path
    assert p(None, FAKE, FAKE, 4, FAKE, None) == B.GHD_ERR_NULL
    assert p(FAKE, None, FAKE, 4, FAKE, None) == B.GHD_ERR_NULL
    assert p(FAKE, FAKE, FAKE, 4, None, None) == B.GHD_ERR_NULL
    assert p(FAKE, FAKE, FAKE, 0, FAKE, None) == B.GHD_ERR_SHAPE
    assert p(FAKE, FAKE, FAKE, 129, FAKE, None) == B.GHD_ERR_SHAPE
    q = lib.ghd_accept_greedy_static
    assert q(None, FAKE, FAKE, 4, 10, FAKE, None, None) == B.GHD_ERR_NULL
    assert q(FAKE, FAKE, FAKE, 4, 10, None, None, None) == B.GHD_ERR_NULL
    assert q(FAKE, FAKE, FAKE, 129, 10, FAKE, None, None) == B.GHD_ERR_SHAPE
    assert q(FAKE, FAKE, FAKE, 4, 0, FAKE, None, None) == B.GHD_ERR_SHAPE


def test_accept_rejects_bad_arguments(lib):
    f = lib.ghd_accept_greedy
    assert f(None, FAKE, FAKE, 4, 10, FAKE, None, FAKE, 1 << 20, None) == B.GHD_ERR_NULL
    assert f(FAKE, FAKE, FAKE, 4, 10, None, None, FAKE, 1 << 20, None) == B.GHD_ERR_NULL
    assert f(FAKE, FAKE, FAKE, 0, 10, FAKE, None, FAKE, 1 << 20, None) == B.GHD_ERR_SHAPE
    assert f(FAKE, FAKE, FAKE, 4, 0, FAKE, None, FAKE, 1 << 20, None) == B.GHD_ERR_SHAPE
    assert f(FAKE, FAKE, FAKE, 4, 10, FAKE, None, None, 1 << 20, None) == B.GHD_ERR_WORKSPACE
    assert f(FAKE, FAKE, FAKE, 4, 10, FAKE, None, FAKE, 4, None) == B.GHD_ERR_WORKSPACE


def test_workspace_sizes_grow_with_the_problem(lib):
    cfg = _cfg(wl.LLAMA_7B, 4096)
    a = lib.ghd_workspace_bytes(C.byref(cfg), 1, 2048)
    b = lib.ghd_workspace_bytes(C.byref(cfg), 64, 2048)
    assert 0 < a < b < (1 << 30)
    assert lib.ghd_attention_workspace_bytes(64, 2048, 32, 128) > 0
    assert lib.ghd_accept_workspace_bytes(64) >= 64 * 4


def test_commit_path_rejects_bad_arguments(lib):
    cfg = _cfg(wl.TINY, 256)
    kv = B.KV(FAKE, FAKE)
    f = lib.ghd_commit_path
    assert f(None, C.byref(kv), FAKE, 8, 100, None) == B.GHD_ERR_NULL
    assert f(C.byref(cfg), None, FAKE, 8, 100, None) == B.GHD_ERR_NULL
    assert f(C.byref(cfg), C.byref(kv), None, 8, 100, None) == B.GHD_ERR_NULL
    assert f(C.byref(cfg), C.byref(kv), FAKE, 0, 100, None) == B.GHD_ERR_SHAPE
    assert f(C.byref(cfg), C.byref(kv), FAKE, 8, 250, None) == B.GHD_ERR_CAPACITY
    assert f(C.byref(cfg), C.byref(B.KV(FAKE + 2, FAKE)), FAKE, 8, 100, None) == B.GHD_ERR_ALIGN
    assert f(C.byref(cfg), C.byref(B.KV(None, FAKE)), FAKE, 8, 100, None) == B.GHD_ERR_NULL


# ---- drafting side -----------------------------------------------------------------------
@pytest.mark.parametrize("K,R,M,seed", [(4, 3, 16, 0), (5, 10, 64, 1), (2, 2, 7, 2), (3, 1, 9, 3), (5, 4, 128, 4)])
def test_tree_build_equals_the_oracle(lib, orc32, K, R, M, seed):
    rng = np.random.default_rng(seed)
    acc = np.sort(rng.uniform(0.01, 0.95, size=(K, R)), axis=1)[:, ::-1].copy()
    parent, rank, e = B.ghd_tree_build(acc.tolist(), M)
    p0, r0, e0 = orc32.tree_build(acc, M)
    assert parent == p0.tolist() and rank == r0.tolist() and e == e0
    assert B.ghd_tree_validate(parent) == B.GHD_OK


def test_tree_build_with_equal_accuracies_breaks_ties_like_the_oracle(lib, orc32):
    acc = np.full((3, 3), 0.5)
    parent, rank, e = B.ghd_tree_build(acc.tolist(), 12)
    p0, r0, e0 = orc32.tree_build(acc, 12)
    assert parent == p0.tolist() and rank == r0.tolist() and e == e0


def test_tree_build_rejects_bad_arguments(lib):
    acc = (C.c_double * 4)(0.5, 0.4, 0.3, 0.2)
    out = (C.c_int32 * 8)()
    ap, op = C.cast(acc, C.c_void_p), C.cast(out, C.c_void_p)
    assert lib.ghd_tree_build(None, 2, 2, 4, op, op, None) == B.GHD_ERR_NULL
    assert lib.ghd_tree_build(ap, 0, 2, 4, op, op, None) == B.GHD_ERR_SHAPE
    assert lib.ghd_tree_build(ap, 2, 2, 129, op, op, None) == B.GHD_ERR_SHAPE
    bad = (C.c_double * 4)(0.5, 1.5, 0.3, 0.2)
    assert lib.ghd_tree_build(C.cast(bad, C.c_void_p), 2, 2, 4, op, op, None) == B.GHD_ERR_SHAPE
    nan = (C.c_double * 4)(0.5, float("nan"), 0.3, 0.2)
    assert lib.ghd_tree_build(C.cast(nan, C.c_void_p), 2, 2, 4, op, op, None) == B.GHD_ERR_SHAPE


def test_drafting_calls_reject_bad_arguments(lib):
    assert lib.ghd_embed(None, FAKE, FAKE, 4, 64, 100, None) == B.GHD_ERR_NULL
    assert lib.ghd_embed(FAKE, FAKE, FAKE, 4, 60, 100, None) == B.GHD_ERR_SHAPE
    assert lib.ghd_embed(FAKE, FAKE, FAKE, 129, 64, 100, None) == B.GHD_ERR_SHAPE
    assert lib.ghd_embed(FAKE + 8, FAKE, FAKE, 4, 64, 100, None) == B.GHD_ERR_ALIGN
    assert lib.ghd_draft_workspace_bytes(5, 10, 4096, 32000) > 5 * 32000 * 4
    assert lib.ghd_draft_workspace_bytes(17, 10, 4096, 32000) == 0      # K <= 16
    assert lib.ghd_draft_workspace_bytes(5, 33, 4096, 32000) == 0       # R <= 32
    assert lib.ghd_draft_workspace_bytes(9, 4, 4096, 32000) == 0        # K*V <= 262144

    def draft(**kw):
        a = dict(g=FAKE, W=FAKE, K=2, R=3, H=64, V=100, eps=1e-6, x=FAKE, res=FAKE, parent=FAKE,
                 rank=FAKE, M=8, tokens=FAKE, topk=None, logits=None, ws=FAKE, ws_bytes=1 << 30)
        a.update(kw)
        return lib.ghd_draft_tokens(a["g"], a["W"], a["K"], a["R"], a["H"], a["V"], a["eps"], a["x"],
                                    a["res"], a["parent"], a["rank"], a["M"], a["tokens"], a["topk"],
                                    a["logits"], a["ws"], a["ws_bytes"], None)

    assert draft(W=None) == B.GHD_ERR_NULL
    assert draft(tokens=None) == B.GHD_ERR_NULL
    assert draft(R=101) == B.GHD_ERR_SHAPE
    assert draft(M=0) == B.GHD_ERR_SHAPE
    assert draft(H=60) == B.GHD_ERR_SHAPE
    assert draft(x=FAKE + 4) == B.GHD_ERR_ALIGN
    assert draft(ws=None) == B.GHD_ERR_WORKSPACE
    assert draft(ws_bytes=1024) == B.GHD_ERR_WORKSPACE


def test_spec_step_rejects_bad_arguments(lib):
    cfg = B.make_cfg(wl.TINY, 256)
    m = B.SpecModel(C.addressof(cfg), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, 3)
    need = lib.ghd_spec_workspace_bytes(C.byref(m), 8, 100)
    assert need > lib.ghd_workspace_bytes(C.byref(cfg), 8, 100)
    assert lib.ghd_spec_step(None, FAKE, FAKE, 8, 100, FAKE, FAKE, FAKE, need, None) == B.GHD_ERR_NULL
    assert lib.ghd_spec_step(C.byref(m), FAKE, FAKE, 8, 100, None, FAKE, FAKE, need, None) == B.GHD_ERR_NULL
    assert lib.ghd_spec_step(C.byref(m), FAKE, FAKE, 8, 250, FAKE, FAKE, FAKE, need, None) == B.GHD_ERR_CAPACITY
    assert lib.ghd_spec_step(C.byref(m), FAKE, FAKE, 8, 100, FAKE, FAKE, FAKE, need - 1, None) == B.GHD_ERR_WORKSPACE
    assert lib.ghd_spec_step(C.byref(m), FAKE, FAKE, 8, 100, FAKE, FAKE, None, need, None) == B.GHD_ERR_WORKSPACE
    m.K = 0
    assert lib.ghd_spec_step(C.byref(m), FAKE, FAKE, 8, 100, FAKE, FAKE, FAKE, need, None) == B.GHD_ERR_SHAPE
    assert lib.ghd_spec_workspace_bytes(C.byref(m), 8, 100) == 0


def test_choose_width_equals_the_oracle(lib, orc32):
    acc = wl.head_accuracies(5, 10)
    widths = [1, 2, 4, 8, 16, 32, 64, 128]
    for latency in ([110.0, 110.2, 110.5, 111.0, 112.5, 120.6, 141.6, 230.0], [1.0] * 8,
                    [float(w) for w in widths]):
        i, rate = B.ghd_choose_width(acc.tolist(), widths, latency)
        i0, rate0 = orc32.choose_width(acc, widths, latency)
        assert i == i0 and rate == rate0.tolist()
    assert lib.ghd_choose_width(None, 1, 1, None, None, 1, None) == B.GHD_ERR_NULL
    a = (C.c_double * 1)(0.5)
    w = (C.c_int32 * 1)(200)
    t = (C.c_double * 1)(1.0)
    cast = lambda x: C.cast(x, C.c_void_p)
    assert lib.ghd_choose_width(cast(a), 1, 1, cast(w), cast(t), 1, None) == B.GHD_ERR_SHAPE
    w[0], t[0] = 4, 0.0
    assert lib.ghd_choose_width(cast(a), 1, 1, cast(w), cast(t), 1, None) == B.GHD_ERR_SHAPE


def test_masked_attention_rejects_bad_arguments(lib):
    def call(**kw):
        a = dict(out=FAKE, q=FAKE, k=FAKE, v=FAKE, mask=FAKE, M=8, kv_len=64, nh=2, d=128, ksh=128 * 128,
                 kst=128, vsh=128 * 128, vsc=128, scale=0.1, ws=FAKE, ws_bytes=1 << 30)
        a.update(kw)
        return lib.ghd_masked_attention(a["out"], a["q"], a["k"], a["v"], a["mask"], a["M"], a["kv_len"],
                                        a["nh"], a["d"], a["ksh"], a["kst"], a["vsh"], a["vsc"], a["scale"],
                                        a["ws"], a["ws_bytes"], None)

    assert call(mask=None) == B.GHD_ERR_NULL
    assert call(mask=FAKE + 4) == B.GHD_ERR_ALIGN
    assert call(M=129) == B.GHD_ERR_SHAPE
    assert call(d=96) == B.GHD_ERR_SHAPE
    assert call(vsc=64) == B.GHD_ERR_CAPACITY
    assert call(ws=None) == B.GHD_ERR_WORKSPACE


def test_benchmark_loop_tree_is_pinned(lib, orc32):
    """The tree the decoding-loop benchmark verifies: the library's design equals the
    oracle's, and both equal the committed fixture (written by tests/golden/make_loop_tree.py
    from the oracle alone)."""
    import json
    with open(os.path.join(ROOT, "tests", "golden", "loop_tree.json")) as f:
        gold = json.load(f)
    acc = wl.head_accuracies(gold["heads"], gold["candidates"])
    parent, rank, e = B.ghd_tree_build(acc.tolist(), gold["nodes"])
    assert parent == gold["parent"] and rank == gold["rank"]
    assert abs(e - gold["expected_acceptance_length"]) < 1e-12
    p0, r0, e0 = orc32.tree_build(acc, gold["nodes"])
    assert p0.tolist() == gold["parent"] and r0.tolist() == gold["rank"] and e0 == e
    # a tree over 5 heads never goes deeper than 5 drafted levels
    assert orc32.tree_depth(p0).max() <= gold["heads"]
