"""The allocation-free acceptance entry point against the workspace one.

ghd_accept_greedy_static keeps its per-segment maxima in an array of the library's
device image; every call on a GPU shares it.  Two calls in a row, the second on a
smaller input, must each equal ghd_accept_greedy on the same inputs bit for bit,
and the oracle's acceptance on those logits.
"""
import numpy as np
import pytest
import torch

from paper_2505_23219_amd import workloads as wl

pytestmark = pytest.mark.gpu


def planted(M, V, parent, seed):
    """Logits with a planted accepted path: random logits, tokens of a root path set to
    the parents' argmax."""
    rng = np.random.default_rng(seed)
    logits = rng.standard_normal((M, V)).astype(np.float32)
    tokens = rng.integers(0, V, size=M, dtype=np.int32)
    amax = logits.argmax(axis=1)
    node = M - 1
    while node > 0:                       # the root path of the last node is right
        tokens[node] = amax[parent[node]]
        node = parent[node]
    return logits, tokens


def run_both(B, orc32, M, V, parent, seed):
    logits, tokens = planted(M, V, parent, seed)
    ld, td, pd = torch.from_numpy(logits).cuda(), torch.from_numpy(tokens).cuda(), torch.from_numpy(parent).cuda()
    res_ws, amax_ws = B.ghd_accept_greedy(ld, td, pd)
    res_st = torch.full((2 + M,), -7, dtype=torch.int32, device="cuda")
    amax_st = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    B.ghd_accept_greedy_static(ld, td, pd, res_st, amax_st)
    torch.cuda.synchronize()
    n = int(res_ws[0])
    assert np.array_equal(res_st.cpu().numpy()[:2 + n], res_ws.cpu().numpy()[:2 + n])
    assert np.array_equal(amax_st.cpu().numpy(), amax_ws.cpu().numpy())
    ref_n, ref_next, ref_path, ref_amax = orc32.accept_greedy(logits, tokens, parent)
    r = res_st.cpu().numpy()
    assert r[0] == ref_n and r[1] == ref_next and np.array_equal(r[2:2 + ref_n], ref_path)
    assert np.array_equal(amax_st.cpu().numpy(), ref_amax)
    return n


def test_static_acceptance_equals_workspace_acceptance_twice():
    from oracle import Oracle
    from paper_2505_23219_amd import binding as B
    B.lib()
    orc32 = Oracle("f32")
    # the largest tree first, then a smaller input that reuses the same static array
    n_big = run_both(B, orc32, 128, 32000, wl.tree_random(128, 9, 11), 11)
    assert n_big >= 2
    n_small = run_both(B, orc32, 9, 257, wl.tree_random(9, 3, 12), 12)
    assert n_small >= 2
    run_both(B, orc32, 1, 10, wl.tree_chain(1), 13)


def test_static_acceptance_rejects_bad_arguments():
    from paper_2505_23219_amd import binding as B
    import ctypes as C
    lib = B.lib()
    t = torch.zeros(4, dtype=torch.float32, device="cuda")
    i = torch.zeros(4, dtype=torch.int32, device="cuda")
    p = lambda x: C.c_void_p(x.data_ptr())
    assert lib.ghd_accept_greedy_static(None, p(i), p(i), 1, 4, p(i), None, None) == B.GHD_ERR_NULL
    assert lib.ghd_accept_greedy_static(p(t), p(i), p(i), 129, 4, p(i), None, None) == B.GHD_ERR_SHAPE
    assert lib.ghd_accept_greedy_static(p(t), p(i), p(i), 0, 4, p(i), None, None) == B.GHD_ERR_SHAPE
