"""Thin ctypes binding of libghd.so: argument marshalling only.

Every step of the verification path runs in the HIP kernels behind the C ABI
(include/ghd.h); this module turns torch tensors into raw device pointers and
checks status codes.  torch is used for device memory and streams, nothing
else.  There is no CPU fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libghd.so")

GHD_OK = 0
GHD_ERR_NULL, GHD_ERR_SHAPE, GHD_ERR_TREE, GHD_ERR_CAPACITY = -1, -2, -3, -4
GHD_ERR_WORKSPACE, GHD_ERR_ALIGN, GHD_ERR_HIP = -5, -6, -7
GHD_OUT_F32, GHD_OUT_F16 = 0, 1
GHD_PACK_PLAIN, GHD_PACK_QKV, GHD_PACK_GATE_UP = 0, 1, 2
GHD_MAX_M = 128


class GhdError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        extra = ""
        if status == GHD_ERR_HIP:
            extra = ", hip error %d" % lib().ghd_last_hip_error()
        super().__init__("%s: %s (status %d%s)" % (what, status_str(status), status, extra))


class ModelCfg(C.Structure):
    _fields_ = [("H", C.c_int32), ("nh", C.c_int32), ("d", C.c_int32), ("F", C.c_int32),
                ("V", C.c_int32), ("L", C.c_int32), ("kv_capacity", C.c_int32),
                ("rope_base", C.c_float), ("rms_eps", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g_attn", "Wqkv", "Wo", "g_ffn", "Wgu", "Wdown")]


class KV(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p)]


class SpecModel(C.Structure):
    _fields_ = [("cfg", C.c_void_p), ("layers_host", C.c_void_p), ("kv_host", C.c_void_p),
                ("g_final", C.c_void_p), ("Wlm", C.c_void_p), ("embed", C.c_void_p),
                ("Wheads", C.c_void_p), ("K", C.c_int32), ("R", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """Loads libghd.so (built in-tree by paper_2505_23219_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libghd.so is not built: run `python -m paper_2505_23219_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz, u32, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_size_t, C.c_uint32, C.c_float
        sig = {
            "ghd_status_str": (C.c_char_p, [C.c_int32]),
            "ghd_last_hip_error": (C.c_int, []),
            "ghd_tree_validate": (C.c_int32, [vp, i32]),
            "ghd_tree_mask": (C.c_int32, [vp, i32, vp, vp, sz, vp]),
            "ghd_tree_mask_workspace_bytes": (sz, []),
            "ghd_step_status": (C.c_int32, [vp, vp, vp]),
            "ghd_step_status_reset": (C.c_int32, [vp, vp]),
            "ghd_packed_weight_bytes": (sz, [i32, i32]),
            "ghd_pack_weight": (C.c_int32, [vp, vp, i32, i32, i32, i32, vp]),
            "ghd_linear_skinny": (C.c_int32, [vp, vp, vp, i32, i32, i32, i64, i64, u32, vp, sz, vp]),
            "ghd_linear_workspace_bytes": (sz, [i32, i32, i32]),
            "ghd_tree_attention": (C.c_int32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, i64, i64, f32,
                                               vp, sz, vp]),
            "ghd_attention_workspace_bytes": (sz, [i32, i32, i32, i32]),
            "ghd_tree_part_attention_coo": (C.c_int32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, i64, i64,
                                                        f32, vp, sz, vp]),
            "ghd_masked_attention": (C.c_int32, [vp, vp, vp, vp, vp, i32, i32, i32, i32, i64, i64, i64, i64, f32,
                                                 vp, sz, vp]),
            "ghd_verify_layer": (C.c_int32, [vp, vp, vp, vp, vp, i32, i32, vp, sz, vp]),
            "ghd_verify_stack": (C.c_int32, [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, sz,
                                             vp]),
            "ghd_workspace_bytes": (sz, [vp, i32, i32]),
            "ghd_verify_stack_argmax": (C.c_int32, [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz,
                                                    vp]),
            "ghd_accept_path": (C.c_int32, [vp, vp, vp, i32, vp, vp]),
            "ghd_accept_greedy": (C.c_int32, [vp, vp, vp, i32, i32, vp, vp, vp, sz, vp]),
            "ghd_accept_workspace_bytes": (sz, [i32]),
            "ghd_accept_greedy_static": (C.c_int32, [vp, vp, vp, i32, i32, vp, vp, vp]),
            "ghd_commit_path": (C.c_int32, [vp, vp, vp, i32, i32, vp]),
            "ghd_embed": (C.c_int32, [vp, vp, vp, i32, i32, i32, vp]),
            "ghd_tree_build": (C.c_int, [vp, i32, i32, i32, vp, vp, vp]),
            "ghd_choose_width": (C.c_int, [vp, i32, i32, vp, vp, i32, vp]),
            "ghd_draft_tokens": (C.c_int32, [vp, vp, i32, i32, i32, i32, f32, vp, vp, vp, vp, i32, vp, vp,
                                             vp, vp, sz, vp]),
            "ghd_draft_workspace_bytes": (sz, [i32, i32, i32, i32]),
            "ghd_spec_step": (C.c_int32, [vp, vp, vp, i32, i32, vp, vp, vp, sz, vp]),
            "ghd_spec_workspace_bytes": (sz, [vp, i32, i32]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


EXPORTS = ["ghd_status_str", "ghd_last_hip_error", "ghd_tree_validate", "ghd_tree_mask",
           "ghd_tree_mask_workspace_bytes", "ghd_step_status", "ghd_step_status_reset",
           "ghd_packed_weight_bytes", "ghd_pack_weight", "ghd_linear_skinny",
           "ghd_linear_workspace_bytes", "ghd_tree_attention", "ghd_attention_workspace_bytes",
           "ghd_masked_attention", "ghd_tree_part_attention_coo",
           "ghd_verify_layer", "ghd_verify_stack", "ghd_workspace_bytes", "ghd_accept_greedy",
           "ghd_accept_workspace_bytes", "ghd_accept_greedy_static", "ghd_verify_stack_argmax", "ghd_accept_path", "ghd_commit_path", "ghd_embed", "ghd_tree_build",
           "ghd_choose_width",
           "ghd_draft_tokens", "ghd_draft_workspace_bytes", "ghd_spec_step",
           "ghd_spec_workspace_bytes"]


def status_str(status: int) -> str:
    return lib().ghd_status_str(status).decode()


def _check(status: int, what: str) -> None:
    if status != GHD_OK:
        raise GhdError(status, what)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype)
    return t


def _devs(t: torch.Tensor, dtype) -> torch.Tensor:
    """A device tensor that may be a strided view (its last axis contiguous): the entry
    points that take explicit strides."""
    assert t.is_cuda and t.dtype == dtype and t.stride(-1) == 1, (t.device, t.dtype, t.stride())
    return t


def make_cfg(shape, kv_capacity: int) -> ModelCfg:
    return ModelCfg(shape.H, shape.nh, shape.d, shape.F, shape.V, shape.L, kv_capacity,
                    shape.rope_base, shape.rms_eps)


def workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ---- tree -------------------------------------------------------------------
def ghd_tree_validate(parent_host: Sequence[int]) -> int:
    arr = (C.c_int32 * len(parent_host))(*[int(p) for p in parent_host])
    return lib().ghd_tree_validate(C.cast(arr, C.c_void_p), len(parent_host))


def ghd_tree_mask(parent: torch.Tensor) -> torch.Tensor:
    """parent int32 [M] on the GPU -> int64 [M, 2] holding the 128-bit masks."""
    M = parent.numel()
    mask = torch.zeros((M, 2), dtype=torch.int64, device=parent.device)
    ws = workspace(lib().ghd_tree_mask_workspace_bytes(), parent.device)
    _check(lib().ghd_tree_mask(_ptr(_dev(parent, torch.int32)), M, _ptr(mask), _ptr(ws), ws.numel(),
                               _stream()), "ghd_tree_mask")
    return mask


def ghd_step_status(ws: torch.Tensor) -> int:
    """Synchronises the stream; 0 = the last step on `ws` completed, 1 = a bounded wait gave up."""
    st = C.c_int32(-1)
    _check(lib().ghd_step_status(_ptr(ws), C.byref(st), _stream()), "ghd_step_status")
    return int(st.value)


# ---- weights ----------------------------------------------------------------
def ghd_pack_weight(W: torch.Tensor, kind: int = GHD_PACK_PLAIN, head_dim: int = 0) -> torch.Tensor:
    """Row-major fp16 [N, K] on the GPU -> packed bytes (uint8 tensor)."""
    N, K = W.shape
    out = torch.empty(lib().ghd_packed_weight_bytes(N, K), dtype=torch.uint8, device=W.device)
    _check(lib().ghd_pack_weight(_ptr(out), _ptr(_dev(W, torch.float16)), N, K, kind, head_dim,
                                 _stream()), "ghd_pack_weight")
    return out


# ---- skinny linear ----------------------------------------------------------
def ghd_linear_skinny(x: torch.Tensor, Wp: torch.Tensor, N: int, out_dtype=torch.float32,
                      ws: Optional[torch.Tensor] = None, y: Optional[torch.Tensor] = None
                      ) -> torch.Tensor:
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=out_dtype, device=x.device)
    if ws is None:
        ws = workspace(lib().ghd_linear_workspace_bytes(M, N, K), x.device)
    flags = GHD_OUT_F16 if y.dtype == torch.float16 else GHD_OUT_F32
    assert y.stride(-1) == 1
    _check(lib().ghd_linear_skinny(_ptr(y), _ptr(_devs(x, torch.float16)), _ptr(Wp), M, N, K,
                                   x.stride(0), y.stride(0), flags, _ptr(ws), ws.numel(), _stream()),
           "ghd_linear_skinny")
    return y


# ---- tree attention ---------------------------------------------------------
def ghd_tree_attention(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                       parent: torch.Tensor, kv_len: int, scale: Optional[float] = None,
                       ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """q fp16 [M, nh, d]; k_cache fp16 [nh, cap, d]; v_cache fp16 [nh, d, cap]
    (channel-major); returns fp16 [M, nh, d]."""
    M, nh, d = q.shape
    out = torch.empty_like(q)
    if scale is None:
        scale = 1.0 / (d ** 0.5)
    if ws is None:
        ws = workspace(lib().ghd_attention_workspace_bytes(M, kv_len, nh, d), q.device)
    _check(lib().ghd_tree_attention(_ptr(out), _ptr(_dev(q, torch.float16)),
                                    _ptr(_devs(k_cache, torch.float16)),
                                    _ptr(_devs(v_cache, torch.float16)),
                                    _ptr(_dev(parent, torch.int32)), M, kv_len, nh, d,
                                    k_cache.stride(0), k_cache.stride(1), v_cache.stride(0),
                                    v_cache.stride(1), scale, _ptr(ws), ws.numel(),
                                    _stream()), "ghd_tree_attention")
    return out


def ghd_tree_part_attention_coo(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                                parent: torch.Tensor, kv_len: int, scale: Optional[float] = None,
                                ws: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The drafted tokens' own attention block from the nonzeros of the tree mask: token i
    over its ancestors-or-self only (cache rows kv_len + j); the committed rows are not
    attended.  Layouts as for ghd_tree_attention."""
    M, nh, d = q.shape
    if out is None:
        out = torch.empty_like(q)
    if scale is None:
        scale = 1.0 / (d ** 0.5)
    if ws is None:
        ws = workspace(lib().ghd_attention_workspace_bytes(M, kv_len, nh, d), q.device)
    _check(lib().ghd_tree_part_attention_coo(_ptr(out), _ptr(_dev(q, torch.float16)),
                                             _ptr(_dev(k_cache, torch.float16)),
                                             _ptr(_dev(v_cache, torch.float16)),
                                             _ptr(_dev(parent, torch.int32)), M, kv_len, nh, d,
                                             k_cache.stride(0), k_cache.stride(1), v_cache.stride(0),
                                             v_cache.stride(1), scale, _ptr(ws), ws.numel(),
                                             _stream()), "ghd_tree_part_attention_coo")
    return out


def ghd_masked_attention(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor,
                         mask: torch.Tensor, kv_len: int, scale: Optional[float] = None,
                         ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """As ghd_tree_attention with the relation between the drafted tokens given as int64
    [M, 2] bit masks (bit j of row i: token i sees token j)."""
    M, nh, d = q.shape
    out = torch.empty_like(q)
    if scale is None:
        scale = 1.0 / (d ** 0.5)
    if ws is None:
        ws = workspace(lib().ghd_attention_workspace_bytes(M, kv_len, nh, d), q.device)
    assert mask.shape == (M, 2)
    _check(lib().ghd_masked_attention(_ptr(out), _ptr(_dev(q, torch.float16)),
                                      _ptr(_dev(k_cache, torch.float16)),
                                      _ptr(_dev(v_cache, torch.float16)),
                                      _ptr(_dev(mask, torch.int64)), M, kv_len, nh, d,
                                      k_cache.stride(0), k_cache.stride(1), v_cache.stride(0),
                                      v_cache.stride(1), scale, _ptr(ws), ws.numel(),
                                      _stream()), "ghd_masked_attention")
    return out


# ---- layer / stack ----------------------------------------------------------
def layer_struct(w: dict) -> LayerWeights:
    return LayerWeights(*[w[n].data_ptr() for n in ("g_attn", "Wqkv", "Wo", "g_ffn", "Wgu", "Wdown")])


def ghd_verify_layer(cfg: ModelCfg, w: dict, k_cache: torch.Tensor, v_cache: torch.Tensor,
                     x: torch.Tensor, parent: torch.Tensor, kv_len: int,
                     ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x float32 [M, H], updated in place; w holds packed matrices and fp16 gains."""
    M = x.shape[0]
    if ws is None:
        ws = workspace(lib().ghd_workspace_bytes(C.byref(cfg), M, kv_len), x.device)
    lw, kv = layer_struct(w), KV(k_cache.data_ptr(), v_cache.data_ptr())
    _check(lib().ghd_verify_layer(C.byref(cfg), C.byref(lw), C.byref(kv), _ptr(_dev(x, torch.float32)),
                                  _ptr(_dev(parent, torch.int32)), M, kv_len, _ptr(ws), ws.numel(),
                                  _stream()), "ghd_verify_layer")
    return x


class Stack:
    """Host-side pointer tables of a whole model, built once."""

    def __init__(self, cfg: ModelCfg, layers: List[dict], caches: List[tuple], head: dict):
        self.cfg = cfg
        self.keep = (layers, caches, head)
        L = cfg.L
        assert len(layers) == L and len(caches) == L
        self.lw = (LayerWeights * L)(*[layer_struct(w) for w in layers])
        self.kv = (KV * L)(*[KV(k.data_ptr(), v.data_ptr()) for k, v in caches])
        self.g_final = head["g_final"]
        self.Wlm = head["Wlm"]


def ghd_verify_stack(stack: Stack, x_in: torch.Tensor, parent: torch.Tensor, kv_len: int,
                     logits: Optional[torch.Tensor] = None, x_out: Optional[torch.Tensor] = None,
                     ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    cfg = stack.cfg
    M = x_in.shape[0]
    if logits is None:
        logits = torch.empty((M, cfg.V), dtype=torch.float32, device=x_in.device)
    if ws is None:
        ws = workspace(lib().ghd_workspace_bytes(C.byref(cfg), M, kv_len), x_in.device)
    _check(lib().ghd_verify_stack(C.byref(cfg), stack.lw, stack.kv, _ptr(stack.g_final),
                                  _ptr(stack.Wlm), _ptr(_dev(x_in, torch.float16)),
                                  _ptr(_dev(parent, torch.int32)), M, kv_len, _ptr(logits),
                                  _ptr(x_out), _ptr(ws), ws.numel(), _stream()), "ghd_verify_stack")
    return logits


def ghd_verify_stack_argmax(stack: Stack, x_in: torch.Tensor, parent: torch.Tensor, kv_len: int,
                            logits: Optional[torch.Tensor] = None, x_out: Optional[torch.Tensor] = None,
                            ws: Optional[torch.Tensor] = None, amax: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The stack with the row argmaxes from the LM-head finish; returns amax int32 [M].
    `logits` (optional) is filled as by ghd_verify_stack when given."""
    cfg = stack.cfg
    M = x_in.shape[0]
    if amax is None:
        amax = torch.empty(M, dtype=torch.int32, device=x_in.device)
    if ws is None:
        ws = workspace(lib().ghd_workspace_bytes(C.byref(cfg), M, kv_len), x_in.device)
    _check(lib().ghd_verify_stack_argmax(C.byref(cfg), stack.lw, stack.kv, _ptr(stack.g_final),
                                         _ptr(stack.Wlm), _ptr(_dev(x_in, torch.float16)),
                                         _ptr(_dev(parent, torch.int32)), M, kv_len, _ptr(amax), _ptr(logits),
                                         _ptr(x_out), _ptr(ws), ws.numel(), _stream()), "ghd_verify_stack_argmax")
    return amax


def ghd_accept_path(amax: torch.Tensor, tokens: torch.Tensor, parent: torch.Tensor,
                    res: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The tree walk of greedy acceptance from given row argmaxes; returns res int32 [2+M]."""
    M = amax.shape[0]
    if res is None:
        res = torch.zeros(2 + M, dtype=torch.int32, device=amax.device)
    _check(lib().ghd_accept_path(_ptr(_dev(amax, torch.int32)), _ptr(_dev(tokens, torch.int32)),
                                 _ptr(_dev(parent, torch.int32)), M, _ptr(res), _stream()), "ghd_accept_path")
    return res


def ghd_workspace_bytes(cfg: ModelCfg, M: int, kv_len: int) -> int:
    return lib().ghd_workspace_bytes(C.byref(cfg), M, kv_len)


# ---- acceptance -------------------------------------------------------------
def ghd_accept_greedy(logits: torch.Tensor, tokens: torch.Tensor, parent: torch.Tensor,
                      res: Optional[torch.Tensor] = None, amax: Optional[torch.Tensor] = None,
                      ws: Optional[torch.Tensor] = None):
    """Returns (res int32 [2+M], amax int32 [M]) on the GPU; res[0] = length,
    res[1] = next token, res[2:2+res[0]] = accepted nodes, root first."""
    M, V = logits.shape
    if res is None:
        res = torch.zeros(2 + M, dtype=torch.int32, device=logits.device)
    if amax is None:
        amax = torch.empty(M, dtype=torch.int32, device=logits.device)
    if ws is None:
        ws = workspace(lib().ghd_accept_workspace_bytes(M), logits.device)
    _check(lib().ghd_accept_greedy(_ptr(_dev(logits, torch.float32)), _ptr(_dev(tokens, torch.int32)),
                                   _ptr(_dev(parent, torch.int32)), M, V, _ptr(res), _ptr(amax),
                                   _ptr(ws), ws.numel(), _stream()), "ghd_accept_greedy")
    return res, amax


def ghd_accept_greedy_static(logits: torch.Tensor, tokens: torch.Tensor, parent: torch.Tensor,
                             res: torch.Tensor, amax: Optional[torch.Tensor] = None) -> None:
    """ghd_accept_greedy without a workspace (the library's own static scratch); `res` and
    `amax` are the caller's: the call itself allocates nothing."""
    M, V = logits.shape
    _check(lib().ghd_accept_greedy_static(_ptr(_dev(logits, torch.float32)), _ptr(_dev(tokens, torch.int32)),
                                          _ptr(_dev(parent, torch.int32)), M, V, _ptr(_dev(res, torch.int32)),
                                          _ptr(amax) if amax is not None else None, _stream()),
           "ghd_accept_greedy_static")


def ghd_commit_path(stack: Stack, res: torch.Tensor, M: int, kv_len: int) -> None:
    """Moves the K/V rows of the accepted path (res from ghd_accept_greedy, on the device)
    to rows kv_len.. of every layer's cache, in place."""
    _check(lib().ghd_commit_path(C.byref(stack.cfg), stack.kv, _ptr(_dev(res, torch.int32)), M, kv_len,
                                 _stream()), "ghd_commit_path")


# ---- drafting side ------------------------------------------------------------
def ghd_embed(table: torch.Tensor, tokens: torch.Tensor, x16: Optional[torch.Tensor] = None) -> torch.Tensor:
    """table fp16 [V, H], tokens int32 [M] on the GPU -> fp16 [M, H]."""
    V, H = table.shape
    M = tokens.numel()
    if x16 is None:
        x16 = torch.empty((M, H), dtype=torch.float16, device=table.device)
    _check(lib().ghd_embed(_ptr(x16), _ptr(_dev(table, torch.float16)), _ptr(_dev(tokens, torch.int32)),
                           M, H, V, _stream()), "ghd_embed")
    return x16


def ghd_tree_build(acc, M: int):
    """acc: K rows of R head accuracies (host).  Returns (parent, rank, expected acceptance
    length) as Python lists / float."""
    K, R = len(acc), len(acc[0])
    flat = (C.c_double * (K * R))(*[float(a) for row in acc for a in row])
    parent, rank = (C.c_int32 * M)(), (C.c_int32 * M)()
    e = C.c_double(0.0)
    n = lib().ghd_tree_build(C.cast(flat, C.c_void_p), K, R, M, C.cast(parent, C.c_void_p),
                             C.cast(rank, C.c_void_p), C.cast(C.pointer(e), C.c_void_p))
    if n < 0:
        raise GhdError(n, "ghd_tree_build")
    return list(parent[:n]), list(rank[:n]), float(e.value)


def ghd_choose_width(acc, widths: Sequence[int], latency: Sequence[float]):
    """Returns (index of the chosen width, expected accepted tokens per unit time of each)."""
    K, R, n = len(acc), len(acc[0]), len(widths)
    flat = (C.c_double * (K * R))(*[float(a) for row in acc for a in row])
    w = (C.c_int32 * n)(*[int(x) for x in widths])
    lat = (C.c_double * n)(*[float(x) for x in latency])
    rate = (C.c_double * n)()
    i = lib().ghd_choose_width(C.cast(flat, C.c_void_p), K, R, C.cast(w, C.c_void_p),
                               C.cast(lat, C.c_void_p), n, C.cast(rate, C.c_void_p))
    if i < 0:
        raise GhdError(i, "ghd_choose_width")
    return i, list(rate)


def ghd_draft_tokens(g_final: torch.Tensor, Wheads: torch.Tensor, K: int, R: int, V: int, rms_eps: float,
                     x_final: torch.Tensor, res: torch.Tensor, parent: torch.Tensor, rank: torch.Tensor,
                     tokens: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """Returns (tokens int32 [M], topk int32 [K, R], head logits float [K, V]) on the GPU."""
    M, H = x_final.shape
    dev = x_final.device
    if tokens is None:
        tokens = torch.empty(M, dtype=torch.int32, device=dev)
    topk = torch.empty((K, R), dtype=torch.int32, device=dev)
    logits = torch.empty((K, V), dtype=torch.float32, device=dev)
    if ws is None:
        ws = workspace(lib().ghd_draft_workspace_bytes(K, R, H, V), dev)
    _check(lib().ghd_draft_tokens(_ptr(_dev(g_final, torch.float16)), _ptr(Wheads), K, R, H, V, rms_eps,
                                  _ptr(_dev(x_final, torch.float32)), _ptr(_dev(res, torch.int32)),
                                  _ptr(_dev(parent, torch.int32)), _ptr(_dev(rank, torch.int32)), M,
                                  _ptr(_dev(tokens, torch.int32)), _ptr(topk), _ptr(logits), _ptr(ws),
                                  ws.numel(), _stream()), "ghd_draft_tokens")
    return tokens, topk, logits


class SpecState:
    """Pointer block of ghd_spec_step for a Stack plus embedding table and drafting heads."""

    def __init__(self, stack: Stack, embed: torch.Tensor, Wheads: torch.Tensor, K: int, R: int):
        self.stack = stack
        self.keep = (embed, Wheads)
        self.c = SpecModel(C.addressof(stack.cfg), C.addressof(stack.lw), C.addressof(stack.kv),
                           stack.g_final.data_ptr(), stack.Wlm.data_ptr(),
                           _dev(embed, torch.float16).data_ptr(), Wheads.data_ptr(), K, R)

    def workspace_bytes(self, M: int, kv_len: int) -> int:
        return lib().ghd_spec_workspace_bytes(C.byref(self.c), M, kv_len)


def ghd_spec_step(spec: SpecState, parent: torch.Tensor, rank: torch.Tensor, kv_len: int,
                  tokens: torch.Tensor, res: torch.Tensor, ws: torch.Tensor) -> None:
    """One predict-then-verify step, enqueued; tokens (in/out) and res (out) on the GPU."""
    M = parent.numel()
    _check(lib().ghd_spec_step(C.byref(spec.c), _ptr(_dev(parent, torch.int32)),
                               _ptr(_dev(rank, torch.int32)), M, kv_len, _ptr(_dev(tokens, torch.int32)),
                               _ptr(_dev(res, torch.int32)), _ptr(ws), ws.numel(), _stream()),
           "ghd_spec_step")
