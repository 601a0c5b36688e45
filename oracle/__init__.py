"""ctypes front end of the CPU oracle (``ghd_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module,
and this module never imports the product package.

``Oracle("f32")`` is the reference the GPU path is compared with (fp32
arithmetic on the exact fp16 inputs); ``Oracle("f64")`` is the same source
built in double, used to bound the fp32 build's rounding noise.

All tensors cross this boundary as numpy arrays: fp16 data as ``uint16`` bit
patterns (``arr.view(np.uint16)``), working-type data as float32/float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ghd_oracle.c")
_LIBS = {"f32": ("libghd_oracle_f32.so", "float"), "f64": ("libghd_oracle_f64.so", "double")}


def build(force: bool = False) -> None:
    """Compile both precisions of the oracle with gcc."""
    for kind, (name, ctype) in _LIBS.items():
        out = os.path.join(_HERE, name)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O3", "-mavx2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-std=c11", "-Wall", "-DORC_REAL=" + ctype, _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


class _Cfg(C.Structure):
    _fields_ = [("H", C.c_int32), ("nh", C.c_int32), ("d", C.c_int32), ("F", C.c_int32),
                ("V", C.c_int32), ("L", C.c_int32), ("kv_capacity", C.c_int32),
                ("rope_base", C.c_float), ("rms_eps", C.c_float)]


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


class Oracle:
    def __init__(self, kind: str = "f32"):
        name, _ = _LIBS[kind]
        path = os.path.join(_HERE, name)
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_SRC):
            build()
        self.lib = C.CDLL(path)
        self.kind = kind
        self.real = np.float32 if kind == "f32" else np.float64
        self.creal = C.c_float if kind == "f32" else C.c_double
        self.lib.orc_real_bytes.restype = C.c_int
        assert self.lib.orc_real_bytes() == np.dtype(self.real).itemsize
        self.lib.orc_half_to_float.restype = C.c_float
        self.lib.orc_half_to_float.argtypes = [C.c_uint16]
        self.lib.orc_float_to_half.restype = C.c_uint16
        self.lib.orc_float_to_half.argtypes = [C.c_float]
        for fn in ("orc_tree_validate",):
            getattr(self.lib, fn).restype = C.c_int
        for fn in ("orc_tree_depth", "orc_tree_mask", "orc_linear", "orc_rmsnorm", "orc_rope",
                   "orc_swiglu", "orc_tree_attention", "orc_verify_layer", "orc_lm_head",
                   "orc_verify_stack", "orc_accept_greedy", "orc_commit_path", "orc_embed",
                   "orc_draft_logits", "orc_topk", "orc_tree_tokens", "orc_masked_attention"):
            getattr(self.lib, fn).restype = None
        self.lib.orc_tree_build.restype = C.c_int
        self.lib.orc_choose_width.restype = C.c_int

    # ---- helpers
    def _r(self, a) -> np.ndarray:
        return np.ascontiguousarray(a, dtype=self.real)

    def half_to_float(self, bits: int) -> float:
        return float(self.lib.orc_half_to_float(C.c_uint16(bits)))

    def float_to_half(self, f: float) -> int:
        return int(self.lib.orc_float_to_half(C.c_float(f)))

    # ---- tree
    def tree_validate(self, parent) -> bool:
        p = _i32(parent)
        return self.lib.orc_tree_validate(_p(p), C.c_int(len(p))) == 0

    def tree_depth(self, parent) -> np.ndarray:
        p = _i32(parent)
        out = np.zeros(len(p), dtype=np.int32)
        self.lib.orc_tree_depth(_p(p), C.c_int(len(p)), _p(out))
        return out

    def tree_mask(self, parent) -> np.ndarray:
        p = _i32(parent)
        M = len(p)
        out = np.zeros((M, M), dtype=np.uint8)
        self.lib.orc_tree_mask(_p(p), C.c_int(M), _p(out))
        return out

    # ---- pieces
    def linear(self, x, W16) -> np.ndarray:
        x = self._r(x)
        W = _u16(W16)
        M, K = x.shape
        N = W.shape[0]
        assert W.shape[1] == K
        y = np.empty((M, N), dtype=self.real)
        self.lib.orc_linear(_p(y), _p(x), _p(W), C.c_int(M), C.c_int(N), C.c_int(K))
        return y

    def rmsnorm(self, x, g16, eps: float) -> np.ndarray:
        x = self._r(x)
        g = _u16(g16)
        M, H = x.shape
        out = np.empty_like(x)
        self.lib.orc_rmsnorm(_p(out), _p(x), _p(g), C.c_int(M), C.c_int(H), self.creal(eps))
        return out

    def rope(self, t, pos, base: float) -> np.ndarray:
        t = self._r(t).copy()
        M, nh, d = t.shape
        pos = _i32(pos)
        self.lib.orc_rope(_p(t), _p(pos), C.c_int(M), C.c_int(nh), C.c_int(d), C.c_double(base))
        return t

    def swiglu(self, gu) -> np.ndarray:
        gu = self._r(gu)
        M, F2 = gu.shape
        a = np.empty((M, F2 // 2), dtype=self.real)
        self.lib.orc_swiglu(_p(a), _p(gu), C.c_int(M), C.c_int(F2 // 2))
        return a

    def tree_attention(self, q, kc16, vc16, parent, kv_len: int, scale: Optional[float] = None
                       ) -> np.ndarray:
        """q [M,nh,d]; kc16/vc16 [nh,cap,d] fp16 with tree rows at kv_len+j."""
        q = self._r(q)
        kc, vc = _u16(kc16), _u16(vc16)
        p = _i32(parent)
        M, nh, d = q.shape
        assert kc.shape[0] == nh and kc.shape[2] == d and kc.shape[1] >= kv_len + M
        if scale is None:
            scale = 1.0 / np.sqrt(d)
        out = np.empty_like(q)
        self.lib.orc_tree_attention(_p(out), _p(q), _p(kc), _p(vc), _p(p), C.c_int(M),
                                    C.c_int(kv_len), C.c_int(nh), C.c_int(d),
                                    C.c_int64(kc.shape[1] * d), C.c_int64(d), self.creal(scale))
        return out

    def masked_attention(self, q, kc16, vc16, mask, kv_len: int, scale: Optional[float] = None
                         ) -> np.ndarray:
        """As tree_attention, with the relation between the drafted tokens given as a 0/1
        matrix mask [M, M] (row i: the drafted tokens that token i sees)."""
        q = self._r(q)
        kc, vc = _u16(kc16), _u16(vc16)
        mk = np.ascontiguousarray(mask, dtype=np.uint8)
        M, nh, d = q.shape
        assert mk.shape == (M, M)
        assert kc.shape[0] == nh and kc.shape[2] == d and kc.shape[1] >= kv_len + M
        if scale is None:
            scale = 1.0 / np.sqrt(d)
        out = np.empty_like(q)
        self.lib.orc_masked_attention(_p(out), _p(q), _p(kc), _p(vc), _p(mk), C.c_int(M),
                                      C.c_int(kv_len), C.c_int(nh), C.c_int(d),
                                      C.c_int64(kc.shape[1] * d), C.c_int64(d), self.creal(scale))
        return out

    # ---- layer / stack
    @staticmethod
    def _cfg(shape, capacity: int) -> _Cfg:
        return _Cfg(shape.H, shape.nh, shape.d, shape.F, shape.V, shape.L, capacity,
                    shape.rope_base, shape.rms_eps)

    def verify_layer(self, shape, w: Dict[str, np.ndarray], kc16, vc16, x, parent, kv_len: int,
                     round16: bool) -> np.ndarray:
        """Returns the updated residual stream; kc16/vc16 (uint16 views) get the tree rows."""
        kc, vc = _u16(kc16), _u16(vc16)
        assert kc.flags.writeable and vc.flags.writeable
        cfg = self._cfg(shape, kc.shape[1])
        x = self._r(x).copy()
        p = _i32(parent)
        ws = {k: _u16(v) for k, v in w.items()}
        self.lib.orc_verify_layer(C.byref(cfg), _p(ws["g_attn"]), _p(ws["Wqkv"]), _p(ws["Wo"]),
                                  _p(ws["g_ffn"]), _p(ws["Wgu"]), _p(ws["Wdown"]), _p(kc), _p(vc),
                                  _p(x), _p(p), C.c_int(len(p)), C.c_int(kv_len),
                                  C.c_int(int(round16)))
        return x

    def lm_head(self, shape, g_final16, Wlm16, x, round16: bool) -> np.ndarray:
        x = self._r(x)
        cfg = self._cfg(shape, 0)
        g, W = _u16(g_final16), _u16(Wlm16)
        logits = np.empty((x.shape[0], shape.V), dtype=self.real)
        self.lib.orc_lm_head(C.byref(cfg), _p(g), _p(W), _p(x), _p(logits), C.c_int(x.shape[0]),
                             C.c_int(int(round16)))
        return logits

    def verify_stack(self, shape, layers: Sequence[Dict[str, np.ndarray]], kcs: List[np.ndarray],
                     vcs: List[np.ndarray], head: Optional[Dict[str, np.ndarray]], x_in16, parent,
                     kv_len: int, round16: bool):
        """Returns (logits or None, final residual stream)."""
        L = shape.L
        assert len(layers) == L and len(kcs) == L and len(vcs) == L
        keep = []

        def arr(name):
            a = (C.c_void_p * L)()
            for l in range(L):
                t = _u16(layers[l][name])
                keep.append(t)
                a[l] = t.ctypes.data
            return a

        def arr_kv(lst):
            a = (C.c_void_p * L)()
            for l in range(L):
                t = _u16(lst[l])
                assert t.flags.writeable and t.ctypes.data == _u16(lst[l]).ctypes.data
                keep.append(t)
                a[l] = t.ctypes.data
            return a

        cfg = self._cfg(shape, kcs[0].shape[1])
        x16 = _u16(x_in16)
        p = _i32(parent)
        M = len(p)
        x_out = np.empty((M, shape.H), dtype=self.real)
        logits = None
        g, W = None, None
        if head is not None:
            g, W = _u16(head["g_final"]), _u16(head["Wlm"])
            logits = np.empty((M, shape.V), dtype=self.real)
        self.lib.orc_verify_stack(C.byref(cfg), arr("g_attn"), arr("Wqkv"), arr("Wo"), arr("g_ffn"),
                                  arr("Wgu"), arr("Wdown"), arr_kv(kcs), arr_kv(vcs),
                                  _p(g) if g is not None else None,
                                  _p(W) if W is not None else None, _p(x16), _p(p), C.c_int(M),
                                  C.c_int(kv_len), _p(logits) if logits is not None else None,
                                  _p(x_out), C.c_int(int(round16)))
        return logits, x_out

    # ---- acceptance
    def accept_greedy(self, logits, tokens, parent):
        """Returns (path length, next token, path node indices, per-node argmax)."""
        lg = self._r(logits)
        t, p = _i32(tokens), _i32(parent)
        M, V = lg.shape
        res = np.zeros(2 + M, dtype=np.int32)
        amax = np.zeros(M, dtype=np.int32)
        self.lib.orc_accept_greedy(_p(lg), _p(t), _p(p), C.c_int(M), C.c_int(V), _p(res), _p(amax))
        n = int(res[0])
        return n, int(res[1]), res[2:2 + n].copy(), amax

    # ---- commit of the accepted path
    def commit_path(self, kc16, vc16, kv_len: int, path) -> None:
        """Moves the K/V rows of the accepted nodes to rows kv_len.. in path order, in place
        (caches [nh, cap, d] as uint16 views)."""
        kc, vc = _u16(kc16), _u16(vc16)
        assert kc.flags.writeable and vc.flags.writeable
        p = _i32(path)
        nh, cap, d = kc.shape
        self.lib.orc_commit_path(_p(kc), _p(vc), C.c_int(nh), C.c_int(cap), C.c_int(d),
                                 C.c_int(kv_len), _p(p), C.c_int(len(p)))

    # ---- drafting
    def embed(self, table16, tokens) -> np.ndarray:
        """Rows tokens[i] of the embedding table, as uint16 bit patterns [M, H]."""
        tb, t = _u16(table16), _i32(tokens)
        assert t.min() >= 0 and t.max() < tb.shape[0]
        x = np.empty((len(t), tb.shape[1]), dtype=np.uint16)
        self.lib.orc_embed(_p(x), _p(tb), _p(t), C.c_int(len(t)), C.c_int(tb.shape[1]))
        return x

    def draft_logits(self, x_row, g_final16, Wheads16, K: int, eps: float, round16: bool) -> np.ndarray:
        """Logits [K, V] of the K drafting heads (stacked [K*V, H]) for one hidden state [H]."""
        x = self._r(x_row).reshape(-1)
        g, W = _u16(g_final16), _u16(Wheads16)
        H = x.shape[0]
        assert W.shape[1] == H and W.shape[0] % K == 0
        V = W.shape[0] // K
        out = np.empty((K, V), dtype=self.real)
        self.lib.orc_draft_logits(_p(out), _p(x), _p(g), _p(W), C.c_int(K), C.c_int(V), C.c_int(H),
                                  self.creal(eps), C.c_int(int(round16)))
        return out

    def topk(self, v, R: int) -> np.ndarray:
        """Indices [rows, R] of the R largest entries of every row, best first, lowest index on ties."""
        a = self._r(v)
        rows, V = a.shape
        assert 1 <= R <= V
        idx = np.empty((rows, R), dtype=np.int32)
        self.lib.orc_topk(_p(idx), _p(a), C.c_int(rows), C.c_int(V), C.c_int(R))
        return idx

    def tree_tokens(self, parent, rank, topk, root_token: int) -> np.ndarray:
        p, r = _i32(parent), _i32(rank)
        tk = _i32(topk)
        out = np.empty(len(p), dtype=np.int32)
        self.lib.orc_tree_tokens(_p(out), _p(p), _p(r), C.c_int(len(p)), _p(tk), C.c_int(tk.shape[1]),
                                 C.c_int(int(root_token)))
        return out

    def tree_build(self, acc, M: int):
        """Greedy tree design from head accuracies acc [K, R].  Returns (parent, rank, expected
        acceptance length); the tree may have fewer than M nodes when the candidates run out."""
        a = np.ascontiguousarray(acc, dtype=np.float64)
        K, R = a.shape
        parent = np.zeros(M, dtype=np.int32)
        rank = np.zeros(M, dtype=np.int32)
        e = C.c_double(0.0)
        n = self.lib.orc_tree_build(_p(a), C.c_int(K), C.c_int(R), C.c_int(M), _p(parent), _p(rank),
                                    C.byref(e))
        return parent[:n].copy(), rank[:n].copy(), float(e.value)

    def choose_width(self, acc, widths, latency):
        """Index of the width with the most expected accepted tokens per unit of step time,
        and the rate of every candidate."""
        a = np.ascontiguousarray(acc, dtype=np.float64)
        w = _i32(widths)
        lat = np.ascontiguousarray(latency, dtype=np.float64)
        rate = np.zeros(len(w), dtype=np.float64)
        i = self.lib.orc_choose_width(_p(a), C.c_int(a.shape[0]), C.c_int(a.shape[1]), _p(w), _p(lat),
                                      C.c_int(len(w)), _p(rate))
        return int(i), rate

    # ---- one predict-then-verify step (section 2.1), composed of the pieces above
    def spec_step(self, shape, layers, kcs, vcs, head, table16, tokens, parent, kv_len: int,
                  round16: bool):
        """The tree's tokens (root = the last produced token, not yet in the cache) are
        embedded, verified in one pass, the longest valid root path is accepted and its K/V
        rows are committed (the caches are updated in place).  Returns a dict: `n` accepted
        nodes (the context grows by n), `produced` = the n tokens this step adds to the output
        (the accepted drafted tokens, then the model's next token), `next_token`, `path`,
        `amax`, `logits`, `x_last` = final hidden state of the last accepted node (input of
        the drafting heads)."""
        t, p = _i32(tokens), _i32(parent)
        x16 = self.embed(table16, t)
        logits, x_out = self.verify_stack(shape, layers, kcs, vcs, head, x16, p, kv_len, round16)
        n, nxt, path, amax = self.accept_greedy(logits, t, p)
        for l in range(shape.L):
            self.commit_path(kcs[l], vcs[l], kv_len, path)
        produced = [int(t[i]) for i in path[1:]] + [nxt]
        return {"n": n, "produced": produced, "next_token": nxt, "path": path, "amax": amax,
                "logits": logits, "x_last": x_out[path[-1]].copy()}

    def draft(self, x_last, g_final16, Wheads16, K: int, R: int, eps: float, parent, rank,
              root_token: int, round16: bool):
        """Tokens of the next tree from the drafting heads' top-R candidates.  Returns
        (tokens [M], topk [K, R], head logits [K, V])."""
        hl = self.draft_logits(x_last, g_final16, Wheads16, K, eps, round16)
        tk = self.topk(hl, R)
        return self.tree_tokens(parent, rank, tk, root_token), tk, hl
