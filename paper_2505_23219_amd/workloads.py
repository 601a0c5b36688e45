"""Seeded synthetic inputs for the tree-verification step.

This module only *draws* inputs: model shapes, random fp16 weights, a committed
KV cache, draft trees (``parent[]`` arrays) and draft tokens.  It holds none of
the method's arithmetic (no linear layer, attention, normalisation, rotation or
acceptance code) and imports neither the HIP binding nor the CPU oracle, so
both sides of a parity test can be fed the same bits from here.

The shapes stand in for the paper's Vicuna-7B + Medusa workload (section 4.1,
"Model and Speculative Decoding"): the trained weights and the four evaluation
datasets are not available, so weights are random and draft tokens are uniform.
"""
from __future__ import annotations

import dataclasses
import hashlib
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch


# --------------------------------------------------------------------------
# shapes
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class ModelShape:
    """LLaMA-style decoder shape (the architecture of the paper's Vicuna-7B)."""
    name: str
    H: int          # hidden size
    nh: int         # attention heads (multi-head attention: kv heads == heads)
    d: int          # head dim
    F: int          # SwiGLU FFN size
    V: int          # vocabulary (LM head rows)
    L: int          # layers
    rope_base: float = 10000.0
    rms_eps: float = 1e-6

    def weight_bytes_per_layer(self) -> int:
        return 2 * (4 * self.H * self.H + 3 * self.H * self.F)

    def lm_head_bytes(self) -> int:
        return 2 * self.V * self.H


TINY = ModelShape("tiny", H=256, nh=4, d=64, F=688, V=1000, L=1)
LLAMA_7B = ModelShape("7b", H=4096, nh=32, d=128, F=11008, V=32000, L=32)
LLAMA_13B = ModelShape("13b", H=5120, nh=40, d=128, F=13824, V=32000, L=40)


def with_layers(shape: ModelShape, L: int) -> ModelShape:
    return dataclasses.replace(shape, L=L)


# --------------------------------------------------------------------------
# draft trees.  parent[0] == -1, 0 <= parent[i] < i (topological order).
# --------------------------------------------------------------------------
def _depths(parent: Sequence[int]) -> List[int]:
    depth = [0] * len(parent)
    for i in range(1, len(parent)):
        depth[i] = depth[parent[i]] + 1
    return depth


def tree_chain(M: int) -> np.ndarray:
    """A single path: node i hangs under node i-1."""
    return np.arange(-1, M - 1, dtype=np.int32)


def tree_star(M: int) -> np.ndarray:
    """Every drafted node is a child of the root."""
    p = np.zeros(M, dtype=np.int32)
    p[0] = -1
    return p


def tree_random(M: int, max_depth: int, seed: int) -> np.ndarray:
    """parent[i] uniform over earlier nodes whose depth is < max_depth."""
    rng = np.random.default_rng(seed)
    parent = [-1]
    depth = [0]
    for i in range(1, M):
        cands = [j for j in range(i) if depth[j] < max_depth]
        p = int(cands[int(rng.integers(len(cands)))])
        parent.append(p)
        depth.append(depth[p] + 1)
    return np.asarray(parent, dtype=np.int32)


def tree_product(branching: Sequence[int]) -> np.ndarray:
    """Full product tree: every node at level l has branching[l] children.

    Levels are emitted breadth first, so the order is topological.  This is the
    shape of a Medusa verification tree in which head l contributes its top
    branching[l] candidates under every candidate of head l-1 (section 2.3).
    """
    parent = [-1]
    level = [0]
    for b in branching:
        nxt = []
        for node in level:
            for _ in range(b):
                parent.append(node)
                nxt.append(len(parent) - 1)
        level = nxt
    return np.asarray(parent, dtype=np.int32)


def tree_medusa(M: int, branching: Sequence[int], seed: int) -> np.ndarray:
    """Product tree cut down to M nodes by seeded frontier sampling.

    Start from {root}; repeatedly add a uniformly chosen node of the product
    tree whose parent is already in; insertion order is node order.
    """
    full = tree_product(branching)
    if M > len(full):
        raise ValueError("product tree has only %d nodes" % len(full))
    rng = np.random.default_rng(seed)
    new_index = {0: 0}
    parent = [-1]
    frontier = [i for i in range(1, len(full)) if full[i] == 0]
    while len(parent) < M:
        pick = frontier.pop(int(rng.integers(len(frontier))))
        new_index[pick] = len(parent)
        parent.append(new_index[int(full[pick])])
        frontier.extend(i for i in range(1, len(full)) if full[i] == pick)
    return np.asarray(parent, dtype=np.int32)


def tree_wide_shallow(M: int, fanout: int, seed: int) -> np.ndarray:
    """Depth-2 tree: root, `fanout` children, the rest grandchildren whose
    parent is uniform over the children."""
    if M < 1 + fanout:
        raise ValueError("M too small for the fanout")
    rng = np.random.default_rng(seed)
    parent = [-1] + [0] * fanout
    for _ in range(M - 1 - fanout):
        parent.append(1 + int(rng.integers(fanout)))
    return np.asarray(parent, dtype=np.int32)


def all_trees(M: int):
    """Every valid parent[] of size M (there are (M-1)! of them)."""
    def rec(prefix):
        if len(prefix) == M:
            yield np.asarray(prefix, dtype=np.int32)
            return
        for p in range(len(prefix)):
            yield from rec(prefix + [p])
    yield from rec([-1])


def tree_max_depth(parent: Sequence[int]) -> int:
    return max(_depths(list(parent)))


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------
def _gen(seed: int, *tags, device: str = "cpu") -> torch.Generator:
    """A generator whose stream depends on (seed, tags) only, so any layer or
    matrix can be drawn on its own."""
    h = hashlib.sha256(repr((int(seed),) + tuple(tags)).encode()).digest()
    g = torch.Generator(device=device)
    g.manual_seed(int.from_bytes(h[:8], "little") & 0x7FFFFFFFFFFFFFFF)
    return g


def _normal_fp16(shape, std: float, mean: float, gen: torch.Generator,
                 device: str) -> torch.Tensor:
    # drawn in fp32, rounded once to fp16: these fp16 bits are the input
    t = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return t.to(torch.float16)


def layer_weights(shape: ModelShape, seed: int, layer: int,
                  device: str = "cpu") -> Dict[str, torch.Tensor]:
    """fp16 weights of one decoder layer, row-major [out_features, in_features].

    Wqkv stacks the q, k and v projections (rows [0,H), [H,2H), [2H,3H));
    Wgu stacks gate then up.  Matrices ~ N(0, 0.02); norm gains ~ 1 + N(0, 0.02)
    so that a dropped gain multiply is visible.
    """
    H, F = shape.H, shape.F
    out = {}
    for name, shp in (("Wqkv", (3 * H, H)), ("Wo", (H, H)),
                      ("Wgu", (2 * F, H)), ("Wdown", (H, F))):
        out[name] = _normal_fp16(shp, 0.02, 0.0,
                                 _gen(seed, shape.name, layer, name, device=device), device)
    for name in ("g_attn", "g_ffn"):
        out[name] = _normal_fp16((H,), 0.02, 1.0,
                                 _gen(seed, shape.name, layer, name, device=device), device)
    return out


def head_weights(shape: ModelShape, seed: int, device: str = "cpu") -> Dict[str, torch.Tensor]:
    """Final norm gain and LM head [V, H]."""
    return {
        "g_final": _normal_fp16((shape.H,), 0.02, 1.0,
                                _gen(seed, shape.name, "g_final", device=device), device),
        "Wlm": _normal_fp16((shape.V, shape.H), 0.02, 0.0,
                            _gen(seed, shape.name, "Wlm", device=device), device),
    }


def kv_cache(shape: ModelShape, capacity: int, kv_len: int, seed: int, layer: int,
             device: str = "cpu"):
    """Committed cache of one layer, head-major [nh, capacity, d] fp16.

    Rows [0, kv_len) ~ N(0, 1) (taken as already rotated keys); the rest zero.
    Returns (k, v).
    """
    outs = []
    for name in ("k", "v"):
        t = torch.zeros((shape.nh, capacity, shape.d), dtype=torch.float16, device=device)
        if kv_len > 0:
            t[:, :kv_len, :] = _normal_fp16((shape.nh, kv_len, shape.d), 1.0, 0.0,
                                            _gen(seed, shape.name, layer, "kv", name,
                                                 device=device), device)
        outs.append(t)
    return outs[0], outs[1]


def activations(M: int, width: int, seed: int, tag: str = "x", std: float = 1.0,
                device: str = "cpu") -> torch.Tensor:
    """[M, width] fp16 ~ N(0, std)."""
    return _normal_fp16((M, width), std, 0.0, _gen(seed, tag, M, width, device=device), device)


def embedding_table(shape: ModelShape, seed: int, device: str = "cpu") -> torch.Tensor:
    """Token embeddings [V, H] fp16 ~ N(0, 1)."""
    return _normal_fp16((shape.V, shape.H), 1.0, 0.0, _gen(seed, shape.name, "embed", device=device),
                        device)


def drafting_heads(shape: ModelShape, K: int, seed: int, device: str = "cpu") -> torch.Tensor:
    """The K drafting heads as one stacked matrix [K*V, H] fp16 ~ N(0, 0.02) (untrained:
    their candidates are as good as random)."""
    return _normal_fp16((K * shape.V, shape.H), 0.02, 0.0,
                        _gen(seed, shape.name, "heads", K, device=device), device)


def head_accuracies(K: int, R: int) -> np.ndarray:
    """Synthetic per-head, per-candidate accuracies [K, R] of the shape reported for
    multi-head drafting: the first candidate of the first head is right most often, and
    accuracy falls with the head index and, faster, with the candidate rank."""
    k = np.arange(K)[:, None]
    r = np.arange(R)[None, :]
    return 0.6 * 0.8 ** k * 0.35 ** r


def draft_tokens(M: int, V: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng([seed, 7919])
    return rng.integers(0, V, size=M, dtype=np.int32)


# --------------------------------------------------------------------------
# the named workloads
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    kv_len: int
    M: int
    parent: np.ndarray
    seed: int
    with_head: bool

    @property
    def capacity(self) -> int:
        # committed rows + tree rows, rounded up to whole 64-row tiles
        return ((self.kv_len + self.M + 63) // 64) * 64

    def algorithmic_bytes(self) -> int:
        """Bytes the step must move: every weight once, every cache row
        (committed + tree) of every layer once."""
        s = self.shape
        w = s.L * s.weight_bytes_per_layer() + (s.lm_head_bytes() if self.with_head else 0)
        kv = 2 * 2 * s.L * (self.kv_len + self.M) * s.H
        return w + kv


def workload(name: str) -> Workload:
    if name == "tiny":
        return Workload(name, TINY, 128, 8, tree_random(8, 3, 0), 0, True)
    if name == "layer7b":
        return Workload(name, with_layers(LLAMA_7B, 1), 1024, 16,
                        tree_medusa(16, (4, 2, 1, 1), 1), 1, False)
    if name == "stack7b":
        return Workload(name, LLAMA_7B, 2048, 64, tree_random(64, 5, 2), 2, True)
    if name == "stack7b_decode":
        return Workload(name, LLAMA_7B, 2048, 1, tree_chain(1), 2, True)
    if name == "stack13b":
        return Workload(name, LLAMA_13B, 8192, 64, tree_wide_shallow(64, 32, 4), 4, True)
    raise KeyError(name)


def sweep_workload(M: int, kind: str, L: int = 1) -> Workload:
    """One 7B-shaped layer at KV 2048 for the tree-size sweep."""
    if M == 1 or kind == "chain":
        parent = tree_chain(M)
    elif kind == "bushy":
        parent = tree_random(M, 5, 3)
    else:
        raise KeyError(kind)
    return Workload("sweep_%s_%d" % (kind, M), with_layers(LLAMA_7B, L), 2048, M, parent, 3, False)
