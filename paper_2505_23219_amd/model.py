"""Device-side model tables: uploads fp16 weights, packs the matrices with
ghd_pack_weight and builds the pointer tables ghd_verify_stack takes.
Plumbing only; no arithmetic of the method happens here."""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import torch

from . import binding as B

MATRICES = ("Wqkv", "Wo", "Wgu", "Wdown")


def upload_layer(w: Dict[str, torch.Tensor], head_dim: int, device="cuda") -> Dict[str, torch.Tensor]:
    """fp16 layer weights (row-major, any device) -> gains + packed matrices on the GPU."""
    # the row orders ghd_verify_layer / ghd_verify_stack expect
    kinds = {"Wqkv": B.GHD_PACK_QKV, "Wgu": B.GHD_PACK_GATE_UP}
    out = {}
    for name, t in w.items():
        t = t.to(device)
        if name in MATRICES:
            out[name] = B.ghd_pack_weight(t, kinds.get(name, B.GHD_PACK_PLAIN), head_dim)
        else:
            out[name] = t.contiguous()
    return out


def upload_cache(k: torch.Tensor, v: torch.Tensor, device="cuda") -> Tuple[torch.Tensor, torch.Tensor]:
    """[nh, capacity, d] K and V (any device) -> the device layouts of the library:
    K as is, V channel-major [nh, d, capacity].  A copy, no arithmetic."""
    return k.to(device).contiguous(), v.to(device).transpose(1, 2).contiguous()


def rows_of_v(v_dev: torch.Tensor) -> torch.Tensor:
    """The library's channel-major V cache back as [nh, capacity, d] (for comparisons)."""
    return v_dev.transpose(1, 2)


def upload_head(h: Dict[str, torch.Tensor], device="cuda") -> Dict[str, torch.Tensor]:
    return {"g_final": h["g_final"].to(device).contiguous(),
            "Wlm": B.ghd_pack_weight(h["Wlm"].to(device))}


def build_stack(shape, capacity: int, layers: List[Dict[str, torch.Tensor]],
                caches: List[Tuple[torch.Tensor, torch.Tensor]],
                head: Dict[str, torch.Tensor]) -> B.Stack:
    return B.Stack(B.make_cfg(shape, capacity), layers, caches, head)
