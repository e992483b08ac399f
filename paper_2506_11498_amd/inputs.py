"""Seeded synthetic inputs for the LRSA hot path (Q, K, V, dO).

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: it only draws random tensors, applies the
value structure each workload asks for, and rounds once to the workload dtype.

The paper's own workloads are activations of a 1.5B-parameter decoder on long
question-answer documents (Experiment section: 32K context, lag L = 1024,
evaluation grid L = context/32).  Those are not available, so each workload
here takes its shape family from that grid (L = n/32, K = L/4, bf16) and puts a
stated structure on top of N(0,1) draws.

Randomness is counter based (Philox): every (tensor, batch, head) slice has its
own key, so any subset of heads can be regenerated on its own and is identical
to the same slice of the full tensor.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Iterable, Optional

import numpy as np
import torch

_TENSOR_ID = {"Q": 1, "K": 2, "V": 3, "dO": 4, "structure": 5}


@dataclass(frozen=True)
class Workload:
    """Shape and value recipe of one synthetic LRSA workload.

    Symbols follow the paper's Method section: sink size S, lag (= chunk) size
    L, retained tokens per lag window K = r*L, head dimension d (d_h), sequence
    length n.
    """

    name: str
    B: int
    Hq: int
    Hkv: int
    d: int
    n: int
    L: int
    K: int
    S: int
    dtype: str  # "f32" or "bf16"
    seed: int
    structure: str  # none | outlier_channels | channel_scale | mean_drift | heavy_tokens

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", 1, 1, 1, 64, 1024, 128, 32, 4, "f32", 1001, "none"),
    "C2": Workload("C2", 2, 8, 8, 128, 4096, 256, 64, 16, "bf16", 1002, "outlier_channels"),
    "C3": Workload("C3", 1, 32, 32, 128, 16384, 512, 128, 16, "bf16", 1003, "channel_scale"),
    "C4": Workload("C4", 1, 32, 8, 128, 32768, 1024, 256, 64, "bf16", 1004, "mean_drift"),
    "C5": Workload("C5", 1, 64, 8, 128, 131072, 2048, 512, 64, "bf16", 1005, "heavy_tokens"),
    # the paper's own fine-tuning shape (Experiment Setup): 32K tokens, lag 1024, retention r = 0.5, on the
    # head geometry of the 1.5B model it trains (12 query heads, 2 KV heads, head_dim 128); sink as in C4
    "C6": Workload("C6", 1, 12, 2, 128, 32768, 1024, 512, 64, "bf16", 1006, "mean_drift"),
}


def _rng(seed: int, tensor: str, b: int, h: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, (_TENSOR_ID[tensor] << 40) | (b << 20) | h]))


def _normal(w: Workload, tensor: str, b: int, h: int) -> np.ndarray:
    return _rng(w.seed, tensor, b, h).standard_normal((w.n, w.d), dtype=np.float32)


def outlier_channels(w: Workload, h: int) -> np.ndarray:
    """The 4 distinct channel ids of KV head h that carry the x8 outliers (structure 'outlier_channels')."""
    return np.sort(_rng(w.seed, "structure", 0, h).permutation(w.d)[:4])


def _kv_slice(w: Workload, which: str, b: int, h: int, structured: bool) -> np.ndarray:
    x = _normal(w, which, b, h)
    if not structured or w.structure == "none":
        return x
    g = _rng(w.seed, "structure", 0 if w.structure in ("outlier_channels", "channel_scale") else b + 1, h)
    if w.structure == "outlier_channels":
        if which == "K":
            x[:, outlier_channels(w, h)] *= np.float32(8.0)
    elif w.structure == "channel_scale":
        if which == "K":
            x *= g.uniform(0.5, 4.0, size=(1, w.d)).astype(np.float32)
    elif w.structure == "mean_drift":
        if which == "K":
            steps = g.standard_normal((w.n, w.d), dtype=np.float32)
            steps[0] = 0.0
            x += np.cumsum(0.01 * steps.astype(np.float64), axis=0).astype(np.float32)
    elif w.structure == "heavy_tokens":
        heavy = g.random(w.n) < 0.01
        x[heavy] *= np.float32(10.0)
    else:
        raise ValueError(f"unknown structure {w.structure!r}")
    return x


def make_tensor(w: Workload, which: str, heads: Optional[Iterable[int]] = None,
                structured: bool = True) -> torch.Tensor:
    """One of Q, K, V, dO as a CPU tensor [B, H, n, d] in the workload dtype.

    `heads` restricts the head axis to the given head ids (query heads for Q and
    dO, KV heads for K and V); slices are identical to those of the full tensor.
    `structured=False` returns the plain N(0,1) draw without the workload's
    value structure (used by invariance tests).
    """
    nheads = w.Hq if which in ("Q", "dO") else w.Hkv
    heads = list(range(nheads)) if heads is None else list(heads)
    out = torch.empty((w.B, len(heads), w.n, w.d), dtype=w.torch_dtype)
    for b in range(w.B):
        for j, h in enumerate(heads):
            if which in ("K", "V"):
                x = _kv_slice(w, which, b, h, structured)
            else:
                x = _normal(w, which, b, h)
            out[b, j] = torch.from_numpy(x).to(w.torch_dtype)
    return out


def make_inputs(w: Workload, q_heads: Optional[Iterable[int]] = None,
                kv_heads: Optional[Iterable[int]] = None, structured: bool = True) -> Dict[str, torch.Tensor]:
    """Q, K, V, dO for workload `w` (CPU tensors, workload dtype, contiguous [B,H,n,d])."""
    return {
        "Q": make_tensor(w, "Q", q_heads),
        "K": make_tensor(w, "K", kv_heads, structured),
        "V": make_tensor(w, "V", kv_heads, structured),
        "dO": make_tensor(w, "dO", q_heads),
    }


def small_workload(name: str = "micro", *, B=1, Hq=2, Hkv=1, d=64, n=80, L=16, K=4, S=3,
                   dtype="f32", seed=7, structure="none") -> Workload:
    """A free-form small workload for edge-case and micro tests."""
    return Workload(name, B, Hq, Hkv, d, n, L, K, S, dtype, seed, structure)
