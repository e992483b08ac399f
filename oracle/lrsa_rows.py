"""ctypes front end of the row/column-wise C oracle (lrsa_rows.c) -- TEST INFRASTRUCTURE ONLY.

Used where the dense NumPy oracle (lrsa_ref.py) cannot hold an n x n matrix.  The C code is
itself pinned to the dense oracle on small inputs by the CPU tests.  Nothing in the product
package may import this module.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liblrsa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile lrsa_rows.c into liblrsa_oracle.so with gcc."""
    src = os.path.join(_HERE, "lrsa_rows.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-march=native", "-fopenmp", "-fPIC", "-shared",
                               "-std=c11", "-Wall", "-o", _SO, src, "-lm"])
    return _SO


class _Cfg(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in ("G", "n", "d", "S", "L", "K", "Ns", "local_prev")] + \
               [("scale", ctypes.c_double)]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
        _lib.lrsa_oracle_rows.restype = ctypes.c_int
        _lib.lrsa_oracle_cols.restype = ctypes.c_int
        _lib.lrsa_oracle_count.restype = ctypes.c_int64
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _cfg(Q, S, L, K, idx, local_prev, scale):
    G, n, d = Q.shape
    Ns = 0 if idx is None else idx.shape[0]
    return _Cfg(G, n, d, S, L, K, Ns, local_prev, 1.0 / np.sqrt(d) if scale is None else scale)


def attn_rows(Q, K, V, dO, idx, rows: Sequence[int], S: int, L: int, topk: int,
              local_prev: int = 1, scale=None, want_dq: bool = True) -> dict:
    """O, lse (and D, dQ when dO is given; want_dq=False leaves dQ out, which halves the time) of the listed
    rows for one KV group.  Q, dO: [G, n, d]; K, V: [n, d]; idx: [Ns, K] or None."""
    lib = _load()
    Q, K, V, dO = _f32(Q), _f32(K), _f32(V), _f32(dO)
    idx = None if idx is None or idx.size == 0 else np.ascontiguousarray(idx, dtype=np.int32)
    cfg = _cfg(Q, S, L, topk, idx, local_prev, scale)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    G, n, d = Q.shape
    out = {"O": np.empty((G, len(rows), d)), "lse": np.empty((G, len(rows)))}
    if dO is not None:
        out["D"] = np.empty((G, len(rows)))
        if want_dq:
            out["dQ"] = np.empty((G, len(rows), d))
    rc = lib.lrsa_oracle_rows(ctypes.byref(cfg), _p(Q), _p(K), _p(V), _p(dO), _p(idx), _p(rows),
                              ctypes.c_int64(len(rows)), _p(out["O"]), _p(out["lse"]),
                              _p(out.get("D")), _p(out.get("dQ")))
    if rc != 0:
        raise MemoryError("lrsa_oracle_rows failed")
    return out


def rows_seeing(cols: Sequence[int], n: int, S: int, L: int, idx, local_prev: int = 1) -> np.ndarray:
    """Sorted union of the query rows that see at least one of the listed key columns."""
    sel = np.zeros(n, dtype=bool)
    if idx is not None and np.size(idx):
        sel[np.asarray(idx).reshape(-1)] = True
    need = np.zeros(n, dtype=bool)
    for u in cols:
        if u < S or sel[u]:
            need[u:] = True
        else:
            end = min(n, S + ((u - S) // L + 1 + local_prev) * L)
            need[u:end] = True
    return np.nonzero(need)[0]


def attn_cols(Q, K, V, dO, idx, cols: Sequence[int], S: int, L: int, topk: int,
              local_prev: int = 1, scale=None, lse_all=None, D_all=None) -> dict:
    """dK, dV of the listed key columns for one KV group (summed over its G heads).
    lse_all, D_all ([G, n], from attn_rows over all rows) may be passed to skip their recomputation."""
    lib = _load()
    Q, K, V, dO = _f32(Q), _f32(K), _f32(V), _f32(dO)
    idx = None if idx is None or idx.size == 0 else np.ascontiguousarray(idx, dtype=np.int32)
    cfg = _cfg(Q, S, L, topk, idx, local_prev, scale)
    G, n, d = Q.shape
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    if lse_all is None or D_all is None:
        need = rows_seeing(cols, n, S, L, idx, local_prev)
        r = attn_rows(Q, K, V, dO, idx, need, S, L, topk, local_prev, scale)
        lse_all = np.full((G, n), np.nan)
        D_all = np.full((G, n), np.nan)
        lse_all[:, need] = r["lse"]
        D_all[:, need] = r["D"]
    lse_all = np.ascontiguousarray(lse_all, dtype=np.float64)
    D_all = np.ascontiguousarray(D_all, dtype=np.float64)
    out = {"dK": np.empty((len(cols), d)), "dV": np.empty((len(cols), d))}
    rc = lib.lrsa_oracle_cols(ctypes.byref(cfg), _p(Q), _p(K), _p(V), _p(dO), _p(idx), _p(lse_all),
                              _p(D_all), _p(cols), ctypes.c_int64(len(cols)), _p(out["dK"]), _p(out["dV"]))
    if rc != 0:
        raise MemoryError("lrsa_oracle_cols failed")
    return out


def attn_group(Q, K, V, dO, idx, S: int, L: int, topk: int, local_prev: int = 1, scale=None) -> dict:
    """Everything for one KV group: O, lse, dQ over all rows and dK, dV over all columns."""
    n = Q.shape[1]
    allpos = np.arange(n)
    out = attn_rows(Q, K, V, dO, idx, allpos, S, L, topk, local_prev, scale)
    out.update(attn_cols(Q, K, V, dO, idx, allpos, S, L, topk, local_prev, scale, out["lse"], out["D"]))
    return out


def count_visible(n, d, S, L, topk, idx, t, local_prev: int = 1) -> int:
    lib = _load()
    idx = None if idx is None or idx.size == 0 else np.ascontiguousarray(idx, dtype=np.int32)
    cfg = _Cfg(1, n, d, S, L, topk, 0 if idx is None else idx.shape[0], local_prev, 1.0)
    return int(lib.lrsa_oracle_count(ctypes.byref(cfg), _p(idx), ctypes.c_int64(t)))
