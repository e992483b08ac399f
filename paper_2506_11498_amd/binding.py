"""Thin ctypes binding of liblrsa.so: argument marshalling only.

Every step of the path (score, select, attention forward and backward) runs in the HIP
kernels behind the C ABI declared in include/lrsa.h; torch is used here for device memory
and the current stream, nothing else.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblrsa.so")

LRSA_F32, LRSA_BF16 = 0, 1
IMPL_AUTO, IMPL_GENERIC, IMPL_COMPACT = 0, 1, 2
WS_SCORE, WS_SELECT, WS_ATTN_FWD, WS_ATTN_BWD, WS_DECODE_ATTN = 0, 1, 2, 3, 4

EXPORTS = ("lrsa_abi_version", "lrsa_last_error", "lrsa_num_scored_chunks", "lrsa_score_route", "lrsa_score_poll_limit", "lrsa_workspace_bytes",
           "lrsa_score", "lrsa_select", "lrsa_score_select", "lrsa_check_idx", "lrsa_attn_fwd", "lrsa_attn_bwd",
           "lrsa_cache_compress", "lrsa_decode_attn", "lrsa_decode_attn_static",
           "lrsa_fill_workspace_bytes", "lrsa_attn_fwd_fill", "lrsa_attn_bwd_fill", "lrsa_attn_bwd_finish",
           "lrsa_timing_enable", "lrsa_timing_count", "lrsa_timing_read")


class LrsaParams(ctypes.Structure):
    """Mirror of lrsa_params in include/lrsa.h."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("heads_q", ctypes.c_int32), ("heads_kv", ctypes.c_int32),
        ("seq", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("sink", ctypes.c_int32), ("lag", ctypes.c_int32), ("topk", ctypes.c_int32),
        ("std_ddof", ctypes.c_int32), ("local_prev", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("dtype", ctypes.c_int32), ("impl", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3), ("kv_stride", ctypes.c_int64 * 3),
    ]


class LrsaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"liblrsa error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Load liblrsa.so (built in-tree by paper_2506_11498_amd.build); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2506_11498_amd.build` "
                                    "(or __graft_entry__.build()).  There is no fallback path.")
        L = ctypes.CDLL(LIB_PATH)
        L.lrsa_last_error.restype = ctypes.c_char_p
        L.lrsa_workspace_bytes.restype = ctypes.c_size_t
        L.lrsa_workspace_bytes.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.lrsa_num_scored_chunks.argtypes = [ctypes.c_void_p]
        L.lrsa_score_route.argtypes = [ctypes.c_void_p]
        L.lrsa_score_poll_limit.argtypes = [ctypes.c_int]
        L.lrsa_score_poll_limit.restype = ctypes.c_int
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        L.lrsa_score.argtypes = [vp, vp, vp, vp, vp, sz, vp]
        L.lrsa_select.argtypes = [vp, vp, vp, vp, sz, vp]
        L.lrsa_score_select.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp]
        L.lrsa_check_idx.argtypes = [vp, vp, vp, vp]
        L.lrsa_cache_compress.argtypes = [vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp]
        L.lrsa_decode_attn.argtypes = [vp, vp, vp, vp, ctypes.c_int32, vp, vp, vp, sz, vp]
        L.lrsa_decode_attn_static.argtypes = [vp, vp, vp, vp, ctypes.c_int32, vp, vp, vp]
        i32 = ctypes.c_int32
        L.lrsa_fill_workspace_bytes.restype = ctypes.c_size_t
        L.lrsa_fill_workspace_bytes.argtypes = [vp, i32, i32, ctypes.c_int]
        L.lrsa_attn_fwd_fill.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lrsa_attn_bwd_fill.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lrsa_attn_bwd_finish.argtypes = [vp, vp, vp, vp, vp, vp]
        L.lrsa_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lrsa_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        _lib = L
    return _lib


def _check(rc: int):
    if rc < 0:
        raise LrsaError(rc, lib().lrsa_last_error().decode())
    return rc


def make_params(q_shape, kv_shape, q_stride, kv_stride, *, sink: int, lag: int, topk: int, dtype,
                std_ddof: int = 1, local_prev: int = 1, softmax_scale: float = 0.0,
                impl: int = IMPL_AUTO) -> LrsaParams:
    """Build lrsa_params from [B,H,n,d] shapes and element strides (the last stride must be 1)."""
    B, Hq, n, d = q_shape
    if q_stride[3] != 1 or kv_stride[3] != 1:
        raise ValueError("the channel stride must be 1")
    p = LrsaParams()
    p.batch, p.heads_q, p.heads_kv, p.seq, p.head_dim = B, Hq, kv_shape[1], n, d
    p.sink, p.lag, p.topk, p.std_ddof, p.local_prev = sink, lag, topk, std_ddof, local_prev
    p.softmax_scale = softmax_scale
    p.dtype = LRSA_F32 if dtype == torch.float32 else LRSA_BF16 if dtype == torch.bfloat16 else -1
    p.impl = impl
    for i in range(3):
        p.q_stride[i] = q_stride[i]
        p.kv_stride[i] = kv_stride[i]
    return p


def params_for(Q: torch.Tensor, K: torch.Tensor, **kw) -> LrsaParams:
    return make_params(tuple(Q.shape), tuple(K.shape), Q.stride(), K.stride(), dtype=Q.dtype, **kw)


def num_scored_chunks(p: LrsaParams) -> int:
    return _check(lib().lrsa_num_scored_chunks(ctypes.byref(p)))


def score_route(p: LrsaParams) -> int:
    """Which kernels score these params: 0 none, 1 one workgroup per chunk, 2 sliced, 3 one read (rows kept in
    registers), 4 long chunks."""
    return _check(lib().lrsa_score_route(ctypes.byref(p)))


def score_poll_limit(polls: int) -> int:
    """Sets how often a one-read scoring workgroup polls for its hint words (negative: query only); returns the
    previous value.  Results do not depend on it."""
    return int(lib().lrsa_score_poll_limit(int(polls)))


def workspace_bytes(p: LrsaParams, which: int) -> int:
    return int(lib().lrsa_workspace_bytes(ctypes.byref(p), which))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


_TORCH_DTYPE = {LRSA_F32: torch.float32, LRSA_BF16: torch.bfloat16}


def _expect(name: str, t: Optional[torch.Tensor], shape, stride, dtype, device) -> None:
    """The C ABI describes Q, O, dO, dQ by ONE stride triple and K, V, dK, dV by another, and takes score, idx,
    lse as contiguous: a tensor that differs would be read or written at wrong addresses, so it is refused."""
    if t is None:
        return
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if t.device != device:
        raise ValueError(f"{name}: on {t.device}, expected {device}")
    if stride is None:
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    else:
        for dim, (have, want) in enumerate(zip(t.stride(), stride)):
            if t.shape[dim] > 1 and have != want:
                raise ValueError(f"{name}: stride {tuple(t.stride())}, the params describe {tuple(stride)}")


def _expect_q(p: LrsaParams, device, **tensors) -> None:
    shape = (p.batch, p.heads_q, p.seq, p.head_dim)
    for name, t in tensors.items():
        _expect(name, t, shape, (*p.q_stride, 1), _TORCH_DTYPE.get(p.dtype), device)


def _expect_kv(p: LrsaParams, device, **tensors) -> None:
    shape = (p.batch, p.heads_kv, p.seq, p.head_dim)
    for name, t in tensors.items():
        _expect(name, t, shape, (*p.kv_stride, 1), _TORCH_DTYPE.get(p.dtype), device)


def _workspace(p: LrsaParams, which: int, device, ws: Optional[torch.Tensor]) -> Tuple[Optional[torch.Tensor], int]:
    need = workspace_bytes(p, which)
    if need == 0:
        return None, 0
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws, ws.numel() * ws.element_size()


def lrsa_score(p: LrsaParams, K: torch.Tensor, V: torch.Tensor, score: Optional[torch.Tensor] = None,
               ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """LagKV scores [B, Hkv, Ns, L] fp32 (Eq. 4-8)."""
    Ns = num_scored_chunks(p)
    if score is None:
        score = torch.empty((p.batch, p.heads_kv, Ns, p.lag), dtype=torch.float32, device=K.device)
    _expect_kv(p, K.device, K=K, V=V)
    _expect("score", score, (p.batch, p.heads_kv, Ns, p.lag), None, torch.float32, K.device)
    ws, nb = _workspace(p, WS_SCORE, K.device, ws)
    _check(lib().lrsa_score(ctypes.byref(p), _ptr(K), _ptr(V), _ptr(score), _ptr(ws), nb, _stream()))
    return score


def lrsa_select(p: LrsaParams, score: torch.Tensor, idx: Optional[torch.Tensor] = None,
                ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Top-K positions per (batch, KV head, chunk): int32 [B, Hkv, Ns, K], ascending."""
    Ns = num_scored_chunks(p)
    if idx is None:
        idx = torch.empty((p.batch, p.heads_kv, Ns, p.topk), dtype=torch.int32, device=score.device)
    _expect("score", score, (p.batch, p.heads_kv, Ns, p.lag), None, torch.float32, score.device)
    _expect("idx", idx, (p.batch, p.heads_kv, Ns, p.topk), None, torch.int32, score.device)
    ws, nb = _workspace(p, WS_SELECT, score.device, ws)
    _check(lib().lrsa_select(ctypes.byref(p), _ptr(score), _ptr(idx), _ptr(ws), nb, _stream()))
    return idx


def lrsa_check_idx(p: LrsaParams, idx: Optional[torch.Tensor], bad_rows: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Number of rows of idx that are not K ascending positions of their chunk, as a device int32 tensor of one
    element (0 for a valid idx).  Enqueued like every call: `.item()` on the result synchronises."""
    Ns = num_scored_chunks(p)
    device = idx.device if idx is not None else torch.device("cuda", torch.cuda.current_device())
    if idx is not None:
        _expect("idx", idx, (p.batch, p.heads_kv, Ns, p.topk), None, torch.int32, device)
    if bad_rows is None:
        bad_rows = torch.empty(1, dtype=torch.int32, device=device)
    _expect("bad_rows", bad_rows, (1,), None, torch.int32, device)
    _check(lib().lrsa_check_idx(ctypes.byref(p), _ptr(idx), _ptr(bad_rows), _stream()))
    return bad_rows


def lrsa_score_select(p: LrsaParams, K: torch.Tensor, V: torch.Tensor, score: Optional[torch.Tensor] = None,
                      idx: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """lrsa_score and lrsa_select in one call (the selection is taken by the kernel that finishes the scores):
    (score, idx)."""
    Ns = num_scored_chunks(p)
    if score is None:
        score = torch.empty((p.batch, p.heads_kv, Ns, p.lag), dtype=torch.float32, device=K.device)
    if idx is None:
        idx = torch.empty((p.batch, p.heads_kv, Ns, p.topk), dtype=torch.int32, device=K.device)
    _expect_kv(p, K.device, K=K, V=V)
    _expect("score", score, (p.batch, p.heads_kv, Ns, p.lag), None, torch.float32, K.device)
    _expect("idx", idx, (p.batch, p.heads_kv, Ns, p.topk), None, torch.int32, K.device)
    ws, nb = _workspace(p, WS_SCORE, K.device, ws)
    _check(lib().lrsa_score_select(ctypes.byref(p), _ptr(K), _ptr(V), _ptr(score), _ptr(idx), _ptr(ws), nb, _stream()))
    return score, idx


def lrsa_cache_compress(p: LrsaParams, Kc: torch.Tensor, Vc: torch.Tensor, pos: Optional[torch.Tensor],
                        length: int, done: int):
    """Inference-time cache: compress (in place) while the uncompressed tail holds 2*lag rows.
    Kc, Vc: [B, Hkv, cap, d] with cap = p.seq; pos: int32 [B, Hkv, cap] or None.  Returns (length, done)."""
    new_len, new_done = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().lrsa_cache_compress(ctypes.byref(p), _ptr(Kc), _ptr(Vc), _ptr(pos), int(length), int(done),
                                     ctypes.byref(new_len), ctypes.byref(new_done), _stream()))
    return new_len.value, new_done.value


def lrsa_decode_attn(p: LrsaParams, q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, length: int,
                     O: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                     ws: Optional[torch.Tensor] = None):
    """Single-query attention over cache rows [0, length): q, O [B, Hq, d]; returns (O, lse [B, Hq] fp32)."""
    if O is None:
        O = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((p.batch, p.heads_q), dtype=torch.float32, device=q.device)
    ws, nb = _workspace(p, WS_DECODE_ATTN, q.device, ws)
    _check(lib().lrsa_decode_attn(ctypes.byref(p), _ptr(q), _ptr(Kc), _ptr(Vc), int(length), _ptr(O), _ptr(lse),
                                  _ptr(ws), nb, _stream()))
    return O, lse


def lrsa_decode_attn_static(p: LrsaParams, q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, length: int,
                            O: torch.Tensor, lse: Optional[torch.Tensor]):
    """lrsa_decode_attn without a workspace (the library's built-in scratch array); O and lse are the caller's."""
    _check(lib().lrsa_decode_attn_static(ctypes.byref(p), _ptr(q), _ptr(Kc), _ptr(Vc), int(length), _ptr(O), _ptr(lse),
                                         _stream()))
    return O, lse


def lrsa_attn_fwd(p: LrsaParams, Q, K, V, idx, O: Optional[torch.Tensor] = None,
                  lse: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """Sparse attention forward: returns (O like Q, lse [B, Hq, n] fp32)."""
    if O is None:
        O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    if lse is None:
        lse = torch.empty((p.batch, p.heads_q, p.seq), dtype=torch.float32, device=Q.device)
    _expect_q(p, Q.device, Q=Q, O=O)
    _expect_kv(p, Q.device, K=K, V=V)
    _expect("lse", lse, (p.batch, p.heads_q, p.seq), None, torch.float32, Q.device)
    if idx is not None:
        _expect("idx", idx, (p.batch, p.heads_kv, num_scored_chunks(p), p.topk), None, torch.int32, Q.device)
    ws, nb = _workspace(p, WS_ATTN_FWD, Q.device, ws)
    _check(lib().lrsa_attn_fwd(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(O), _ptr(lse),
                               _ptr(ws), nb, _stream()))
    return O, lse


def lrsa_attn_bwd(p: LrsaParams, Q, K, V, O, dO, lse, idx, dQ=None, dK=None, dV=None,
                  ws: Optional[torch.Tensor] = None):
    """Sparse attention backward: returns (dQ like Q, dK like K, dV like V)."""
    dQ = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device) if dQ is None else dQ
    dK = torch.empty_strided(K.shape, K.stride(), dtype=K.dtype, device=K.device) if dK is None else dK
    dV = torch.empty_strided(K.shape, K.stride(), dtype=K.dtype, device=K.device) if dV is None else dV
    _expect_q(p, Q.device, Q=Q, O=O, dO=dO, dQ=dQ)
    _expect_kv(p, Q.device, K=K, V=V, dK=dK, dV=dV)
    _expect("lse", lse, (p.batch, p.heads_q, p.seq), None, torch.float32, Q.device)
    if idx is not None:
        _expect("idx", idx, (p.batch, p.heads_kv, num_scored_chunks(p), p.topk), None, torch.int32, Q.device)
    ws, nb = _workspace(p, WS_ATTN_BWD, Q.device, ws)
    _check(lib().lrsa_attn_bwd(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(lse), _ptr(idx),
                               _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ws), nb, _stream()))
    return dQ, dK, dV


def fill_workspace_bytes(p: LrsaParams, row_begin: int, row_end: int, which: int) -> int:
    return int(lib().lrsa_fill_workspace_bytes(ctypes.byref(p), int(row_begin), int(row_end), which))


def _fill_ws(p, row_begin, row_end, which, device, ws):
    need = fill_workspace_bytes(p, row_begin, row_end, which)
    if ws is None:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return ws, ws.numel() * ws.element_size()


def lrsa_attn_fwd_fill(p: LrsaParams, row_begin: int, row_end: int, Q, K, V, idx, O=None, lse=None, ws=None):
    """One filling step of the forward: Q, O hold the rows [row_begin, row_end) only; returns (O, lse)."""
    rows = row_end - row_begin
    if O is None:
        O = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
    if lse is None:
        lse = torch.empty((p.batch, p.heads_q, rows), dtype=torch.float32, device=Q.device)
    shape = (p.batch, p.heads_q, rows, p.head_dim)
    for name, t in (("Q", Q), ("O", O)):
        _expect(name, t, shape, (*p.q_stride, 1), _TORCH_DTYPE.get(p.dtype), Q.device)
    _expect_kv(p, Q.device, K=K, V=V)
    _expect("lse", lse, (p.batch, p.heads_q, rows), None, torch.float32, Q.device)
    ws, nb = _fill_ws(p, row_begin, row_end, WS_ATTN_FWD, Q.device, ws)
    _check(lib().lrsa_attn_fwd_fill(ctypes.byref(p), int(row_begin), int(row_end), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx),
                                    _ptr(O), _ptr(lse), _ptr(ws), nb, _stream()))
    return O, lse


def lrsa_attn_bwd_fill(p: LrsaParams, row_begin: int, row_end: int, Q, K, V, O, dO, lse, idx, dK_acc, dV_acc,
                       dQ=None, ws=None):
    """One filling step of the backward: dQ of the rows, and their share ADDED to the fp32 sums dK_acc, dV_acc."""
    rows = row_end - row_begin
    dQ = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device) if dQ is None else dQ
    shape = (p.batch, p.heads_q, rows, p.head_dim)
    for name, t in (("Q", Q), ("O", O), ("dO", dO), ("dQ", dQ)):
        _expect(name, t, shape, (*p.q_stride, 1), _TORCH_DTYPE.get(p.dtype), Q.device)
    _expect_kv(p, Q.device, K=K, V=V)
    for name, t in (("dK_acc", dK_acc), ("dV_acc", dV_acc)):
        _expect(name, t, (p.batch, p.heads_kv, p.seq, p.head_dim), None, torch.float32, Q.device)
    _expect("lse", lse, (p.batch, p.heads_q, rows), None, torch.float32, Q.device)
    ws, nb = _fill_ws(p, row_begin, row_end, WS_ATTN_BWD, Q.device, ws)
    _check(lib().lrsa_attn_bwd_fill(ctypes.byref(p), int(row_begin), int(row_end), _ptr(Q), _ptr(K), _ptr(V), _ptr(O),
                                    _ptr(dO), _ptr(lse), _ptr(idx), _ptr(dQ), _ptr(dK_acc), _ptr(dV_acc), _ptr(ws), nb,
                                    _stream()))
    return dQ


def lrsa_attn_bwd_finish(p: LrsaParams, dK_acc, dV_acc, dK, dV):
    """fp32 sums of the filling steps -> dK, dV."""
    _expect_kv(p, dK_acc.device, dK=dK, dV=dV)
    _check(lib().lrsa_attn_bwd_finish(ctypes.byref(p), _ptr(dK_acc), _ptr(dV_acc), _ptr(dK), _ptr(dV), _stream()))
    return dK, dV


def timing_enable(on: bool) -> None:
    """Switch per-kernel HIP-event timing on (clearing earlier records) or off."""
    _check(lib().lrsa_timing_enable(1 if on else 0))


def timing_records():
    """[(kernel name, milliseconds)] of every launch recorded since timing was switched on (waits for them)."""
    L = lib()
    out = []
    name, ms = ctypes.c_char_p(), ctypes.c_float()
    for i in range(L.lrsa_timing_count()):
        _check(L.lrsa_timing_read(i, ctypes.byref(name), ctypes.byref(ms)))
        out.append((name.value.decode(), ms.value))
    return out
