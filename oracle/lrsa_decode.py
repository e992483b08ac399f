"""CPU oracle for the inference-time use of LagKV compression -- TEST INFRASTRUCTURE ONLY.

The paper evaluates its models with the KV cache compressed by LagKV (evaluation tables, compression
1x / 2x / 4x): the cache keeps the sink, and, lag window by lag window, only the top r*L tokens of a chunk
once the chunk after it is complete (Section 3.2, Attention Filling 1: the older chunk is cut down to its
survivors, the newer one stays whole as the local window; the survivors are the top r*L tokens by score,
text after Eq. 8).  This file writes that procedure out token by token for one KV head, and the
single-query attention over such a cache (Eq. 3 with nothing masked).

It shares no code with the HIP path; it calls the training-time oracle's scoring formula
(lrsa_ref.score_one, Eq. 4-7) on the two oldest uncompressed chunks of the cache.
"""
from __future__ import annotations

import numpy as np

from . import lrsa_ref as ref


def compress_once(Kc: np.ndarray, Vc: np.ndarray, pos: np.ndarray, done: int, S: int, L: int, topk: int,
                  ddof: int = 1, dtype=np.float32):
    """One compression step on a cache whose uncompressed tail holds at least 2L rows: score the first L
    rows of the tail against the next L (Eq. 4-8), keep their top-K in position order, close the gap.
    Kc, Vc: [len, d]; pos: [len] original positions; done: chunks compressed so far."""
    base = S + topk * done
    assert len(pos) - base >= 2 * L
    two = slice(base, base + 2 * L)
    # score_one scores chunk 0 of a sequence "no sink, two chunks" against chunk 1
    sc = (ref.score_one(Kc[two], 0, L, 1, ddof, dtype) + ref.score_one(Vc[two], 0, L, 1, ddof, dtype))[0]
    order = np.argsort(-sc, kind="stable")[:topk]          # ties to the lowest position
    keep = base + np.sort(order)
    rows = np.concatenate([np.arange(base), keep, np.arange(base + L, len(pos))])
    return Kc[rows], Vc[rows], pos[rows], done + 1


def cache_incremental(K: np.ndarray, V: np.ndarray, S: int, L: int, topk: int, ddof: int = 1,
                      dtype=np.float32):
    """The cache of one KV head as the query of its LAST token sees it, after the n rows have been appended
    one token at a time.  A token is appended, attends, and only when the next token arrives is the cache
    compressed if its uncompressed tail has reached 2L rows (the chunk after the one to compress is then
    complete).  K, V: [n, d].  Returns (Kc, Vc, pos, done)."""
    n, d = K.shape
    Kc, Vc = np.empty((0, d), K.dtype), np.empty((0, d), V.dtype)
    pos, done = np.empty((0,), np.int64), 0
    for t in range(n):
        if len(pos) - (S + topk * done) >= 2 * L:
            Kc, Vc, pos, done = compress_once(Kc, Vc, pos, done, S, L, topk, ddof, dtype)
        Kc, Vc = np.concatenate([Kc, K[t:t + 1]]), np.concatenate([Vc, V[t:t + 1]])
        pos = np.append(pos, t)
    return Kc, Vc, pos, done


def decode_attn(q: np.ndarray, Kc: np.ndarray, Vc: np.ndarray, scale=None):
    """softmax(q Kc^T * scale) Vc for single queries (Eq. 3, nothing masked), fp64.
    q: [G, d] (the query heads of one KV group), Kc, Vc: [len, d].  Returns (O [G, d], lse [G])."""
    q, Kc, Vc = (np.asarray(a, np.float64) for a in (q, Kc, Vc))
    scale = 1.0 / np.sqrt(q.shape[-1]) if scale is None else scale
    s = q @ Kc.T * scale
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=-1, keepdims=True)
    return (e / z) @ Vc, (m + np.log(z))[:, 0]
