"""CPU oracle for Lag-Relative Sparse Attention (LRSA) -- TEST INFRASTRUCTURE ONLY.

Plain, slow NumPy written from the paper's definitions.  It shares no code with
the HIP path and must never be imported by the product package; only tests,
the smoke check and the benchmark's cpu_baseline leg use it.

What follows the paper directly
  * partition into sink + lag-size chunks            (Method, text after Eq. 8)
  * LagKV score, Eq. 4-8                              (min/max of the FOLLOWING chunk,
                                                       min-max normalise, Std over channels,
                                                       Softmax over the chunk's tokens, K+V sum)
  * top r*L selection per head per lag window         (text after Eq. 8)
  * the chunked mask                                  (Attention Filling 1 / 2 / repeat)
  * attention = softmax(Q K^T / sqrt(d_h) + M) V      (Eq. 2-3), M = -inf where masked
Backward is the standard calculus of Eq. 3 with the mask held constant.

Readings where the paper is silent (all "parity unpinned" by the paper itself,
pinned only by closed forms in the tests): Std uses ddof=1 by default; a channel
whose max equals its min is divided by 1; the tail chunk and the last full chunk
are never scored; ties go to the lowest position.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- partition
def partition(n: int, S: int, L: int, local_prev: int = 1) -> dict:
    """Sink [0,S), chunks C_p = [S+pL, S+(p+1)L), tail of length R (text after Eq. 8).

    nq  = number of query chunks (the tail counts as one),
    Ns  = number of chunks that are ever seen in compressed form and hence scored:
          chunk p is compressed for query chunks q >= p + local_prev + 1, so p <= nq-2-local_prev.
    """
    rest = max(n - S, 0)
    P = rest // L
    R = rest - P * L
    nq = P + (1 if R > 0 else 0)
    Ns = max(nq - 1 - local_prev, 0)
    return {"P": P, "R": R, "nq": nq, "Ns": Ns}


def chunk_of(u, S: int, L: int):
    """Chunk index of position u >= S."""
    return (np.asarray(u) - S) // L


# --------------------------------------------------------------------------- Eq. 4-8
def score_one(Z: np.ndarray, S: int, L: int, Ns: int, ddof: int, dtype) -> np.ndarray:
    """score(Z_i) of Eq. 7 for one head: Z is [n, d]; returns [Ns, L] in `dtype` arithmetic."""
    Z = np.asarray(Z, dtype=dtype)
    d = Z.shape[1]
    out = np.empty((Ns, L), dtype=dtype)
    for p in range(Ns):
        cur = Z[S + p * L: S + (p + 1) * L]
        nxt = Z[S + (p + 1) * L: S + (p + 2) * L]
        mn = nxt.min(axis=0)                      # Eq. 4, over the sequence axis of chunk p+1
        mx = nxt.max(axis=0)                      # Eq. 5
        den = mx - mn
        den = np.where(den == 0, dtype(1), den)
        zn = (cur - mn) / den                     # Eq. 6
        mean = zn.sum(axis=1, dtype=dtype) / dtype(d)
        dev = zn - mean[:, None]
        sigma = np.sqrt((dev * dev).sum(axis=1, dtype=dtype) / dtype(d - ddof))   # Std. over channels
        e = np.exp(sigma - sigma.max())
        out[p] = e / e.sum(dtype=dtype)           # Softmax over the L tokens of chunk p (Eq. 7)
    return out


def score(K: np.ndarray, V: np.ndarray, S: int, L: int, ddof: int = 1, dtype=np.float32,
          local_prev: int = 1) -> np.ndarray:
    """score_i = score(K_i) + score(V_i), Eq. 8.  K, V: [B, Hkv, n, d] -> [B, Hkv, Ns, L]."""
    B, H, n, _ = K.shape
    Ns = partition(n, S, L, local_prev)["Ns"]
    out = np.empty((B, H, Ns, L), dtype=dtype)
    for b in range(B):
        for h in range(H):
            out[b, h] = score_one(K[b, h], S, L, Ns, ddof, dtype) + score_one(V[b, h], S, L, Ns, ddof, dtype)
    return out


# --------------------------------------------------------------------------- top r*L
def select(sc: np.ndarray, S: int, L: int, K: int) -> np.ndarray:
    """The K highest-scoring positions of each chunk (text after Eq. 8), ties to the lowest
    position, returned ascending as absolute positions.  sc: [..., Ns, L] -> int32 [..., Ns, K]."""
    Ns = sc.shape[-2]
    order = np.argsort(-sc, axis=-1, kind="stable")[..., :K]     # stable: equal scores keep position order
    local = np.sort(order, axis=-1)
    base = (S + np.arange(Ns) * L).reshape((1,) * (sc.ndim - 2) + (Ns, 1))
    return (local + base).astype(np.int32)


# --------------------------------------------------------------------------- the mask
def visible_mask(n: int, S: int, L: int, idx_h: np.ndarray, local_prev: int = 1) -> np.ndarray:
    """Boolean [n, n]: query t may attend key u.

    causal, and one of: u in the sink; t in the sink; u in the query's own chunk or one of the
    `local_prev` chunks before it (kept in full as the sliding window); u survived the
    compression of its chunk (Attention Filling steps).
    """
    t = np.arange(n)[:, None]
    u = np.arange(n)[None, :]
    selected = np.zeros(n, dtype=bool)
    if idx_h is not None and idx_h.size:
        selected[np.asarray(idx_h).reshape(-1)] = True
    ct = (t - S) // L
    cu = (u - S) // L
    keep = (u < S) | (t < S) | (cu >= ct - local_prev) | selected[None, :]
    return (u <= t) & keep


def visible_mask_by_replay(n: int, S: int, L: int, idx_h: np.ndarray, m: int) -> np.ndarray:
    """The same mask derived a second way: replay the chunk-by-chunk prefill with m chunks per
    Attention Filling step, tracking the cache as a list of positions.

    Each step appends the next m chunks to the cache and attends causally over it; a query in
    the j-th new chunk additionally loses, from the chunks it is more than one chunk ahead of,
    every position that the compression of those chunks (which only needs the chunk after
    them, already present) drops.  After the step the cache keeps sink + survivors + the last
    chunk in full.
    """
    part = partition(n, S, L)
    nq = part["nq"]
    bounds = [(S + p * L, min(S + (p + 1) * L, n)) for p in range(nq)]
    vis = np.zeros((n, n), dtype=bool)
    for t in range(min(S, n)):
        vis[t, : t + 1] = True
    kept = {}                                   # chunk -> survivors once compressed
    cache = list(range(min(S, n)))              # positions currently held
    done = 0
    while done < nq:
        new = list(range(done, min(done + m, nq)))
        for p in new:
            cache += list(range(*bounds[p]))
        for q in new:
            # compression that has become possible before chunk q is attended: chunks <= q-2
            dropped = set()
            for p in range(0, q - 1):
                if p not in kept:
                    kept[p] = set(int(x) for x in idx_h[p])
                dropped |= set(range(*bounds[p])) - kept[p]
            for t in range(*bounds[q]):
                for u in cache:
                    if u <= t and u not in dropped:
                        vis[t, u] = True
        last = new[-1]
        done = last + 1
        if done >= nq:
            break                               # nothing attends after the final step
        cache = list(range(min(S, n)))
        for p in range(0, last):
            if p not in kept:
                kept[p] = set(int(x) for x in idx_h[p])
            cache += sorted(kept[p])
        cache += list(range(*bounds[last]))
    return vis


# --------------------------------------------------------------------------- Eq. 2-3
def attn_fwd_dense(Q, K, V, idx, S: int, L: int, scale=None, local_prev: int = 1):
    """O = softmax(Q K^T * scale + M) V and the row log-sum-exp, in fp64, under the explicit mask.

    Q: [B, Hq, n, d]; K, V: [B, Hkv, n, d]; idx: [B, Hkv, Ns, K] or None.  Query head hq uses
    KV head hq // (Hq/Hkv).  Returns O [B,Hq,n,d], lse [B,Hq,n].
    """
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    B, Hq, n, d = Q.shape
    G = Hq // K.shape[1]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    O = np.empty_like(Q)
    lse = np.empty((B, Hq, n))
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            vis = visible_mask(n, S, L, None if idx is None else idx[b, h], local_prev)
            logits = np.where(vis, (Q[b, hq] @ K[b, h].T) * scale, -np.inf)
            mx = logits.max(axis=1, keepdims=True)
            e = np.exp(logits - mx)
            den = e.sum(axis=1, keepdims=True)
            O[b, hq] = (e / den) @ V[b, h]
            lse[b, hq] = (mx + np.log(den))[:, 0]
    return O, lse


def attn_bwd_dense(Q, K, V, dO, idx, S: int, L: int, scale=None, local_prev: int = 1):
    """Gradients of sum(O * dO) w.r.t. Q, K, V with the mask constant, fp64, matrix form:
    A = softmax(.), dV = A^T dO, dA = dO V^T, dS = A * (dA - rowsum(dO*O)), dQ = scale dS K,
    dK = scale dS^T Q; dK, dV summed over the query heads that share a KV head."""
    Q = np.asarray(Q, np.float64); K = np.asarray(K, np.float64); V = np.asarray(V, np.float64)
    dO = np.asarray(dO, np.float64)
    B, Hq, n, d = Q.shape
    G = Hq // K.shape[1]
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    dQ = np.zeros_like(Q); dK = np.zeros_like(K); dV = np.zeros_like(V)
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            vis = visible_mask(n, S, L, None if idx is None else idx[b, h], local_prev)
            logits = np.where(vis, (Q[b, hq] @ K[b, h].T) * scale, -np.inf)
            e = np.exp(logits - logits.max(axis=1, keepdims=True))
            A = e / e.sum(axis=1, keepdims=True)
            O = A @ V[b, h]
            dA = dO[b, hq] @ V[b, h].T
            D = (dO[b, hq] * O).sum(axis=1, keepdims=True)
            dS = A * (dA - D)
            dV[b, h] += A.T @ dO[b, hq]
            dQ[b, hq] = scale * (dS @ K[b, h])
            dK[b, h] += scale * (dS.T @ Q[b, hq])
    return dQ, dK, dV


def loss(Q, K, V, dO, idx, S, L, scale=None, local_prev: int = 1) -> float:
    """sum(O * dO): the scalar whose gradient attn_bwd_dense returns (idx frozen)."""
    O, _ = attn_fwd_dense(Q, K, V, idx, S, L, scale, local_prev)
    return float((O * np.asarray(dO, np.float64)).sum())


def visible_count(t: int, n: int, S: int, L: int, K: int, local_prev: int = 1) -> int:
    """Closed-form number of keys row t sees: sink + K per compressed chunk + the full local
    chunks + its own chunk up to the diagonal."""
    if t < S:
        return t + 1
    q = (t - S) // L
    return S + K * max(q - local_prev, 0) + L * min(q, local_prev) + (t - (S + q * L) + 1)
