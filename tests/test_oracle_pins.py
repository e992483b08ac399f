"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it pins.  A plausible mistake in the oracle (wrong reference
chunk, wrong axis, dropped term, transposed operand, off-by-one in the mask) fails at least
one of them.
"""
import itertools
import os

import numpy as np
import pytest
import torch

from oracle import lrsa_ref as ref
from oracle import lrsa_rows as rows
from paper_2506_11498_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _np(t):
    return t.to(torch.float32).numpy()


def _micro(**kw):
    w = inputs.small_workload(**kw)
    x = inputs.make_inputs(w)
    return w, {k: _np(v).astype(np.float64) for k, v in x.items()}


def _idx(w, x, dtype=np.float32):
    sc = ref.score(x["K"], x["V"], w.S, w.L, dtype=dtype)
    return sc, ref.select(sc, w.S, w.L, w.K)


def _dense_causal_torch(x):
    """Library routine: torch's fp64 scaled_dot_product_attention with is_causal, plus autograd."""
    Q = torch.tensor(x["Q"], dtype=torch.float64, requires_grad=True)
    K = torch.tensor(x["K"], dtype=torch.float64, requires_grad=True)
    V = torch.tensor(x["V"], dtype=torch.float64, requires_grad=True)
    G = Q.shape[1] // K.shape[1]
    Kr, Vr = K.repeat_interleave(G, dim=1), V.repeat_interleave(G, dim=1)
    O = torch.nn.functional.scaled_dot_product_attention(Q, Kr, Vr, is_causal=True)
    (O * torch.tensor(x["dO"], dtype=torch.float64)).sum().backward()
    return O.detach().numpy(), Q.grad.numpy(), K.grad.numpy(), V.grad.numpy()


# ---------------------------------------------------------------- partition (text after Eq. 8)
def test_partition_of_the_five_workloads():
    expect = {"C1": (7, 124, 8, 6), "C2": (15, 240, 16, 14), "C3": (31, 496, 32, 30),
              "C4": (31, 960, 32, 30), "C5": (63, 1984, 64, 62)}
    for name, (P, R, nq, Ns) in expect.items():
        w = inputs.WORKLOADS[name]
        assert ref.partition(w.n, w.S, w.L) == {"P": P, "R": R, "nq": nq, "Ns": Ns}
    assert ref.partition(10, 3, 4)["Ns"] == 0          # sink + 1 chunk + tail: nothing compressed
    assert ref.partition(3 + 3 * 4, 3, 4) == {"P": 3, "R": 0, "nq": 3, "Ns": 1}


# ---------------------------------------------------------------- Eq. 4-7 by hand
def test_score_closed_form_from_golden_file():
    """Eq. 4-7 evaluated by hand on a 2-token chunk (tests/golden/score_hand_example.txt)."""
    vals = {}
    for line in open(os.path.join(GOLDEN, "score_hand_example.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = np.array([float(t) for t in v.split()])
    mn, mx = vals["ref_min"], vals["ref_max"]
    d = len(mn)
    pat = vals["pattern"]
    row_a = mn + pat * (mx - mn)          # normalises to the 0/1 pattern
    row_b = mn.copy()                     # normalises to all zeros -> sigma 0
    ref_rows = np.stack([mn + pat * (mx - mn), mn + (1 - pat) * (mx - mn)])   # per-channel min=mn, max=mx
    filler = np.stack([mx * 3 + 1, mn * 5 - 2])                               # chunk 2: never used by chunk 0
    Z = np.concatenate([np.stack([row_a, row_b]), ref_rows, filler])[None, None]
    for ddof in (0, 1):
        sig_a = 0.5 * np.sqrt(d / (d - ddof))
        assert np.isclose(sig_a, vals[f"sigma_a_ddof{ddof}"][0], rtol=1e-12)
        expect = np.exp([sig_a, 0.0]) / np.exp([sig_a, 0.0]).sum()
        assert np.allclose(expect, vals[f"score_ddof{ddof}"], rtol=1e-9)
        got = ref.score_one(Z[0, 0], 0, 2, 1, ddof, np.float64)
        assert got.shape == (1, 2)
        assert np.allclose(got[0], expect, rtol=1e-12)
        got32 = ref.score_one(Z[0, 0], 0, 2, 1, ddof, np.float32)
        assert np.allclose(got32[0], expect, rtol=1e-6)
    # Eq. 8: K and V scores add
    sc = ref.score(Z, Z, 0, 2, ddof=1, dtype=np.float64)
    assert np.allclose(sc[0, 0, 0], 2 * np.array(vals["score_ddof1"]), rtol=1e-9)


def _read_golden(name):
    vals = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = np.array([float(t) for t in v.split()])
    return vals


def test_score_adds_the_v_term_hand_example_with_k_different_from_v():
    """Eq. 8 with K != V evaluated by hand (tests/golden/score_kv_hand_example.txt): the V term has its own
    normalisation, Std and softmax; dropping it, or using K twice, gives other numbers."""
    vals = _read_golden("score_kv_hand_example.txt")
    mn, mx = vals["ref_min"], vals["ref_max"]

    def tensor(pat_a, pat_b):
        pat = vals["k_pattern_a"]
        ref_rows = np.stack([mn + pat * (mx - mn), mn + (1 - pat) * (mx - mn)])   # per-channel min = mn, max = mx
        filler = np.stack([mx * 3 + 1, mn * 5 - 2])                               # chunk 2: never used by chunk 0
        return np.concatenate([np.stack([mn + pat_a * (mx - mn), mn + pat_b * (mx - mn)]), ref_rows, filler])[None, None]

    Kt = tensor(vals["k_pattern_a"], vals["k_pattern_b"])
    Vt = tensor(vals["v_pattern_a"], vals["v_pattern_b"])
    assert np.allclose(vals["score_K"] + vals["score_V"], vals["score"], rtol=1e-12)
    for dtype, rtol in ((np.float64, 1e-12), (np.float32, 1e-6)):
        sc = ref.score(Kt, Vt, 0, 2, ddof=1, dtype=dtype)
        assert sc.shape == (1, 1, 1, 2)
        assert np.allclose(sc[0, 0, 0], vals["score"], rtol=rtol)
        assert np.allclose(ref.score_one(Vt[0, 0], 0, 2, 1, 1, dtype)[0], vals["score_V"], rtol=rtol)
    assert not np.allclose(ref.score(Kt, Kt, 0, 2, ddof=1, dtype=np.float64)[0, 0, 0], vals["score"], rtol=1e-3)


def test_score_uses_following_chunk_not_own_chunk():
    """Eq. 4-5: min/max come from chunk p+1.  Scaling only chunk p+1 changes chunk p's score;
    changing chunk p+2 or chunk p-1 does not."""
    w, x = _micro(n=3 + 5 * 8, L=8, S=3, K=2, d=16)
    Z = x["K"][0, 0]
    base = ref.score_one(Z, w.S, w.L, 3, 1, np.float64)
    Z2 = Z.copy(); Z2[w.S + 2 * w.L: w.S + 3 * w.L, 0] *= 3.0        # chunk 2 is the reference of chunk 1
    s2 = ref.score_one(Z2, w.S, w.L, 3, 1, np.float64)
    assert np.allclose(s2[0], base[0]) and not np.allclose(s2[1], base[1])
    Z3 = Z.copy(); Z3[: w.S] += 100.0                                  # sink never enters
    assert np.array_equal(ref.score_one(Z3, w.S, w.L, 3, 1, np.float64), base)


def test_score_sums_to_two_and_is_positive():
    """Eq. 7-8: a softmax over the chunk's tokens for K plus one for V."""
    for name in ("C1",):
        w = inputs.WORKLOADS[name]
        x = inputs.make_inputs(w)
        for dt, tol in ((np.float32, 2e-6), (np.float64, 1e-12)):
            sc = ref.score(_np(x["K"]), _np(x["V"]), w.S, w.L, dtype=dt)
            assert sc.shape == (w.B, w.Hkv, 6, w.L)
            assert np.all(sc > 0) and np.all(sc < 2)
            assert np.allclose(sc.sum(-1, dtype=np.float64), 2.0, atol=tol)


def test_score_affine_invariance_per_channel():
    """Eq. 6: min-max normalisation removes any per-channel affine map a_c z + b_c with a_c > 0."""
    w, x = _micro(n=2 + 4 * 12, L=12, S=2, K=3, d=32)
    Z = x["K"][0, 0]
    rng = np.random.default_rng(0)
    a = rng.uniform(0.5, 4.0, size=Z.shape[1])
    b = rng.normal(size=Z.shape[1])
    s0 = ref.score_one(Z, w.S, w.L, 2, 1, np.float64)
    s1 = ref.score_one(Z * a + b, w.S, w.L, 2, 1, np.float64)
    assert np.allclose(s0, s1, rtol=1e-9)
    # power-of-two scales are exact in fp32: bit-identical scores
    a2 = 2.0 ** rng.integers(-3, 4, size=Z.shape[1])
    f0 = ref.score_one(Z.astype(np.float32), w.S, w.L, 2, 1, np.float32)
    f1 = ref.score_one((Z.astype(np.float32) * a2.astype(np.float32)), w.S, w.L, 2, 1, np.float32)
    assert np.array_equal(f0, f1)


def test_outlier_channels_do_not_change_selection():
    """Consequence of Eq. 6 for the 'outlier_channels' workload: x8 on whole channels of K
    leaves idx bit-identical to the unstructured draw."""
    w = inputs.WORKLOADS["C2"].with_(B=1, Hkv=2, Hq=2, n=16 + 6 * 256)
    a = inputs.make_inputs(w, structured=True)
    b = inputs.make_inputs(w, structured=False)
    assert not torch.equal(a["K"], b["K"])
    ia = ref.select(ref.score(_np(a["K"]), _np(a["V"]), w.S, w.L), w.S, w.L, w.K)
    ib = ref.select(ref.score(_np(b["K"]), _np(b["V"]), w.S, w.L), w.S, w.L, w.K)
    assert np.array_equal(ia, ib)


def test_zero_range_channel_divides_by_one():
    """Reading: max == min in the reference chunk -> denominator 1 (no NaN/inf)."""
    w, x = _micro(n=4 * 8, L=8, S=0, K=2, d=8)
    Z = x["K"][0, 0].copy()
    Z[8:16, 3] = 1.25                       # channel 3 constant over the reference chunk of chunk 0
    s = ref.score_one(Z, 0, 8, 2, 1, np.float64)
    assert np.all(np.isfinite(s))
    zn = (Z[0:8] - Z[8:16].min(0))
    zn[:, [c for c in range(8) if c != 3]] /= (Z[8:16].max(0) - Z[8:16].min(0))[[c for c in range(8) if c != 3]]
    sig = zn.std(axis=1, ddof=1)
    assert np.allclose(s[0], np.exp(sig) / np.exp(sig).sum())


def test_std_is_over_channels_softmax_over_tokens():
    """Eq. 7 axes, against numpy's own std / a hand softmax on a random chunk."""
    w, x = _micro(n=1 + 3 * 10, L=10, S=1, K=2, d=24)
    Z = x["V"][0, 0]
    nxt = Z[11:21]
    zn = (Z[1:11] - nxt.min(0)) / (nxt.max(0) - nxt.min(0))
    for ddof in (0, 1):
        sig = zn.std(axis=1, ddof=ddof)
        expect = np.exp(sig) / np.exp(sig).sum()
        assert np.allclose(ref.score_one(Z, 1, 10, 1, ddof, np.float64)[0], expect, rtol=1e-12)


# ---------------------------------------------------------------- selection (text after Eq. 8)
def test_uniform_chunk_selects_first_positions():
    """All rows of a chunk equal -> all scores 2/L -> ties go to the lowest positions."""
    L, S, K, d = 8, 2, 3, 8
    n = S + 4 * L
    rng = np.random.default_rng(1)
    Kt = rng.normal(size=(1, 1, n, d)); Vt = rng.normal(size=(1, 1, n, d))
    Kt[0, 0, S:S + L] = Kt[0, 0, S]; Vt[0, 0, S:S + L] = Vt[0, 0, S]
    sc = ref.score(Kt, Vt, S, L, dtype=np.float64)
    assert np.allclose(sc[0, 0, 0], 2.0 / L)
    idx = ref.select(sc, S, L, K)
    assert list(idx[0, 0, 0]) == [S, S + 1, S + 2]


def test_select_matches_brute_force_enumeration():
    """Top-K = the subset maximising the score sum, lexicographically smallest among maximisers."""
    rng = np.random.default_rng(2)
    for L, K in ((6, 2), (9, 4), (10, 5), (7, 7), (8, 1)):
        sc = rng.choice([0.1, 0.2, 0.3, 0.4], size=(3, L)).astype(np.float32)   # many ties
        S = 5
        idx = ref.select(sc, S, L, K)
        for p in range(3):
            best = None
            for comb in itertools.combinations(range(L), K):
                key = (-float(np.sum(sc[p, list(comb)], dtype=np.float64)), comb)
                best = key if best is None or key < best else best
            assert tuple(idx[p] - (S + p * L)) == best[1]


def test_select_output_contract():
    w = inputs.WORKLOADS["C1"]
    x = inputs.make_inputs(w)
    sc = ref.score(_np(x["K"]), _np(x["V"]), w.S, w.L)
    idx = ref.select(sc, w.S, w.L, w.K)
    assert idx.dtype == np.int32 and idx.shape == (1, 1, 6, w.K)
    for p in range(6):
        r = idx[0, 0, p]
        assert np.all(np.diff(r) > 0) and r[0] >= w.S + p * w.L and r[-1] < w.S + (p + 1) * w.L
        thr = np.sort(sc[0, 0, p])[-w.K]
        assert np.all(sc[0, 0, p][r - (w.S + p * w.L)] >= thr)


# ---------------------------------------------------------------- the mask (Attention Filling steps)
@pytest.mark.parametrize("m", [1, 2, 3])
def test_mask_equals_procedural_replay(m):
    w, x = _micro(n=3 + 5 * 6 + 4, L=6, S=3, K=2, d=8, Hq=1)
    _, idx = _idx(w, x)
    a = ref.visible_mask(w.n, w.S, w.L, idx[0, 0])
    b = ref.visible_mask_by_replay(w.n, w.S, w.L, idx[0, 0], m)
    assert np.array_equal(a, b)


def test_attention_filling_narrative_on_four_chunks():
    """Chunk 3's queries (the paper's 'third chunk') see chunk 0 compressed and chunk 1 in full;
    chunk 4's see chunk 1 compressed: checked position by position."""
    S, L, K = 2, 4, 1
    n = S + 4 * L
    idx = np.array([[S + 1], [S + L + 2]])          # survivors of chunks 0 and 1
    vis = ref.visible_mask(n, S, L, idx)
    t = S + 2 * L + 1                                 # in chunk 2
    assert sorted(np.nonzero(vis[t])[0]) == [0, 1, S + 1] + list(range(S + L, t + 1))
    t = S + 3 * L                                     # first row of chunk 3
    assert sorted(np.nonzero(vis[t])[0]) == [0, 1, S + 1, S + L + 2] + list(range(S + 2 * L, t + 1))
    t = S + L - 1                                     # chunk 0: plain causal
    assert sorted(np.nonzero(vis[t])[0]) == list(range(t + 1))


def test_visible_count_closed_form():
    w, x = _micro(n=5 + 6 * 7 + 3, L=7, S=5, K=3, d=8, Hq=1)
    _, idx = _idx(w, x)
    vis = ref.visible_mask(w.n, w.S, w.L, idx[0, 0])
    for t in range(w.n):
        c = ref.visible_count(t, w.n, w.S, w.L, w.K)
        assert vis[t].sum() == c
        assert rows.count_visible(w.n, w.d, w.S, w.L, w.K, idx[0, 0], t) == c
    # the pair counts quoted for the five workloads (used for the flop count)
    for name, pairs in (("C1", 2.69e5), ("C2", 3.27e6), ("C4", 1.73e8)):
        w = inputs.WORKLOADS[name]
        tot = sum(ref.visible_count(t, w.n, w.S, w.L, w.K) for t in range(w.n))
        assert abs(tot - pairs) / pairs < 5e-3


def test_token_level_causality():
    """Changing anything after position t leaves rows <= t bit-identical (selection included)."""
    w, x = _micro(n=2 + 5 * 8 + 3, L=8, S=2, K=3, d=16)
    _, idx = _idx(w, x)
    O, lse = ref.attn_fwd_dense(x["Q"], x["K"], x["V"], idx, w.S, w.L)
    for t in (w.S + 2 * w.L - 1, w.S + 3 * w.L + 2):
        y = {k: v.copy() for k, v in x.items()}
        rng = np.random.default_rng(t)
        for k in ("Q", "K", "V"):
            y[k][:, :, t + 1:] = rng.normal(size=y[k][:, :, t + 1:].shape)
        _, idx2 = _idx(w, y)
        O2, lse2 = ref.attn_fwd_dense(y["Q"], y["K"], y["V"], idx2, w.S, w.L)
        assert np.array_equal(O[:, :, : t + 1], O2[:, :, : t + 1])
        assert np.array_equal(lse[:, :, : t + 1], lse2[:, :, : t + 1])


# ---------------------------------------------------------------- attention = dense routine in the special cases
def test_full_retention_equals_dense_causal():
    """r = 1 (K = L): nothing is dropped, LRSA is causal attention (torch fp64 SDPA + autograd)."""
    w, x = _micro(n=3 + 4 * 8 + 5, L=8, S=3, K=8, d=16, Hq=4, Hkv=2, B=2)
    _, idx = _idx(w, x)
    O, lse = ref.attn_fwd_dense(x["Q"], x["K"], x["V"], idx, w.S, w.L)
    dQ, dK, dV = ref.attn_bwd_dense(x["Q"], x["K"], x["V"], x["dO"], idx, w.S, w.L)
    tO, tdQ, tdK, tdV = _dense_causal_torch(x)
    for a, b in ((O, tO), (dQ, tdQ), (dK, tdK), (dV, tdV)):
        assert np.allclose(a, b, rtol=1e-10, atol=1e-12)
    # lse against its definition on one row
    t = w.n - 1
    s = (x["Q"][1, 3, t] @ x["K"][1, 1, : t + 1].T) / np.sqrt(w.d)
    assert np.isclose(lse[1, 3, t], np.log(np.exp(s).sum()))


def test_short_sequence_is_dense_causal_for_any_K():
    """Attention Filling 1: sink + two chunks is a full lower-triangular mask."""
    w, x = _micro(n=3 + 2 * 8, L=8, S=3, K=2, d=16, Hq=2, Hkv=1)
    assert ref.partition(w.n, w.S, w.L)["Ns"] == 0
    O, _ = ref.attn_fwd_dense(x["Q"], x["K"], x["V"], None, w.S, w.L)
    dQ, dK, dV = ref.attn_bwd_dense(x["Q"], x["K"], x["V"], x["dO"], None, w.S, w.L)
    tO, tdQ, tdK, tdV = _dense_causal_torch(x)
    for a, b in ((O, tO), (dQ, tdQ), (dK, tdK), (dV, tdV)):
        assert np.allclose(a, b, rtol=1e-10, atol=1e-12)


def test_sparse_case_differs_from_dense_and_matches_masked_torch():
    """K < L: equals torch SDPA under the explicit boolean mask, and is not causal attention."""
    w, x = _micro(n=3 + 5 * 8 + 2, L=8, S=3, K=2, d=16, Hq=2, Hkv=1)
    _, idx = _idx(w, x)
    O, _ = ref.attn_fwd_dense(x["Q"], x["K"], x["V"], idx, w.S, w.L)
    vis = torch.tensor(ref.visible_mask(w.n, w.S, w.L, idx[0, 0]))
    Q, K, V = (torch.tensor(x[k]) for k in ("Q", "K", "V"))
    tO = torch.nn.functional.scaled_dot_product_attention(Q, K.repeat_interleave(2, 1), V.repeat_interleave(2, 1),
                                                          attn_mask=vis)
    assert np.allclose(O, tO.numpy(), rtol=1e-10, atol=1e-12)
    assert not np.allclose(O, _dense_causal_torch(x)[0], rtol=1e-3)


def test_key_shift_invariance():
    """Adding one constant vector to every K row changes neither the scores (Eq. 6) nor O (Eq. 3)."""
    w, x = _micro(n=2 + 4 * 8, L=8, S=2, K=3, d=16)
    sc, idx = _idx(w, x, np.float64)
    c = np.random.default_rng(3).normal(size=w.d)
    sc2 = ref.score(x["K"] + c, x["V"], w.S, w.L, dtype=np.float64)
    assert np.allclose(sc, sc2, rtol=1e-9)
    O, _ = ref.attn_fwd_dense(x["Q"], x["K"], x["V"], idx, w.S, w.L)
    O2, _ = ref.attn_fwd_dense(x["Q"], x["K"] + c, x["V"], idx, w.S, w.L)
    assert np.allclose(O, O2, rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------- backward: finite differences
def test_backward_matches_finite_differences_every_element():
    w, x = _micro(n=2 + 3 * 6 + 2, L=6, S=2, K=2, d=4, Hq=2, Hkv=1)
    _, idx = _idx(w, x)
    dQ, dK, dV = ref.attn_bwd_dense(x["Q"], x["K"], x["V"], x["dO"], idx, w.S, w.L)
    eps = 1e-5
    for name, g in (("Q", dQ), ("K", dK), ("V", dV)):
        fd = np.zeros_like(g)
        it = np.nditer(x[name], flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            y = {k: v.copy() for k, v in x.items()}
            y[name][i] += eps
            lp = ref.loss(y["Q"], y["K"], y["V"], x["dO"], idx, w.S, w.L)
            y[name][i] -= 2 * eps
            lm = ref.loss(y["Q"], y["K"], y["V"], x["dO"], idx, w.S, w.L)
            fd[i] = (lp - lm) / (2 * eps)
        assert np.allclose(fd, g, rtol=1e-6, atol=1e-8), name


def test_backward_directional_derivatives_on_C1():
    w = inputs.WORKLOADS["C1"]
    x = {k: _np(v).astype(np.float64) for k, v in inputs.make_inputs(w).items()}
    _, idx = _idx(w, x)
    dQ, dK, dV = ref.attn_bwd_dense(x["Q"], x["K"], x["V"], x["dO"], idx, w.S, w.L)
    rng = np.random.default_rng(4)
    eps = 1e-5
    for _ in range(6):
        v = {k: rng.normal(size=x[k].shape) for k in ("Q", "K", "V")}
        lp = ref.loss(x["Q"] + eps * v["Q"], x["K"] + eps * v["K"], x["V"] + eps * v["V"], x["dO"], idx, w.S, w.L)
        lm = ref.loss(x["Q"] - eps * v["Q"], x["K"] - eps * v["K"], x["V"] - eps * v["V"], x["dO"], idx, w.S, w.L)
        ana = (dQ * v["Q"]).sum() + (dK * v["K"]).sum() + (dV * v["V"]).sum()
        assert np.isclose((lp - lm) / (2 * eps), ana, rtol=1e-6)


def test_softmax_row_invariants():
    """Rows of A sum to 1; rows of dS sum to 0 -> <dQ,Q> summed over a group equals <dK,K>, and
    <dV,V> equals the loss."""
    w, x = _micro(n=2 + 4 * 8 + 3, L=8, S=2, K=3, d=16, Hq=4, Hkv=2)
    _, idx = _idx(w, x)
    dQ, dK, dV = ref.attn_bwd_dense(x["Q"], x["K"], x["V"], x["dO"], idx, w.S, w.L)
    assert np.isclose((dQ * x["Q"]).sum(), (dK * x["K"]).sum(), rtol=1e-9)
    assert np.isclose((dV * x["V"]).sum(), ref.loss(x["Q"], x["K"], x["V"], x["dO"], idx, w.S, w.L), rtol=1e-9)


# ---------------------------------------------------------------- the C row/column oracle = the dense oracle
@pytest.mark.parametrize("cfg", [
    dict(n=3 + 5 * 8 + 2, L=8, S=3, K=2, d=16, Hq=4, Hkv=2, B=2),
    dict(n=0 + 6 * 5, L=5, S=0, K=5, d=8, Hq=2, Hkv=2, B=1),
    dict(n=4 + 2 * 8 - 1, L=8, S=4, K=3, d=8, Hq=3, Hkv=1, B=1),       # Ns = 0
])
def test_rowwise_c_oracle_equals_dense_oracle(cfg):
    w, x = _micro(**cfg)
    Ns = ref.partition(w.n, w.S, w.L)["Ns"]
    idx = _idx(w, x)[1] if Ns else None
    O, lse = ref.attn_fwd_dense(x["Q"], x["K"], x["V"], idx, w.S, w.L)
    dQ, dK, dV = ref.attn_bwd_dense(x["Q"], x["K"], x["V"], x["dO"], idx, w.S, w.L)
    G = w.G
    for b in range(w.B):
        for h in range(w.Hkv):
            sl = slice(h * G, (h + 1) * G)
            r = rows.attn_group(x["Q"][b, sl], x["K"][b, h], x["V"][b, h], x["dO"][b, sl],
                                None if idx is None else idx[b, h], w.S, w.L, w.K)
            assert np.allclose(r["O"], O[b, sl], rtol=1e-11, atol=1e-13)
            assert np.allclose(r["lse"], lse[b, sl], rtol=1e-12)
            assert np.allclose(r["dQ"], dQ[b, sl], rtol=1e-10, atol=1e-13)
            assert np.allclose(r["dK"], dK[b, h], rtol=1e-10, atol=1e-13)
            assert np.allclose(r["dV"], dV[b, h], rtol=1e-10, atol=1e-13)
    # sampled rows / columns agree with the full evaluation
    pick = np.array([0, w.S, w.n // 2, w.n - 1])
    r = rows.attn_rows(x["Q"][0, :G], x["K"][0, 0], x["V"][0, 0], x["dO"][0, :G],
                       None if idx is None else idx[0, 0], pick, w.S, w.L, w.K)
    assert np.allclose(r["O"], O[0, :G][:, pick], rtol=1e-11, atol=1e-13)
    # a caller that wants lse and D only gets the same O, lse and D, and no dQ
    r2 = rows.attn_rows(x["Q"][0, :G], x["K"][0, 0], x["V"][0, 0], x["dO"][0, :G],
                        None if idx is None else idx[0, 0], pick, w.S, w.L, w.K, want_dq=False)
    assert "dQ" not in r2 and all(np.array_equal(r2[k], r[k]) for k in ("O", "lse", "D"))
    c = rows.attn_cols(x["Q"][0, :G], x["K"][0, 0], x["V"][0, 0], x["dO"][0, :G],
                       None if idx is None else idx[0, 0], pick, w.S, w.L, w.K)
    assert np.allclose(c["dK"], dK[0, 0][pick], rtol=1e-10, atol=1e-13)
    assert np.allclose(c["dV"], dV[0, 0][pick], rtol=1e-10, atol=1e-13)


def test_local_prev_two_keeps_two_chunks():
    w, x = _micro(n=2 + 6 * 6, L=6, S=2, K=2, d=8, Hq=1)
    sc = ref.score(x["K"], x["V"], w.S, w.L, local_prev=2)
    assert sc.shape[2] == ref.partition(w.n, w.S, w.L, 2)["Ns"] == 3
    idx = ref.select(sc, w.S, w.L, w.K)
    vis = ref.visible_mask(w.n, w.S, w.L, idx[0, 0], local_prev=2)
    t = w.S + 4 * w.L
    assert vis[t, w.S + 2 * w.L: t + 1].all()
    assert vis[t, w.S: w.S + 2 * w.L].sum() == 2 * w.K
    for tt in range(w.n):
        assert vis[tt].sum() == ref.visible_count(tt, w.n, w.S, w.L, w.K, 2)


# ---------------------------------------------------------------- input generator
def test_inputs_are_seeded_and_sliceable():
    w = inputs.WORKLOADS["C2"].with_(n=16 + 3 * 256)
    a = inputs.make_tensor(w, "K")
    b = inputs.make_tensor(w, "K", heads=[5, 2])
    assert torch.equal(a[:, 5], b[:, 0]) and torch.equal(a[:, 2], b[:, 1])
    assert a.dtype == torch.bfloat16 and a.shape == (2, 8, w.n, 128)
    ch = inputs.outlier_channels(w, 5)
    plain = inputs.make_tensor(w, "K", heads=[5], structured=False)
    assert torch.equal(b[:, 0][..., ch], plain[:, 0][..., ch] * 8)
    w5 = inputs.WORKLOADS["C5"].with_(n=4096, Hq=8, Hkv=1)
    k5 = inputs.make_tensor(w5, "K").float(); p5 = inputs.make_tensor(w5, "K", structured=False).float()
    v5 = inputs.make_tensor(w5, "V").float(); q5 = inputs.make_tensor(w5, "V", structured=False).float()
    heavy_k = (k5 != p5).any(-1)[0, 0]; heavy_v = (v5 != q5).any(-1)[0, 0]
    assert torch.equal(heavy_k, heavy_v) and 10 < heavy_k.sum() < 90
    w4 = inputs.WORKLOADS["C4"].with_(n=4096, Hq=4, Hkv=1)
    drift = inputs.make_tensor(w4, "K").float() - inputs.make_tensor(w4, "K", structured=False).float()
    assert drift[0, 0, 0].abs().max() < 0.02 and 0.2 < drift[0, 0, -1].std() < 1.5


# ------------------------------------------------------------------ inference-time cache (oracle/lrsa_decode.py)
def test_incremental_cache_equals_gather_list_plus_window():
    """Token-by-token compression of the cache must leave exactly what the training-time mask lets the
    last query see: the sink, the survivors of the compressed chunks (the selection depends only on the
    original rows of a chunk and of the chunk after it), the previous chunk in full and the own chunk --
    with and without a tail, exactly at a chunk boundary and one token past it."""
    from oracle import lrsa_decode as dec
    rng = np.random.default_rng(11)
    for (n, S, L, K) in [(3 + 5 * 8 + 5, 3, 8, 3), (4 + 6 * 8, 4, 8, 2), (0 + 4 * 6 + 1, 0, 6, 6),
                         (2 + 2 * 8 - 1, 2, 8, 4), (2 + 2 * 8 + 1, 2, 8, 4), (5, 9, 8, 4)]:
        Kh = rng.standard_normal((n, 16)).astype(np.float32)
        Vh = rng.standard_normal((n, 16)).astype(np.float32)
        Kc, Vc, pos, done = dec.cache_incremental(Kh, Vh, S, L, K)
        part = ref.partition(n, S, L)
        assert done == part["Ns"]
        if part["Ns"]:
            idx = ref.select(ref.score(Kh[None, None], Vh[None, None], S, L), S, L, K)[0, 0]
        else:
            idx = np.zeros((0, K), np.int32)
        want = np.concatenate([np.arange(min(S, n)), idx.reshape(-1), np.arange(S + L * done, n)]) if n > S else np.arange(n)
        assert np.array_equal(pos, want)
        assert np.array_equal(Kc, Kh[pos]) and np.array_equal(Vc, Vh[pos])
        # ... which is the visible set of the last row of the training-time mask
        vis = np.flatnonzero(ref.visible_mask(n, S, L, idx if part["Ns"] else None)[n - 1])
        assert np.array_equal(np.sort(pos), vis)


def test_decode_attention_equals_last_row_of_the_masked_attention():
    from oracle import lrsa_decode as dec
    rng = np.random.default_rng(12)
    n, S, L, K, d, G = 2 + 5 * 8 + 3, 2, 8, 3, 16, 3
    Q = rng.standard_normal((1, G, n, d)); Kh = rng.standard_normal((1, 1, n, d)).astype(np.float32)
    Vh = rng.standard_normal((1, 1, n, d)).astype(np.float32)
    idx = ref.select(ref.score(Kh, Vh, S, L), S, L, K)
    O_ref, lse_ref = ref.attn_fwd_dense(Q, Kh, Vh, idx, S, L)
    Kc, Vc, pos, done = dec.cache_incremental(Kh[0, 0], Vh[0, 0], S, L, K)
    O, lse = dec.decode_attn(Q[0, :, n - 1], Kc, Vc)
    assert np.allclose(O, O_ref[0, :, n - 1], rtol=1e-12, atol=1e-12)
    assert np.allclose(lse, lse_ref[0, :, n - 1], rtol=1e-12, atol=1e-12)
    # closed form: one key -> the output is that key's value row, lse = the logit
    O1, l1 = dec.decode_attn(Q[0, :, 0], Kh[0, 0, :1], Vh[0, 0, :1])
    assert np.allclose(O1, np.repeat(Vh[0, 0, :1], G, 0)) and np.allclose(l1, Q[0, :, 0] @ Kh[0, 0, 0] / np.sqrt(d))
