"""Inference-time LagKV cache on the GPU (lrsa_cache_compress, lrsa_decode_attn) against the CPU oracle.

Bars: the compressed cache and its position array are copies of input rows, so they must equal the oracle's
bit for bit whenever the selection does (it is checked against the oracle's tie window otherwise, as for the
training-time selection); the attention output within 1e-4 (fp32) / 2e-2 (bf16) relative, lse within 1e-3.
"""
import numpy as np
import pytest
import torch

import paper_2506_11498_amd as lrsa
from paper_2506_11498_amd import inputs
from oracle import lrsa_decode as dec
from oracle import lrsa_ref as ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    dict(n=3 + 5 * 16 + 7, L=16, S=3, K=4, d=64, Hq=2, Hkv=1, B=2, dtype="f32"),
    dict(n=0 + 4 * 24 + 1, L=24, S=0, K=24, d=128, Hq=2, Hkv=2, B=1, dtype="f32"),          # keep everything
    dict(n=8 + 5 * 32 + 11, L=32, S=8, K=8, d=64, Hq=4, Hkv=2, B=1, dtype="bf16"),
    dict(n=16 + 4 * 256 + 100, L=256, S=16, K=64, d=128, Hq=8, Hkv=2, B=2, dtype="bf16"),
    dict(n=64 + 3 * 1024 + 500, L=1024, S=64, K=256, d=128, Hq=12, Hkv=1, B=1, dtype="bf16"),  # group of 12: two passes
    dict(n=5, L=8, S=16, K=2, d=64, Hq=1, Hkv=1, B=1, dtype="f32"),                          # shorter than the sink
]


def feed_cache(w, x, feed):
    """Appends the rows of K, V to a device cache `feed` tokens at a time (never past a tail of 2L), compressing
    before each append as the header asks.  Returns (Kc, Vc, pos, length, done) as the last token sees them."""
    cap = w.S + 2 * w.L + w.n            # generous
    Kc = torch.zeros((w.B, w.Hkv, cap, w.d), dtype=x["K"].dtype, device=DEV)
    Vc = torch.zeros_like(Kc)
    p = lrsa.make_params((w.B, w.Hq, cap, w.d), tuple(Kc.shape), (w.Hq * cap * w.d, cap * w.d, w.d, 1), Kc.stride(),
                         dtype=Kc.dtype, sink=w.S, lag=w.L, topk=w.K)
    pos = torch.full((w.B, w.Hkv, cap), -1, dtype=torch.int32, device=DEV)
    Kd, Vd = x["K"].to(DEV), x["V"].to(DEV)
    length = done = t = 0
    while t < w.n:
        length, done = lrsa.lrsa_cache_compress(p, Kc, Vc, pos, length, done)
        room = (w.S + w.K * done + 2 * w.L) - length     # rows until the tail holds 2L
        m = max(1, min(feed, w.n - t, room))
        Kc[:, :, length:length + m] = Kd[:, :, t:t + m]
        Vc[:, :, length:length + m] = Vd[:, :, t:t + m]
        pos[:, :, length:length + m] = torch.arange(t, t + m, dtype=torch.int32, device=DEV)
        length += m
        t += m
    return p, Kc, Vc, pos, length, done


@pytest.mark.parametrize("feed", [1, 7, 4096])
@pytest.mark.parametrize("cfg", CASES, ids=[f"n{c['n']}_L{c['L']}_{c['dtype']}" for c in CASES])
def test_cache_and_decode_attention_against_oracle(cfg, feed):
    if feed == 1 and cfg["n"] > 600:
        pytest.skip("token-by-token feeding is exercised on the short cases")
    w = inputs.small_workload(**cfg)
    x = inputs.make_inputs(w)
    p, Kc, Vc, pos, length, done = feed_cache(w, x, feed)
    Kf, Vf = x["K"].float().numpy(), x["V"].float().numpy()
    t = 1e-4 if w.dtype == "f32" else 2e-2
    q = x["Q"][:, :, w.n - 1].contiguous().to(DEV)           # the last token's queries
    O, lse = lrsa.lrsa_decode_attn(p, q, Kc, Vc, length)
    O, lse = O.float().cpu().numpy(), lse.cpu().numpy()
    for b in range(w.B):
        for h in range(w.Hkv):
            Ko, Vo, po, do = dec.cache_incremental(Kf[b, h], Vf[b, h], w.S, w.L, w.K)
            assert (length, done) == (len(po), do)
            got = pos[b, h, :length].cpu().numpy()
            if not np.array_equal(got, po):
                # the two selections may differ only inside the oracle's fp32 tie window
                sc = ref.score(Kf[b:b + 1, h:h + 1], Vf[b:b + 1, h:h + 1], w.S, w.L)[0, 0]
                for c in range(do):
                    a, o = got[w.S + c * w.K: w.S + (c + 1) * w.K], po[w.S + c * w.K: w.S + (c + 1) * w.K]
                    s = sc[c]
                    diff = np.setxor1d(a, o) - (w.S + c * w.L)
                    assert np.all(np.abs(s[diff] - np.sort(s)[-w.K]) <= 1e-6)
                Ko, Vo = Kf[b, h][got], Vf[b, h][got]
            assert np.array_equal(Kc[b, h, :length].float().cpu().numpy(), Ko)
            assert np.array_equal(Vc[b, h, :length].float().cpu().numpy(), Vo)
            sl = slice(h * w.G, (h + 1) * w.G)
            O_ref, lse_ref = dec.decode_attn(x["Q"][b, sl, w.n - 1].float().numpy(), Ko, Vo)
            top = max(np.abs(O_ref).max(), 1e-2)
            assert np.abs(O[b, sl] - O_ref).max() / top < t
            assert np.abs(lse[b, sl] - lse_ref).max() < 1e-3


def test_compress_is_a_no_op_below_two_chunks_and_rejects_bad_lengths():
    w = inputs.small_workload(n=100, L=16, S=4, K=4, d=64, Hq=1, Hkv=1, B=1, dtype="f32")
    Kc = torch.randn((1, 1, 128, 64), device=DEV)
    p = lrsa.make_params((1, 1, 128, 64), (1, 1, 128, 64), Kc.stride(), Kc.stride(), dtype=torch.float32, sink=4, lag=16, topk=4)
    Vc = torch.randn_like(Kc)
    K0 = Kc.clone()
    assert lrsa.lrsa_cache_compress(p, Kc, Vc, None, 4 + 31, 0) == (35, 0)
    assert torch.equal(Kc, K0)
    assert lrsa.lrsa_cache_compress(p, Kc, Vc, None, 4 + 32, 0) == (4 + 4 + 16, 1)
    with pytest.raises(lrsa.LrsaError):
        lrsa.lrsa_cache_compress(p, Kc, Vc, None, 200, 0)       # beyond the capacity
    with pytest.raises(lrsa.LrsaError):
        lrsa.lrsa_decode_attn(p, torch.randn((1, 1, 64), device=DEV), Kc, Vc, 0)
