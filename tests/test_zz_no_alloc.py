"""lrsa_decode_attn_static (the entry point that allocates nothing: its slice records live in an array inside
the library) against lrsa_decode_attn (same kernels with a caller's workspace), through the C ABI.

Bar: bit-identical O and lse, on two calls in a row on the same GPU, the second with a smaller input (fewer
cache rows, fewer heads), so that records left by the first call must not leak into the second; then the size
limit is checked on the host side.
"""
import ctypes

import pytest
import torch

import paper_2506_11498_amd as lrsa
from paper_2506_11498_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(B, Hq, Hkv, cap, d, length, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    Kc = torch.randn((B, Hkv, cap, d), generator=g).to(torch.bfloat16).to(DEV)
    Vc = torch.randn((B, Hkv, cap, d), generator=g).to(torch.bfloat16).to(DEV)
    q = torch.randn((B, Hq, d), generator=g).to(torch.bfloat16).to(DEV)
    p = lrsa.make_params((B, Hq, cap, d), (B, Hkv, cap, d), (Hq * cap * d, cap * d, d, 1), Kc.stride(),
                         dtype=torch.bfloat16, sink=16, lag=256, topk=64)
    return p, q, Kc, Vc, length


def _both(p, q, Kc, Vc, length):
    L = lrsa.lib()
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    B, Hq, d = q.shape
    O_ws, O_st = torch.zeros_like(q), torch.zeros_like(q)
    lse_ws = torch.zeros((B, Hq), dtype=torch.float32, device=DEV)
    lse_st = torch.zeros_like(lse_ws)
    need = lrsa.workspace_bytes(p, binding.WS_DECODE_ATTN)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    rc = L.lrsa_decode_attn(ctypes.byref(p), vp(q), vp(Kc), vp(Vc), length, vp(O_ws), vp(lse_ws), vp(ws), need, stream)
    assert rc == 0, L.lrsa_last_error()
    rc = L.lrsa_decode_attn_static(ctypes.byref(p), vp(q), vp(Kc), vp(Vc), length, vp(O_st), vp(lse_st), stream)
    assert rc == 0, L.lrsa_last_error()
    torch.cuda.synchronize()
    return (O_ws, lse_ws), (O_st, lse_st)


def test_static_scratch_decode_equals_workspace_decode_twice_in_a_row():
    big = _case(B=2, Hq=16, Hkv=4, cap=9600, d=128, length=9536, seed=11)     # 37 slices per (batch, KV head)
    small = _case(B=1, Hq=4, Hkv=2, cap=1024, d=128, length=700, seed=12)     # 3 slices
    for case in (big, small):
        (O_ws, lse_ws), (O_st, lse_st) = _both(*case)
        assert torch.isfinite(O_st.float()).all() and O_st.float().abs().max() > 0
        assert torch.equal(O_st, O_ws) and torch.equal(lse_st, lse_ws)


def test_static_scratch_decode_rejects_what_does_not_fit():
    # batch * heads_q * slices * (d + 2) * 4 bytes: 8 * 64 * 64 * 130 * 4 = 17 MB > 4 MiB
    p, q, Kc, Vc, length = _case(B=8, Hq=64, Hkv=1, cap=16384, d=128, length=16384, seed=13)
    L = lrsa.lib()
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    O = torch.zeros_like(q)
    rc = L.lrsa_decode_attn_static(ctypes.byref(p), vp(q), vp(Kc), vp(Vc), length, vp(O), None, None)
    assert rc == -1 and b"scratch" in L.lrsa_last_error()
    torch.cuda.synchronize()
    assert float(O.float().abs().max()) == 0.0          # nothing was launched
