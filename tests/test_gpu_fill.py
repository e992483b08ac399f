"""Attention by filling steps (lrsa_attn_fwd_fill / lrsa_attn_bwd_fill / lrsa_attn_bwd_finish; Section 3.2 of the
paper, Attention Filling 1 / 2 / repeat): m query chunks per step against sink + survivors + the previous chunk.

Bars: O, lse and dQ of the steps, put together, equal the one-shot calls bit for bit (same tiles, same walk);
dK, dV equal them within the bf16 tolerance (the fp32 additions come in another order); everything is within
2e-2 relative of the fp64 oracle, which knows nothing of steps.  The workspace of a step is printed beside the
one-shot workspace.
"""
import numpy as np
import pytest
import torch

import paper_2506_11498_amd as lrsa
from paper_2506_11498_amd import inputs
from oracle import lrsa_ref as ref

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = [
    dict(name="gqa", n=16 + 6 * 64 + 40, L=64, S=16, K=16, d=128, Hq=8, Hkv=2, B=2),
    dict(name="odd_sizes_no_tail_chunk", n=5 + 7 * 100, L=100, S=5, K=37, d=128, Hq=2, Hkv=1, B=1),
    dict(name="no_sink_long_chunks", n=0 + 5 * 320 + 100, L=320, S=0, K=80, d=128, Hq=4, Hkv=1, B=1),
    dict(name="many_chunks", n=64 + 20 * 128 + 9, L=128, S=64, K=32, d=128, Hq=8, Hkv=1, B=1),
]


def windows(w, m):
    """Row windows of the filling steps: the sink with the first m chunks, then m chunks at a time."""
    if w.n <= w.S:
        return [(0, w.n)]
    nq = -(-(w.n - w.S) // w.L)
    cuts = [0] + [w.S + q * w.L for q in range(m, nq, m)] + [w.n]
    return list(zip(cuts[:-1], cuts[1:]))


def rel(x, r):
    x = np.asarray(x, np.float64); r = np.asarray(r, np.float64)
    return max(np.abs(x - r).max() / np.abs(r).max(), np.linalg.norm(x - r) / np.linalg.norm(r))


@pytest.mark.parametrize("m", [1, 2, 3])
@pytest.mark.parametrize("local_prev", [1, 2])
@pytest.mark.parametrize("cfg", SHAPES, ids=[c["name"] for c in SHAPES])
def test_filling_steps_equal_one_shot_and_oracle(cfg, m, local_prev):
    if local_prev == 2 and cfg["name"] != "gqa":
        pytest.skip("local_prev = 2 is exercised on one shape")
    cfg = {k: v for k, v in cfg.items() if k != "name"}
    w = inputs.small_workload(dtype="bf16", **cfg)
    x = inputs.make_inputs(w)
    xf = {k: v.float().numpy() for k, v in x.items()}
    xd = {k: v.to(DEV) for k, v in x.items()}
    p = lrsa.params_for(xd["Q"], xd["K"], sink=w.S, lag=w.L, topk=w.K, local_prev=local_prev)
    Ns = lrsa.num_scored_chunks(p)
    idx_ref = ref.select(ref.score(xf["K"], xf["V"], w.S, w.L, local_prev=local_prev), w.S, w.L, w.K) if Ns else None
    idx = torch.from_numpy(idx_ref).to(DEV) if Ns else None
    O1, lse1 = lrsa.lrsa_attn_fwd(p, xd["Q"], xd["K"], xd["V"], idx)
    dQ1, dK1, dV1 = lrsa.lrsa_attn_bwd(p, xd["Q"], xd["K"], xd["V"], O1, xd["dO"], lse1, idx)

    O = torch.zeros_like(O1); lse = torch.zeros_like(lse1); dQ = torch.zeros_like(dQ1)
    accK = torch.zeros(xd["K"].shape, dtype=torch.float32, device=DEV)
    accV = torch.zeros_like(accK)
    steps = windows(w, m)
    ws_fwd = ws_bwd = 0
    for a, b in steps:
        Qs = xd["Q"][:, :, a:b].contiguous()
        pf = lrsa.params_for(Qs, xd["K"], sink=w.S, lag=w.L, topk=w.K, local_prev=local_prev)
        pf.seq = w.n
        ws_fwd = max(ws_fwd, lrsa.fill_workspace_bytes(pf, a, b, 2))
        Os, ls = lrsa.lrsa_attn_fwd_fill(pf, a, b, Qs, xd["K"], xd["V"], idx)
        O[:, :, a:b] = Os
        lse[:, :, a:b] = ls
    assert torch.equal(O, O1) and torch.equal(lse, lse1)
    for a, b in reversed(steps):
        Qs, Os, dOs = (xd[k][:, :, a:b].contiguous() if k != "O" else O[:, :, a:b].contiguous() for k in ("Q", "O", "dO"))
        pf = lrsa.params_for(Qs, xd["K"], sink=w.S, lag=w.L, topk=w.K, local_prev=local_prev)
        pf.seq = w.n
        ws_bwd = max(ws_bwd, lrsa.fill_workspace_bytes(pf, a, b, 3))
        dQ[:, :, a:b] = lrsa.lrsa_attn_bwd_fill(pf, a, b, Qs, xd["K"], xd["V"], Os, dOs, lse[:, :, a:b].contiguous(), idx, accK, accV)
    dK, dV = torch.empty_like(xd["K"]), torch.empty_like(xd["K"])
    lrsa.lrsa_attn_bwd_finish(p, accK, accV, dK, dV)
    torch.cuda.synchronize()
    print(f"m={m}: workspace per step fwd {ws_fwd} / bwd {ws_bwd} bytes; one-shot fwd {lrsa.workspace_bytes(p, 2)} / "
          f"bwd {lrsa.workspace_bytes(p, 3)} bytes")
    assert torch.equal(dQ, dQ1)
    assert rel(dK.float().cpu().numpy(), dK1.float().cpu().numpy()) < 2e-2
    assert rel(dV.float().cpu().numpy(), dV1.float().cpu().numpy()) < 2e-2
    O_ref, lse_ref = ref.attn_fwd_dense(xf["Q"], xf["K"], xf["V"], idx_ref, w.S, w.L, local_prev=local_prev)
    g = ref.attn_bwd_dense(xf["Q"], xf["K"], xf["V"], xf["dO"], idx_ref, w.S, w.L, local_prev=local_prev)
    assert rel(O.float().cpu().numpy(), O_ref) < 2e-2
    assert np.abs(lse.cpu().numpy() - lse_ref).max() < 1e-3
    assert rel(dQ.float().cpu().numpy(), g[0]) < 2e-2
    assert rel(dK.float().cpu().numpy(), g[1]) < 2e-2
    assert rel(dV.float().cpu().numpy(), g[2]) < 2e-2


def test_filling_steps_at_full_size_C4_equal_the_one_shot_call():
    """The headline workload (32K tokens, 32/8 heads) in steps of 4 chunks, with the library's own selection:
    O, lse and dQ bit for bit, dK and dV within 2e-3 of the one-shot call (which the full-size parity tests hold
    against the oracle); the step-wise schedule's time and workspace are printed beside the one-shot call's."""
    w = inputs.WORKLOADS["C4"]
    xd = {k: v.to(DEV) for k, v in inputs.make_inputs(w).items()}
    p = lrsa.params_for(xd["Q"], xd["K"], sink=w.S, lag=w.L, topk=w.K)
    _, idx = lrsa.lrsa_score_select(p, xd["K"], xd["V"])
    O1, lse1 = lrsa.lrsa_attn_fwd(p, xd["Q"], xd["K"], xd["V"], idx)
    dQ1, dK1, dV1 = lrsa.lrsa_attn_bwd(p, xd["Q"], xd["K"], xd["V"], O1, xd["dO"], lse1, idx)
    torch.cuda.synchronize()
    m = 4
    steps = windows(w, m)
    O = torch.empty_like(O1); lse = torch.empty_like(lse1); dQ = torch.empty_like(dQ1)
    accK = torch.zeros(xd["K"].shape, dtype=torch.float32, device=DEV)
    accV = torch.zeros_like(accK)
    dK, dV = torch.empty_like(xd["K"]), torch.empty_like(xd["K"])
    params = {}
    for a, b in steps:
        pf = lrsa.params_for(xd["Q"][:, :, a:b], xd["K"], sink=w.S, lag=w.L, topk=w.K)   # Q, O, dO, dQ rows as views
        pf.seq = w.n
        params[(a, b)] = pf
    ws = torch.empty(max(max(lrsa.fill_workspace_bytes(params[s_], s_[0], s_[1], k) for s_ in steps) for k in (2, 3)) + 256,
                     dtype=torch.uint8, device=DEV)
    lse_rows = {s_: torch.empty((w.B, w.Hq, s_[1] - s_[0]), dtype=torch.float32, device=DEV) for s_ in steps}   # contiguous per step
    for timed in (False, True):          # the first pass warms the allocator and the code objects up
        accK.zero_(); accV.zero_()
        t0, t1, t2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        t0.record()
        for a, b in steps:
            lrsa.lrsa_attn_fwd_fill(params[(a, b)], a, b, xd["Q"][:, :, a:b], xd["K"], xd["V"], idx, O[:, :, a:b], lse_rows[(a, b)], ws)
        t1.record()
        for a, b in reversed(steps):
            lrsa.lrsa_attn_bwd_fill(params[(a, b)], a, b, xd["Q"][:, :, a:b], xd["K"], xd["V"], O[:, :, a:b], xd["dO"][:, :, a:b],
                                    lse_rows[(a, b)], idx, accK, accV, dQ[:, :, a:b], ws)
        lrsa.lrsa_attn_bwd_finish(p, accK, accV, dK, dV)
        t2.record()
        torch.cuda.synchronize()
    for a, b in steps:
        lse[:, :, a:b] = lse_rows[(a, b)]
    print(f"C4 in {len(steps)} steps of {m} chunks: forward {t0.elapsed_time(t1):.2f} ms, backward {t1.elapsed_time(t2):.2f} ms "
          f"(host-driven, includes launch gaps); workspace {ws.numel() / 1e6:.0f} MB + {2 * accK.numel() * 4 / 1e6:.0f} MB of accumulators "
          f"against {lrsa.workspace_bytes(p, 3) / 1e6:.0f} MB one-shot")
    assert torch.equal(O, O1) and torch.equal(lse, lse1) and torch.equal(dQ, dQ1)
    for name, x, r in (("dK", dK, dK1), ("dV", dV, dV1)):
        x = x.float(); r = r.float()
        e = max(((x - r).abs().max() / r.abs().max()).item(), ((x - r).norm() / r.norm()).item())
        assert e < 2e-3, (name, e)


def test_fill_rejects_windows_off_the_chunk_grid():
    w = inputs.small_workload(n=16 + 6 * 64 + 40, L=64, S=16, K=16, d=128, Hq=4, Hkv=2, B=1, dtype="bf16")
    xd = {k: v.to(DEV) for k, v in inputs.make_inputs(w).items()}
    p = lrsa.params_for(xd["Q"], xd["K"], sink=w.S, lag=w.L, topk=w.K)
    for a, b in ((0, 50), (17, 16 + 64), (16 + 64, 16 + 64), (16, w.n + 1)):
        assert lrsa.fill_workspace_bytes(p, a, b, 3) == 0
