"""The one-read (streaming) scoring kernels against the oracle, on shapes that the library routes to them.

Which kernel scores a shape is the library's choice (bf16, head_dim 128 and enough (batch, KV head) streams to
fill the chip go to the streaming kernel); each case here first checks, through the library's kernel timers,
that the streaming kernel is the one that ran, so that the comparison below is a test of it.  Bars as in
test_gpu_parity.py: scores within 2e-5 (relative) of the oracle's fp32 scores, selections equal to the
oracle's outside a 1e-6 window around each chunk's K-th largest score.
"""
import numpy as np
import pytest
import torch

import paper_2506_11498_amd as lrsa
from paper_2506_11498_amd import inputs
from oracle import lrsa_ref as ref
from test_gpu_parity import check_selection_in_tie_window, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

STREAMED = [
    # whole chunks per workgroup, one block of rows per chunk, two chunk ranges per stream
    dict(name="whole_chunks", n=16 + 16 * 128 + 5, L=128, S=16, K=32, d=128, Hq=64, Hkv=64, B=1, dtype="bf16"),
    # two sibling workgroups per chunk (they exchange min / max), two blocks per slice
    dict(name="siblings", n=16 + 16 * 512 + 100, L=512, S=16, K=100, d=128, Hq=32, Hkv=32, B=1, dtype="bf16"),
    # slices of 300 rows: the last block of a slice overlaps the one before it
    dict(name="siblings_ragged", n=16 + 16 * 600 + 100, L=600, S=16, K=100, d=128, Hq=32, Hkv=32, B=1, dtype="bf16"),
    # batch of two, 200-row chunks (a ragged second block), three ranges of 8, 8 and 6 chunks
    dict(name="batch_ragged_ranges", n=7 + 23 * 200 + 100, L=200, S=7, K=50, d=128, Hq=16, Hkv=16, B=2, dtype="bf16"),
]


def kernels_of(fn):
    lrsa.timing_enable(True)
    try:
        out = fn()
        torch.cuda.synchronize()
        names = {k for k, _ in lrsa.timing_records()}
    finally:
        lrsa.timing_enable(False)
    return out, names


@pytest.mark.parametrize("cfg", STREAMED, ids=[c["name"] for c in STREAMED])
def test_streamed_scores_and_selection_match_the_oracle(cfg):
    cfg = {k: v for k, v in cfg.items() if k != "name"}
    w = inputs.small_workload(**cfg)
    x = inputs.make_inputs(w)
    xd = {k: x[k].to(DEV) for k in ("Q", "K", "V")}
    p = lrsa.params_for(xd["Q"], xd["K"], sink=w.S, lag=w.L, topk=w.K)
    (score, idx), names = kernels_of(lambda: lrsa.lrsa_score_select(p, xd["K"], xd["V"]))
    assert names == {"k_score_stream", "k_softmax_select"}, names
    sc_ref = ref.score(x["K"].float().numpy(), x["V"].float().numpy(), w.S, w.L)
    idx_ref = ref.select(sc_ref, w.S, w.L, w.K)
    assert np.allclose(to_np(score), sc_ref, rtol=2e-5, atol=1e-9)
    _, outside_rel = check_selection_in_tie_window(w, idx.cpu().numpy(), idx_ref, sc_ref)
    assert outside_rel == 0
    # the score-only entry point takes the same kernels without the selection: the same bits
    score_only, names = kernels_of(lambda: lrsa.lrsa_score(p, xd["K"], xd["V"]))
    assert names == {"k_score_stream", "k_softmax"}, names
    assert torch.equal(score_only, score)
    # and the stand-alone selection of those scores is the fused one
    assert torch.equal(lrsa.lrsa_select(p, score), idx)


def test_streamed_results_do_not_depend_on_call_history_or_layout():
    """The sibling workgroups' mailboxes live in library-owned device memory and survive a call: repeated
    calls, calls on other shapes in between, and K / V stored token-major ([B, n, Hkv, d], rows of one head
    Hkv * d elements apart) must all give the bits of the first call."""
    cfg = dict(n=16 + 16 * 512 + 100, L=512, S=16, K=100, d=128, Hq=32, Hkv=32, B=1, dtype="bf16")
    other = dict(n=16 + 16 * 600 + 100, L=600, S=16, K=100, d=128, Hq=32, Hkv=32, B=1, dtype="bf16")
    w, w2 = inputs.small_workload(**cfg), inputs.small_workload(seed=11, **other)
    x, x2 = inputs.make_inputs(w), inputs.make_inputs(w2)
    xd = {k: x[k].to(DEV) for k in ("Q", "K", "V")}
    xd2 = {k: x2[k].to(DEV) for k in ("Q", "K", "V")}
    p = lrsa.params_for(xd["Q"], xd["K"], sink=w.S, lag=w.L, topk=w.K)
    p2 = lrsa.params_for(xd2["Q"], xd2["K"], sink=w2.S, lag=w2.L, topk=w2.K)
    score0, idx0 = lrsa.lrsa_score_select(p, xd["K"], xd["V"])
    for _ in range(3):
        lrsa.lrsa_score_select(p2, xd2["K"], xd2["V"])
        score, idx = lrsa.lrsa_score_select(p, xd["K"], xd["V"])
        assert torch.equal(score, score0) and torch.equal(idx, idx0)
    # token-major storage, viewed as [B, Hkv, n, d]
    Kt = xd["K"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Vt = xd["V"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert Kt.stride(2) == w.Hkv * w.d
    pt = lrsa.params_for(xd["Q"], Kt, sink=w.S, lag=w.L, topk=w.K)
    (score_t, idx_t), names = kernels_of(lambda: lrsa.lrsa_score_select(pt, Kt, Vt))
    assert "k_score_stream" in names
    assert torch.equal(score_t, score0) and torch.equal(idx_t, idx0)
