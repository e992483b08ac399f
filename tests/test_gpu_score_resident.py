"""The one-read (chunk-resident) scoring kernel against the oracle, on shapes that the library routes to it.

Which kernel scores a shape is the library's choice (bf16, head_dim 128 and chunks of 64 to 4096 rows go to the
kernel that keeps a part of a chunk in registers from its min / max to its scores); each case here first checks,
through the library's kernel timers, that this kernel is the one that ran, so that the comparison below is a
test of it.  Bars as in test_gpu_parity.py: scores within 2e-5 (relative) of the oracle's fp32 scores,
selections equal to the oracle's outside a 1e-6 window around each chunk's K-th largest score.
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

RESIDENT = [
    # 64-row chunks: workgroups of one wave (it publishes and polls), one part per chunk
    dict(name="one_wave", n=8 + 5 * 64 + 3, L=64, S=8, K=16, d=128, Hq=1, Hkv=1, B=1, dtype="bf16"),
    # 100-row chunks cut into two parts of 64 rows, the second moved back by 28 rows
    dict(name="two_waves_overlap", n=5 + 7 * 100 + 33, L=100, S=5, K=37, d=128, Hq=2, Hkv=1, B=1, dtype="bf16"),
    # 128-thread workgroups, one part per chunk, 128 streams
    dict(name="whole_chunks", n=16 + 16 * 128 + 5, L=128, S=16, K=32, d=128, Hq=64, Hkv=64, B=1, dtype="bf16"),
    # two parts of 256 rows per chunk: a reader collects the words of two writers
    dict(name="two_parts", n=16 + 16 * 512 + 100, L=512, S=16, K=100, d=128, Hq=32, Hkv=32, B=1, dtype="bf16"),
    # 600 rows: three parts, the last one overlaps the second by 168 rows
    dict(name="three_parts_overlap", n=16 + 16 * 600 + 100, L=600, S=16, K=100, d=128, Hq=32, Hkv=32, B=1, dtype="bf16"),
    # batch of two, 200-row chunks (two parts of 128 rows that overlap by 56)
    dict(name="batch_overlap", n=7 + 23 * 200 + 100, L=200, S=7, K=50, d=128, Hq=16, Hkv=16, B=2, dtype="bf16"),
    # the longest chunk the kernel takes: sixteen parts, a reader polls in four rounds of four
    dict(name="sixteen_parts", n=8 + 4 * 4096 + 9, L=4096, S=8, K=1000, d=128, Hq=1, Hkv=1, B=1, dtype="bf16"),
    # every token of a chunk kept (the selection stops after its first pass) and a single one kept
    dict(name="keep_all", n=9 + 6 * 256 + 30, L=256, S=9, K=256, d=128, Hq=4, Hkv=2, B=1, dtype="bf16"),
    dict(name="keep_one", n=9 + 6 * 256 + 30, L=256, S=9, K=1, d=128, Hq=4, Hkv=2, B=1, dtype="bf16"),
    # more workgroups than mailbox slots (4 * 2 * 1041 = 8328 > 8192): the slots wrap around
    dict(name="slots_wrap", n=4 + 1041 * 64 + 7, L=64, S=4, K=8, d=128, Hq=4, Hkv=4, B=1, dtype="bf16"),
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


@pytest.mark.parametrize("cfg", RESIDENT, ids=[c["name"] for c in RESIDENT])
def test_resident_scores_and_selection_match_the_oracle(cfg):
    cfg = {k: v for k, v in cfg.items() if k != "name"}
    w = inputs.small_workload(**cfg)
    x = inputs.make_inputs(w)
    xd = {k: x[k].to(DEV) for k in ("Q", "K", "V")}
    p = lrsa.params_for(xd["Q"], xd["K"], sink=w.S, lag=w.L, topk=w.K)
    (score, idx), names = kernels_of(lambda: lrsa.lrsa_score_select(p, xd["K"], xd["V"]))
    assert names == {"k_score_resident", "k_softmax_select"}, names
    sc_ref = ref.score(x["K"].float().numpy(), x["V"].float().numpy(), w.S, w.L)
    idx_ref = ref.select(sc_ref, w.S, w.L, w.K)
    assert np.allclose(to_np(score), sc_ref, rtol=2e-5, atol=1e-9)
    _, outside_rel = check_selection_in_tie_window(w, idx.cpu().numpy(), idx_ref, sc_ref)
    assert outside_rel == 0
    # the score-only entry point takes the same kernels without the selection: the same bits
    score_only, names = kernels_of(lambda: lrsa.lrsa_score(p, xd["K"], xd["V"]))
    assert names == {"k_score_resident", "k_softmax"}, names
    assert torch.equal(score_only, score)
    # and the stand-alone selection of those scores is the fused one
    assert torch.equal(lrsa.lrsa_select(p, score), idx)


def test_resident_results_do_not_depend_on_call_history_or_layout():
    """The workgroups' mailboxes live in library-owned device memory and survive a call: repeated
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
    assert "k_score_resident" in names
    assert torch.equal(score_t, score0) and torch.equal(idx_t, idx0)


def test_without_the_hint_words_every_workgroup_reads_its_reference_chunk_and_gets_the_same_bits():
    """A poll limit of 0 makes every workgroup take the path that a late or overwritten mailbox would put it
    on: the min / max of the reference chunk from the rows themselves.  Scores and selections must be the bits
    of the default setting (and so, by the tests above, the oracle's within the bar)."""
    cfgs = [dict(n=16 + 16 * 600 + 100, L=600, S=16, K=100, d=128, Hq=32, Hkv=32, B=1, dtype="bf16"),
            dict(n=8 + 5 * 64 + 3, L=64, S=8, K=16, d=128, Hq=1, Hkv=1, B=1, dtype="bf16"),
            dict(n=8 + 4 * 4096 + 9, L=4096, S=8, K=1000, d=128, Hq=1, Hkv=1, B=1, dtype="bf16")]
    for cfg in cfgs:
        w = inputs.small_workload(**cfg)
        x = inputs.make_inputs(w)
        xd = {k: x[k].to(DEV) for k in ("Q", "K", "V")}
        p = lrsa.params_for(xd["Q"], xd["K"], sink=w.S, lag=w.L, topk=w.K)
        score0, idx0 = lrsa.lrsa_score_select(p, xd["K"], xd["V"])
        before = lrsa.score_poll_limit(0)
        try:
            assert lrsa.score_poll_limit(-1) == 0
            (score, idx), names = kernels_of(lambda: lrsa.lrsa_score_select(p, xd["K"], xd["V"]))
        finally:
            lrsa.score_poll_limit(before)
        assert lrsa.score_poll_limit(-1) == before == 256
        assert "k_score_resident" in names
        assert torch.equal(score, score0) and torch.equal(idx, idx0)


def test_rows_whose_normalised_channels_are_nearly_equal():
    """Eq. 7 on rows for which sum(x^2) and sum(x)^2 / d cancel: rows that sit, channel by channel, at the
    reference chunk's max (every normalised value 1), at its min (every value 0: standard deviation exactly 0),
    a hair below the max, and half way.  The kernel must take the variance of such a row from the deviations about
    the mean; the oracle's two-pass fp32 value is the bar, as for every other row."""
    cfg = dict(n=16 + 6 * 512 + 40, L=512, S=16, K=100, d=128, Hq=2, Hkv=2, B=1, dtype="bf16")
    w = inputs.small_workload(**cfg)
    x = inputs.make_inputs(w)
    K0 = x["K"].clone()
    K = x["K"].clone()
    ref_chunk = K[0, 1, w.S + 3 * w.L: w.S + 4 * w.L].float()      # chunk 3 is the reference of chunk 2
    mx, mn = ref_chunk.max(dim=0).values, ref_chunk.min(dim=0).values
    r0 = w.S + 2 * w.L
    K[0, 1, r0 + 5] = mx.to(K.dtype)
    K[0, 1, r0 + 6] = mn.to(K.dtype)
    K[0, 1, r0 + 7] = (mx - 0.004 * (mx - mn) * torch.rand(w.d, generator=torch.Generator().manual_seed(3))).to(K.dtype)
    K[0, 1, r0 + 300] = (0.5 * (mx + mn)).to(K.dtype)
    K[0, 1, r0 + 511] = mx.to(K.dtype)
    Kd, K0d, Vd, Qd = K.to(DEV), K0.to(DEV), x["V"].to(DEV), x["Q"].to(DEV)
    p = lrsa.params_for(Qd, Kd, sink=w.S, lag=w.L, topk=w.K)
    score = lrsa.lrsa_score(p, Kd, Vd)
    sc_ref = ref.score(K.float().numpy(), x["V"].float().numpy(), w.S, w.L)
    assert np.allclose(to_np(score), sc_ref, rtol=2e-5, atol=1e-9)
    # the rows with the planted values: their standard deviation is (nearly) zero, so their score is the smallest
    # K part a row can have; the row at the min has exactly sigma_K = 0
    # Chunks that neither hold the planted rows (chunk 2 of head 1) nor are normalised by that chunk (chunk 1 of
    # head 1) keep the bits they have without them.
    score_plain = lrsa.lrsa_score(p, K0d, Vd)
    same = torch.ones_like(score, dtype=torch.bool)
    same[0, 1, 2] = False
    same[0, 1, 1] = False
    assert torch.equal(score[same], score_plain[same])


def test_calls_that_overlap_on_two_streams_cost_time_never_results():
    """Two calls that score at the same time share the library's mailbox slots: each may overwrite or clear the
    words the other is waiting for.  A reader that does not find its tags takes the min / max from the rows, so
    both calls must still give the bits they give alone.  (Different shapes, so that the slots of one call mean
    other streams, chunks and parts to the other.)"""
    cfg_a = dict(n=16 + 16 * 512 + 100, L=512, S=16, K=100, d=128, Hq=32, Hkv=32, B=1, dtype="bf16")
    cfg_b = dict(n=7 + 23 * 200 + 100, L=200, S=7, K=50, d=128, Hq=16, Hkv=16, B=2, dtype="bf16")
    wa, wb = inputs.small_workload(**cfg_a), inputs.small_workload(seed=5, **cfg_b)
    xa, xb = inputs.make_inputs(wa), inputs.make_inputs(wb)
    da = {k: xa[k].to(DEV) for k in ("Q", "K", "V")}
    db = {k: xb[k].to(DEV) for k in ("Q", "K", "V")}
    pa = lrsa.params_for(da["Q"], da["K"], sink=wa.S, lag=wa.L, topk=wa.K)
    pb = lrsa.params_for(db["Q"], db["K"], sink=wb.S, lag=wb.L, topk=wb.K)
    sa0, ia0 = lrsa.lrsa_score_select(pa, da["K"], da["V"])
    sb0, ib0 = lrsa.lrsa_score_select(pb, db["K"], db["V"])
    torch.cuda.synchronize()
    before = lrsa.score_poll_limit(64)      # a lost word is given up after 64 polls: keeps the test short
    try:
        st_a, st_b = torch.cuda.Stream(), torch.cuda.Stream()
        outs_a, outs_b = [], []
        for _ in range(8):
            with torch.cuda.stream(st_a):
                outs_a.append(lrsa.lrsa_score_select(pa, da["K"], da["V"]))
            with torch.cuda.stream(st_b):
                outs_b.append(lrsa.lrsa_score_select(pb, db["K"], db["V"]))
        torch.cuda.synchronize()
    finally:
        lrsa.score_poll_limit(before)
    for s_, i_ in outs_a:
        assert torch.equal(s_, sa0) and torch.equal(i_, ia0)
    for s_, i_ in outs_b:
        assert torch.equal(s_, sb0) and torch.equal(i_, ib0)
