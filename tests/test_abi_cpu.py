"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, validates arguments before touching HIP, and its partition arithmetic agrees
with the oracle's."""
import ctypes
import os
import re

import pytest
import torch

import paper_2506_11498_amd as lrsa
from paper_2506_11498_amd import binding
from oracle import lrsa_ref as ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _params(**kw):
    base = dict(B=1, Hq=4, Hkv=2, n=1000, d=128, sink=16, lag=64, topk=16, dtype=torch.bfloat16)
    base.update(kw)
    B, Hq, Hkv, n, d = (base.pop(k) for k in ("B", "Hq", "Hkv", "n", "d"))
    return lrsa.make_params((B, Hq, n, d), (B, Hkv, n, d), (Hq * n * d, n * d, d, 1), (Hkv * n * d, n * d, d, 1), **base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lrsa.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lrsa_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    L = lrsa.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert L.lrsa_abi_version() == 1


def test_struct_layout_matches_header():
    # 13 int32/float fields then 6 int64: 52 bytes padded to 56, plus 48
    assert ctypes.sizeof(binding.LrsaParams) == 104
    assert binding.LrsaParams.q_stride.offset == 56


@pytest.mark.parametrize("n,S,L,lp", [(1024, 4, 128, 1), (4096, 16, 256, 1), (32768, 64, 1024, 1), (131072, 64, 2048, 1),
                                      (100, 7, 13, 1), (100, 7, 13, 2), (30, 0, 10, 1), (5, 16, 8, 1), (33, 1, 16, 1)])
def test_scored_chunks_match_oracle_partition(n, S, L, lp):
    p = _params(n=n, sink=S, lag=L, topk=2, local_prev=lp)
    assert lrsa.num_scored_chunks(p) == ref.partition(n, S, L, lp)["Ns"]


@pytest.mark.parametrize("kw,code", [
    (dict(Hq=3), -1), (dict(topk=65), -1), (dict(topk=0), -1), (dict(lag=1, topk=1), -1), (dict(sink=-1), -1),
    (dict(std_ddof=2), -1), (dict(local_prev=0), -1), (dict(n=0), -1), (dict(d=96), -2), (dict(dtype=torch.float16), -2),
    (dict(impl=7), -1),
])
def test_bad_params_are_rejected(kw, code):
    p = _params(**kw)
    with pytest.raises(lrsa.LrsaError) as e:
        lrsa.num_scored_chunks(p)
    assert e.value.code == code
    assert len(lrsa.lib().lrsa_last_error()) > 0
    assert lrsa.workspace_bytes(p, 0) == 0


def test_bad_strides_are_rejected():
    p = _params()
    p.q_stride[2] = 64          # rows overlap
    with pytest.raises(lrsa.LrsaError):
        lrsa.num_scored_chunks(p)
    p = _params()
    p.kv_stride[1] += 4         # breaks 16-byte alignment of bf16 rows
    with pytest.raises(lrsa.LrsaError):
        lrsa.num_scored_chunks(p)


def test_null_pointers_and_small_workspace_fail_before_any_gpu_work():
    L = lrsa.lib()
    p = _params()
    rc = L.lrsa_score(ctypes.byref(p), None, None, None, None, 0, None)
    assert rc == -1 and b"NULL" in L.lrsa_last_error()
    rc = L.lrsa_attn_fwd(ctypes.byref(p), None, None, None, None, None, None, None, 0, None)
    assert rc == -1
    rc = L.lrsa_attn_bwd(ctypes.byref(p), *([None] * 11), 0, None)
    assert rc == -1
    # non-null (fake, never dereferenced) pointers but a workspace that is too small
    fake = ctypes.c_void_p(4096)
    need = lrsa.workspace_bytes(p, binding.WS_SCORE)
    assert need > 0
    rc = L.lrsa_score(ctypes.byref(p), fake, fake, fake, ctypes.c_void_p(8192), need - 1, None)
    assert rc == -1 and b"workspace" in L.lrsa_last_error()
    rc = L.lrsa_score(ctypes.byref(p), fake, fake, fake, ctypes.c_void_p(8192 + 8), need, None)
    assert rc == -1 and b"aligned" in L.lrsa_last_error()
    rc = L.lrsa_select(ctypes.byref(p), None, None, None, 0, None)
    assert rc == -1
    fake = ctypes.c_void_p(4096)
    assert L.lrsa_check_idx(ctypes.byref(p), fake, None, None) == -1 and b"bad_rows" in L.lrsa_last_error()
    assert L.lrsa_check_idx(ctypes.byref(p), None, fake, None) == -1 and b"idx" in L.lrsa_last_error()


def test_no_compressed_chunks_is_a_legal_noop_for_score_and_select():
    p = _params(n=16 + 2 * 64)      # sink + two chunks: Ns = 0
    L = lrsa.lib()
    assert lrsa.num_scored_chunks(p) == 0
    assert L.lrsa_score(ctypes.byref(p), None, None, None, None, 0, None) == 0
    assert L.lrsa_select(ctypes.byref(p), None, None, None, 0, None) == 0
    assert lrsa.workspace_bytes(p, binding.WS_SCORE) == 0


def test_scoring_route_of_the_workloads_and_of_edge_shapes():
    """Host arithmetic: which kernels score a shape.  bf16 data with head_dim 128 and chunks of 64 to 4096 rows go
    to the one-read kernel; of the rest, few long chunks are cut into slices, chunks beyond 4096 rows take the long
    path and everything else one workgroup per chunk."""
    import torch
    from paper_2506_11498_amd import inputs

    def route(B, Hq, Hkv, d, n, L, K, S, dtype):
        p = lrsa.make_params((B, Hq, n, d), (B, Hkv, n, d), (Hq * n * d, n * d, d, 1), (Hkv * n * d, n * d, d, 1),
                             dtype=dtype, sink=S, lag=L, topk=K)
        return lrsa.score_route(p)

    want = {"C1": 1, "C2": 3, "C3": 3, "C4": 3, "C5": 3, "C6": 3}
    for name, r in want.items():
        w = inputs.WORKLOADS[name]
        assert route(w.B, w.Hq, w.Hkv, w.d, w.n, w.L, w.K, w.S, w.torch_dtype) == r, name
    bf, f32 = torch.bfloat16, torch.float32
    assert route(1, 2, 2, 128, 16 + 2 * 64, 64, 8, 16, bf) == 0                    # nothing is ever seen compressed
    assert route(1, 1, 1, 128, 8 + 3 * 4100 + 9, 4100, 17, 8, bf) == 4             # chunk beyond 4096 tokens
    assert route(1, 32, 32, 128, 16 + 16 * 512 + 100, 512, 100, 16, bf) == 3       # 64 streams, two parts per chunk
    assert route(1, 32, 32, 128, 16 + 16 * 512 + 100, 512, 100, 16, f32) == 1      # the one-read kernel is bf16 only
    assert route(1, 32, 32, 64, 16 + 16 * 512 + 100, 512, 100, 16, bf) == 1        # ... and head_dim 128 only
    assert route(1, 2, 2, 128, 16 + 6 * 1024 + 100, 1024, 256, 16, bf) == 3
    assert route(1, 2, 2, 128, 16 + 6 * 1024 + 100, 1024, 256, 16, f32) == 2       # 10 chunk units of 1024 rows
    assert route(1, 2, 2, 128, 16 + 6 * 640 + 100, 640, 256, 16, f32) == 1         # few units, but short chunks
    assert route(1, 2, 2, 128, 16 + 6 * 48 + 10, 48, 8, 16, bf) == 1               # chunks shorter than a wave of rows
    assert route(1, 2, 2, 128, 8 + 3 * 4096 + 9, 4096, 17, 8, bf) == 3             # the longest chunk: sixteen parts
    assert route(2, 80, 80, 128, 8 + 3 * 4096 + 9, 4096, 17, 8, bf) == 1           # 320 streams x 16 parts: too many
                                                                                   # workgroups between writer and reader


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2506_11498_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f
                assert "liblrsa_oracle" not in text and "lrsa_rows" not in text and "lrsa_ref" not in text, f


def test_inference_cache_calls_validate_on_the_host():
    """lrsa_cache_compress computes the new length and chunk count on the host and launches nothing when the
    tail is short; bad lengths, local_prev != 1 and null outputs fail before any GPU work."""
    L = lrsa.lib()
    p = _params(n=4096, sink=16, lag=256, topk=64)          # seq = capacity of the cache
    new_len, new_done = ctypes.c_int32(-1), ctypes.c_int32(-1)
    out = (ctypes.byref(new_len), ctypes.byref(new_done))
    # tail of 2*lag - 1 rows: nothing to do, no pointer is touched
    assert L.lrsa_cache_compress(ctypes.byref(p), None, None, None, 16 + 511, 0, *out, None) == 0
    assert (new_len.value, new_done.value) == (16 + 511, 0)
    # three compressed chunks and a tail of lag + 5 rows: still nothing to do
    assert L.lrsa_cache_compress(ctypes.byref(p), None, None, None, 16 + 3 * 64 + 261, 3, *out, None) == 0
    assert (new_len.value, new_done.value) == (16 + 3 * 64 + 261, 3)
    # a full tail needs the buffers
    assert L.lrsa_cache_compress(ctypes.byref(p), None, None, None, 16 + 512, 0, *out, None) == -1
    assert (new_len.value, new_done.value) == (16 + 64 + 256, 1)          # the arithmetic is done first
    assert L.lrsa_cache_compress(ctypes.byref(p), None, None, None, 5000, 0, *out, None) == -1    # beyond the capacity
    assert L.lrsa_cache_compress(ctypes.byref(p), None, None, None, 16 + 64 + 10, 1, *out, None) == -1   # too short for 1 chunk
    assert L.lrsa_cache_compress(ctypes.byref(p), None, None, None, 100, 0, None, None, None) == -1
    p2 = _params(n=4096, sink=16, lag=256, topk=64, local_prev=2)
    assert L.lrsa_cache_compress(ctypes.byref(p2), None, None, None, 16 + 512, 0, *out, None) == -2
    # decode attention: length and pointers
    assert L.lrsa_decode_attn(ctypes.byref(p), None, None, None, 0, None, None, None, 0, None) == -1
    assert L.lrsa_decode_attn(ctypes.byref(p), None, None, None, 10, None, None, None, 0, None) == -1
    assert b"NULL" in L.lrsa_last_error()
    assert lrsa.workspace_bytes(p, binding.WS_DECODE_ATTN) > 0
    # the condensed-cache variant asks for a larger attention workspace
    pc = _params(impl=binding.IMPL_COMPACT)
    assert lrsa.workspace_bytes(pc, binding.WS_ATTN_FWD) > lrsa.workspace_bytes(_params(), binding.WS_ATTN_FWD)


def test_binding_refuses_tensors_whose_layout_differs_from_the_params():
    """The ABI carries one stride triple for Q, O, dO, dQ and one for K, V, dK, dV; the binding refuses a
    tensor laid out differently (before any GPU work) instead of letting the kernels address it wrongly."""
    B, Hq, Hkv, n, d = 1, 4, 2, 16 + 5 * 32, 128
    Q = torch.zeros(B, Hq, n, d, dtype=torch.bfloat16)
    K = torch.zeros(B, Hkv, n, d, dtype=torch.bfloat16)
    p = lrsa.params_for(Q, K, sink=16, lag=32, topk=8)
    lse = torch.zeros(B, Hq, n)
    idx = torch.zeros(B, Hkv, lrsa.num_scored_chunks(p), 8, dtype=torch.int32)
    permuted = Q.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)          # same shape, other strides
    with pytest.raises(ValueError, match="stride"):
        lrsa.lrsa_attn_bwd(p, Q, K, K, Q, permuted, lse, idx)
    with pytest.raises(ValueError, match="dtype"):
        lrsa.lrsa_attn_fwd(p, Q, K, K.float(), idx)
    with pytest.raises(ValueError, match="shape"):
        lrsa.lrsa_attn_fwd(p, Q, K, K, idx[:, :, :-1])
    with pytest.raises(ValueError, match="contiguous"):
        lrsa.lrsa_attn_fwd(p, Q, K, K, idx, lse=torch.zeros(B, Hq, 2 * n)[:, :, ::2])
    with pytest.raises(ValueError, match="dtype"):
        lrsa.lrsa_select(p, torch.zeros(B, Hkv, idx.shape[2], 32, dtype=torch.float64))
