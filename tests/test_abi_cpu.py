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


def test_no_compressed_chunks_is_a_legal_noop_for_score_and_select():
    p = _params(n=16 + 2 * 64)      # sink + two chunks: Ns = 0
    L = lrsa.lib()
    assert lrsa.num_scored_chunks(p) == 0
    assert L.lrsa_score(ctypes.byref(p), None, None, None, None, 0, None) == 0
    assert L.lrsa_select(ctypes.byref(p), None, None, None, 0, None) == 0
    assert lrsa.workspace_bytes(p, binding.WS_SCORE) == 0


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2506_11498_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f
                assert "liblrsa_oracle" not in text and "lrsa_rows" not in text and "lrsa_ref" not in text, f
