"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, rejects bad arguments before touching the
device, and the routing helper follows Algorithm 1's normalise-and-assign
tail (same pins as the oracle's: the paper's score table and threshold
counts)."""
import ctypes as C
import os
import re

import pytest

from paper_2604_21026_amd import nvq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "nvq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nvq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = nvq.lib()
    names = declared_symbols()
    assert set(names) == set(nvq.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    L = nvq.lib()
    seen = {L.nvq_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert L.nvq_status_string(99).decode() == "unknown status"


def test_argument_validation_happens_before_any_launch():
    L = nvq.lib()
    a = 0x1000  # fake, aligned, never dereferenced: validation fails first
    assert L.nvq_pack_int4(None, 4, 32, 32, a, a, None) == 1
    assert L.nvq_pack_int4(a, 4, 48, 32, a, a, None) == 2
    assert L.nvq_pack_int4(a, 4, 64, 64, a, a, None) == 4
    assert L.nvq_pack_int4(a + 4, 4, 64, 32, a, a, None) == 3
    assert L.nvq_quant_act_i8(a, 1, 64, 16, a, a, a, None) == 1
    assert L.nvq_quant_act_i8(a, 33, 64, 0, a, a, a, None) == 2
    assert L.nvq_quant_act_i8(a, 1, 64, 0, a, a, None, None) == 1
    assert L.nvq_gemv_w4a16(a, a, 8, 40, a, 1, a, 0, None) == 2
    assert L.nvq_gemv_w4a16(a, a, 8, 64, a, 1, a, 7, None) == 1
    assert L.nvq_gemv_w4a16(a, a, 8, 64, a + 2, 1, a, 0, None) == 3
    assert L.nvq_gemv_w4a8(a, a, 8, 64, a, a, None, 0, 1, a, 0, None, None) == 1
    assert L.nvq_gemv_w4a8(a, a, 0, 64, a, a, a, 0, 1, a, 0, None, None) == 2
    assert L.nvq_stream_read(a, 24, a, None) == 2
    assert L.nvq_gemm_w4a16(a, a, 8, 64, None, 4, a, 0, None) == 1
    assert L.nvq_gemm_w4a16(a, a, 8, 64, a, 4, a, 3, None) == 1
    assert L.nvq_gemm_w4a16(a, a, 8, 48, a, 4, a, 0, None) == 2
    assert L.nvq_gemm_w4a16(a, a, 8, 64, a, 0, a, 0, None) == 2
    assert L.nvq_gemm_w4a16(a + 8, a, 8, 64, a, 4, a, 0, None) == 3
    assert L.nvq_dequant_bf16(a, a, 8, 40, a, None) == 2
    assert L.nvq_dequant_bf16(a, None, 8, 64, a, None) == 1


def test_decode_list_validation_and_workspace_size():
    L = nvq.lib()
    a = 0x1000
    arr = (nvq.Linear * 2)(nvq.Linear(a, a, 16, 64, a, a, 0, 0),
                           nvq.Linear(a, a, 16, 4096, a, a, 0, 1))
    need = L.nvq_decode_workspace_bytes(C.byref(arr), 2, 1, 0)
    assert need >= 4096 + 4 * 128 * 2 and need % 256 == 0
    need4 = L.nvq_decode_workspace_bytes(C.byref(arr), 2, 4, 32)
    assert need4 >= need + 3 * (4096 + 2 * 4 * 128) and need4 % 256 == 0
    assert L.nvq_decode_linears(C.byref(arr), 2, 1, 0, None, 0, None) == 6
    assert L.nvq_decode_linears(C.byref(arr), 2, 1, 0, a, 16, None) == 6
    arr[1].precision = 5
    assert L.nvq_decode_workspace_bytes(C.byref(arr), 2, 1, 0) == 0
    assert L.nvq_decode_linears(C.byref(arr), 2, 1, 0, a, 1 << 20, None) == 1
    assert L.nvq_decode_linears(C.byref(arr), 0, 1, 0, None, 0, None) == 0


def test_precision_from_scores_follows_the_papers_table():
    from tests.test_oracle_act_gemv import _golden
    scores, l1, counts = _golden()
    scores[1] = l1
    for tau, n16 in counts:
        assert sum(nvq.precision_from_scores(scores, tau)) == n16
    assert nvq.precision_from_scores(scores, 0.7) == [0] * 15 + [1]
    assert nvq.precision_from_scores([3.25] * 5, 1e-4, eps=1e-9) == [0] * 5
    assert nvq.precision_from_scores([61.0, 101.5, 142.0], 0.5) == [0, 1, 1]


def test_mcap_scores_follow_the_oracle():
    import numpy as np
    import oracle
    rng = np.random.default_rng(11)
    L, lens = 5, [3, 1, 7, 2]
    attn = rng.random((L, sum(lens))).astype(np.float32) * 10
    ffn = rng.random((L, sum(lens))).astype(np.float32) * 3
    got = nvq.mcap_scores(attn, ffn, lens)
    want = oracle.mcap_scores(attn.astype(np.float64), ffn.astype(np.float64), lens)
    assert np.allclose(got, want, rtol=1e-14, atol=0)
    lib = nvq.lib()
    a = attn.ctypes.data
    assert lib.nvq_mcap_scores(a, a, None, 1, 1, a) == 1
    bad = (C.c_int * 2)(3, 0)
    out = (C.c_double * 5)()
    assert lib.nvq_mcap_scores(a, a, bad, 2, 5, out) == 2
    assert lib.nvq_token_norms(None, 4, None, 0, 1, 0, a, None) == 1
    assert lib.nvq_token_norms(a, 4, None, 3, 1, 0, a, None) == 1
    assert lib.nvq_token_norms(a, 0, None, 0, 1, 0, a, None) == 2
    assert lib.nvq_token_norms(a, 4, None, 0, 1, 9, a, None) == 1


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        nvq.pack_int4(torch.zeros(4, 32))
