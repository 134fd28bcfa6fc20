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


def test_outputs_that_overlap_their_own_phase_are_refused():
    """Inside a phase nothing is ordered: an output over the phase's input, second operand,
    norm weights or a sibling's output is rejected before anything touches a device."""
    L = nvq.lib()
    q, s, x, y0, y1 = 0x10000, 0x20000, 0x30000, 0x40000, 0x50000
    out = (C.c_int32 * 64)()

    def describe(entries):
        arr = (nvq.Linear * len(entries))(*entries)
        return L.nvq_plan_describe(C.byref(arr), len(entries), 1, 0, 0, 256, out, 64)

    lin = lambda y, **kw: nvq.Linear(q, s, 64, 64, kw.get("x", x), y, kw.get("dt", 1), 0,
                                     kw.get("op", 0), 1e-5, kw.get("x2"), kw.get("gamma"),
                                     kw.get("h"))
    assert describe([lin(y0), lin(y1)]) == 0
    assert describe([lin(x)]) == 1                       # y in place over x
    assert describe([lin(x + 64)]) == 1                  # y over the second half of x (bf16 x 64)
    assert describe([lin(x + 128)]) == 0                 # just behind x
    assert describe([lin(y0), lin(y0 + 64)]) == 1        # sibling outputs overlap (bf16 y x 64)
    assert describe([lin(y0), lin(y0 + 128)]) == 0
    assert describe([lin(y0, dt=0), lin(y0 + 128)]) == 1  # the fp32 output is twice as long
    g, x2, h = 0x60000, 0x70000, 0x80000
    assert describe([lin(y0, op=1, x2=x2, gamma=g, h=h)]) == 0
    assert describe([lin(g, op=1, x2=x2, gamma=g, h=h)]) == 1   # y over the norm weights
    assert describe([lin(y0, op=1, x2=x2, gamma=g, h=x2)]) == 1  # residual sum over x2
    assert describe([lin(y0, op=1, x2=x2, gamma=g, h=y0)]) == 1  # residual sum over y
    assert describe([lin(x2, op=2, x2=x2)]) == 1                  # y over the SiLU operand
    # a later phase may of course overwrite an earlier phase's input: that is ordered
    assert describe([lin(y0), lin(x, x=y0)]) == 0
    ws = 0x100000
    arr = (nvq.Linear * 1)(lin(x))
    assert L.nvq_decode_linears(C.byref(arr), 1, 1, 0, ws, 1 << 24, None) == 1
    assert L.nvq_decode_status(None, None, C.byref(C.c_int())) == 1
    assert L.nvq_decode_status(ws, None, None) == 1


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
