"""The walk for callers that cannot allocate (nvq_decode_linears_static: launches only, its
scratch memory a device array inside the library), called through the C ABI and checked against
nvq_decode_linears on the same lists: two calls in a row on the GPU's one scratch array, the
second with a smaller input and fewer tokens."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_21026_amd import nvq
from tests import np_ref
from tests.test_gpu_parity import DEV, block_with_transforms, model_entries, say

pytestmark = pytest.mark.gpu


def clone_outputs(entries):
    """The same list writing to buffers of its own (outputs and residual sums; an input that
    is another entry's output follows it)."""
    moved = {}

    def fresh(t):
        if t is None:
            return None
        if t.data_ptr() not in moved:
            moved[t.data_ptr()] = torch.zeros_like(t)
        return moved[t.data_ptr()]

    for e in entries:
        fresh(e["y"])
        fresh(e.get("h_out"))
    out = []
    for e in entries:
        c = dict(e)
        for k in ("y", "h_out"):
            if e.get(k) is not None:
                c[k] = moved[e[k].data_ptr()]
        for k in ("x", "x2"):
            if e.get(k) is not None and e[k].data_ptr() in moved:
                c[k] = moved[e[k].data_ptr()]
        out.append(c)
    return out


def test_static_walk_matches_the_workspace_walk_on_two_calls_in_a_row():
    # call 1: three tokens, one transformer block with its norms, residual add and SiLU-multiply
    # fused in (both walks run it as launches per phase: the same kernels, equal bits)
    big, _, _ = block_with_transforms(3, 2048, 512, 8192, 9800, (0, 1))
    big_s = clone_outputs(big)
    # call 2: one token, smaller layers, independent inputs (the workspace walk is the
    # persistent kernel: another fp32 summation order)
    small, _ = model_entries([(512, 512, 0), (128, 512, 0), (640, 512, 1), (96, 1408, 2)], (0, 1),
                             seed=9900)
    small_s = clone_outputs(small)
    say("static walk: call 1 (3 tokens, transforms), call 2 (1 token, smaller)")
    ref1 = nvq.DecodeList(big, 3, 0)
    ref1.run()
    ref2 = nvq.DecodeList(small, 1, 0)
    ref2.run()
    s1 = nvq.DecodeList(big_s, 3, 0)
    s2 = nvq.DecodeList(small_s, 1, 0)
    s1.run_static()
    s2.run_static()          # right behind it, same stream, same scratch array
    torch.cuda.synchronize()
    assert not ref2.timed_out()
    for a, b in zip(big, big_s):
        assert a["y"].data_ptr() != b["y"].data_ptr()
        assert float(b["y"].float().abs().max()) > 0
        assert torch.equal(a["y"], b["y"])
        if a.get("h_out") is not None:
            assert torch.equal(a["h_out"], b["h_out"])
    for a, b in zip(small, small_s):
        err = np_ref.rel_l2(b["y"].cpu().numpy(), a["y"].cpu().numpy().astype(np.float64))
        assert err < 1e-3 and err < 1e-5, err
    # and once more the other way round: the larger call after the smaller one
    for e in big_s:
        e["y"].zero_()
    s1.run_static()
    torch.cuda.synchronize()
    for a, b in zip(big, big_s):
        assert torch.equal(a["y"], b["y"])


def test_static_walk_refuses_what_its_scratch_does_not_hold():
    a = 0x10000
    arr = (nvq.Linear * 1)(nvq.Linear(a, a, 16, 65536, a, a + (1 << 24), 0, 0))
    # 32 tokens x 65536 inputs: 2 MiB of codes alone
    assert nvq.lib().nvq_decode_linears_static(C.byref(arr), 1, 32, 0, None) == 6
    assert nvq.lib().nvq_decode_linears_static(C.byref(arr), 1, 0, 0, None) == 2
    assert nvq.lib().nvq_decode_linears_static(None, 1, 1, 0, None) == 1
