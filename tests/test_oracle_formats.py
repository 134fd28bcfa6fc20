"""Pins for the oracle's own number-format conversions (no GPU).

The oracle converts fp16 and bf16 with its own bit code; numpy's float16 and
torch's bfloat16 are independent implementations of the same IEEE formats."""
import struct

import numpy as np
import torch

import oracle


def test_half_to_float_all_65536_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float32).view(np.uint32)
    L = oracle.lib()
    for b in range(65536):
        got = struct.unpack("<I", struct.pack("<f", L.orc_half_to_float(b)))[0]
        w = int(want[b])
        if (w & 0x7fffffff) > 0x7f800000:            # NaN: any NaN will do
            assert (got & 0x7fffffff) > 0x7f800000, hex(b)
        else:
            assert got == w, hex(b)


def _check_float_to_half(vals: np.ndarray):
    vals = vals.astype(np.float32)
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    L = oracle.lib()
    for v, w in zip(vals.tolist(), want.tolist()):
        got = L.orc_float_to_half(v)
        assert got == w, (v, hex(got), hex(w))


def test_float_to_half_random_and_ties():
    rng = np.random.default_rng(1)
    # normal range, subnormal range, underflow, overflow
    _check_float_to_half(rng.normal(0, 0.02, 20000) / 7)
    _check_float_to_half(rng.uniform(-7e4, 7e4, 5000))
    _check_float_to_half(rng.uniform(-1.3e-4, 1.3e-4, 5000))
    _check_float_to_half(rng.uniform(-2e-7, 2e-7, 5000))
    # exact ties between neighbouring halves: (h + h_next)/2 is exact in fp32
    h = rng.integers(0, 0x7bff, 5000).astype(np.uint16)
    a = h.view(np.float16).astype(np.float32)
    b = (h + 1).astype(np.uint16).view(np.float16).astype(np.float32)
    mid = (a + b) / np.float32(2)
    _check_float_to_half(mid)
    _check_float_to_half(-mid)
    # nudged just off the tie
    _check_float_to_half(np.nextafter(mid, np.float32(np.inf)))
    _check_float_to_half(np.nextafter(mid, np.float32(-np.inf)))
    # edges
    _check_float_to_half(np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 65536.0, 1e9,
                                   2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 2.0 ** -26,
                                   2.0 ** -14, np.inf, -np.inf], np.float32))


def test_bf16_round_trip_matches_torch():
    g = torch.Generator().manual_seed(3)
    x = torch.randn(20000, generator=g) * 5
    x[:10] = torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40,
                           65280.0, 0.99609375])
    want = x.to(torch.bfloat16).view(torch.int16).numpy().astype(np.uint16)
    L = oracle.lib()
    for v, w in zip(x.tolist(), want.tolist()):
        got = L.orc_float_to_bf16(v)
        assert got == w, (v, hex(got), hex(w))
        back = L.orc_bf16_to_float(got)
        assert struct.pack("<f", back) == struct.pack("<I", got << 16)
