"""Pins for the oracle's weight quantise + pack step (no GPU).

The paper fixes the block shape (32 weights -> 18 bytes = one fp16 scale plus
16 nibble bytes, 4.5 bits per weight) and the nibble centring at 8 (section
"Per-Layer Precision Dispatch and the W4A8 Path").  The scale rule absmax/7,
round-half-to-even and IEEE division are this build's readings; the hand
cases below use power-of-two scales so that every expected value can be
written down without running any code."""
import numpy as np
import pytest

import oracle
from paper_2604_21026_amd import synth
from tests import np_ref

S7 = 2.0 ** -7       # a scale that fp16 holds exactly; fp16 bits 0x2000


def _group(codes_times):
    """32 weights = multiples of 2^-7, with one element at 7 * 2^-7 so that
    absmax / 7 = 2^-7 exactly."""
    w = np.array(codes_times, np.float32) * np.float32(S7)
    assert w.shape == (32,)
    assert np.max(np.abs(w)) == np.float32(7 * S7)
    return w.reshape(1, 32)


def test_hand_case_layout_bytes_and_scale():
    lo = [j - 7 for j in range(15)] + [0]          # elements 0..15: -7..7, 0
    hi = [7 - j for j in range(15)] + [-1]         # elements 16..31: 7..-7, -1
    q, s = oracle.pack_int4(_group(lo + hi))
    assert s.tolist() == [[0x2000]]
    want = bytes.fromhex("F1E2D3C4B5A69788796A5B4C3D2E1F78")
    assert q.tobytes() == want


def test_hand_case_round_half_to_even():
    # value/scale: 2.5 -> 2, 3.5 -> 4, -0.5 -> 0, 0.5 -> 0, 1.5 -> 2, -2.5 -> -2,
    # -3.5 -> -4, 6.5 -> 6, -6.5 -> -6, 4.5 -> 4, 5.5 -> 6 (half-away would give 3, 1, ...)
    vals = [7, 2.5, 3.5, -0.5, 0.5, 1.5, -2.5, -3.5, 6.5, -6.5, 4.5, 5.5] + [0] * 20
    want = [7, 2, 4, 0, 0, 2, -2, -4, 6, -6, 4, 6] + [0] * 20
    q, s = oracle.pack_int4(_group(vals))
    assert s[0, 0] == 0x2000
    assert np_ref.unpack_codes(q)[0].tolist() == want


def test_negative_absmax_maps_to_minus_seven_not_minus_eight():
    vals = [-7] + [1] * 31
    q, _ = oracle.pack_int4(_group(vals))
    codes = np_ref.unpack_codes(q)[0]
    assert codes[0] == -7 and codes.min() == -7


def test_zero_group_gives_zero_scale_and_zero_codes():
    W = np.zeros((2, 64), np.float32)
    W[1, 40] = 0.5
    q, s = oracle.pack_int4(W)
    assert s[0].tolist() == [0, 0] and s[1, 0] == 0
    codes = np_ref.unpack_codes(q)
    assert not codes[0].any() and not codes[1, :32].any()
    assert q[0].tolist() == [0x88] * 32          # code 0 is stored as nibble 8
    assert codes[1, 40] == 7


def test_packed_size_is_4p5_bits_per_weight():
    for N, K in [(3, 32), (5, 2048), (7, 3072)]:
        W = synth.make_weight(1, N, K).numpy()
        q, s = oracle.pack_int4(W)
        assert q.nbytes + s.nbytes == N * K * 9 // 16 == synth.weight_bytes(N, K)
        assert (q.nbytes + s.nbytes) * 8 / (N * K) == 4.5


@pytest.mark.parametrize("N,K,seed", [(64, 2048, 11), (33, 3072, 12), (8, 14336, 13)])
def test_invariants_on_workload_distribution(N, K, seed):
    W = synth.make_weight(seed, N, K).numpy()
    q, s = oracle.pack_int4(W)
    codes = np_ref.unpack_codes(q)
    assert codes.min() >= -8 and codes.max() <= 7
    assert codes.min() >= -7                       # absmax/7 never produces -8
    sc = np.repeat(np_ref.half_bits_to_f64(s), 32, axis=1)
    err = np.abs(W.astype(np.float64) - codes * sc)
    assert np.all(err <= sc / 2 * (1 + 1e-6))
    # the absmax element of every group has |code| = 7
    Wg = np.abs(W).reshape(N, K // 32, 32)
    cg = np.abs(codes).reshape(N, K // 32, 32)
    am = Wg.argmax(axis=2)
    assert np.all(np.take_along_axis(cg, am[..., None], 2) == 7)


def test_scale_and_codes_against_numpy_float16_and_rint():
    W = synth.make_weight(21, 48, 4096).numpy()
    q, s = oracle.pack_int4(W)
    amax = np.abs(W).reshape(48, 128, 32).max(axis=2)
    s_np = (amax / np.float32(7)).astype(np.float16)
    assert np.array_equal(s, s_np.view(np.uint16))
    sf = np.repeat(s_np.astype(np.float32), 32, axis=1)
    c_np = np.clip(np.rint(W / sf), -8, 7).astype(np.int32)   # float32 divide, half-even
    assert np.array_equal(np_ref.unpack_codes(q), c_np)


def test_idempotent_on_its_own_dequantisation():
    W = synth.make_weight(31, 16, 2048).numpy()
    q, s = oracle.pack_int4(W)
    Wd = oracle.dequant_int4(q, s).astype(np.float32)    # code * scale is exact in fp32
    q2, s2 = oracle.pack_int4(Wd)
    assert np.array_equal(q, q2) and np.array_equal(s, s2)


def test_dequant_agrees_with_numpy_unpack_and_accepts_code_minus_eight():
    rng = np.random.default_rng(5)
    q = rng.integers(0, 256, (6, 48), dtype=np.uint8)      # every nibble incl. 0 (code -8)
    s = rng.integers(0x0400, 0x3c00, (6, 3)).astype(np.uint16)
    assert np.array_equal(oracle.dequant_int4(q, s), np_ref.dequant(q, s))
    assert np_ref.unpack_codes(q).min() == -8


def test_scale_overflow_is_reported():
    W = np.zeros((1, 32), np.float32)
    W[0, 3] = 7 * 70000.0
    with pytest.raises(oracle.OracleError):
        oracle.pack_int4(W)


def test_shape_errors():
    with pytest.raises(oracle.OracleError):
        oracle.pack_int4(np.zeros((2, 48), np.float32))


def test_dequant_bf16_is_the_library_rounding_of_the_exact_product():
    # code * scale is exact in binary32 (4 + 11 significand bits), so the dense bf16 weight is
    # torch's own float32 -> bfloat16 conversion of numpy's unpacked product: a library routine,
    # not the oracle's rounding code.  Random bytes cover every nibble (incl. code -8), scales
    # cover subnormal, ordinary and the largest finite fp16.
    import torch
    rng = np.random.default_rng(31)
    N, K = 24, 256
    q = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    s = rng.integers(0x0001, 0x7c00, (N, K // 32)).astype(np.uint16)
    s[0, 0], s[0, 1], s[0, 2] = 0x0001, 0x7bff, 0x0000
    got = oracle.dequant_bf16(q, s)
    exact = np_ref.unpack_codes(q).astype(np.float64) * np.repeat(s.view(np.float16).astype(np.float64), 32, axis=1)
    assert np.array_equal(exact.astype(np.float32).astype(np.float64), exact)     # exact in fp32
    want = torch.from_numpy(exact.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # ties to even, by hand: code +1 times scale 1 + 2^-8 (fp16 0x3C04) lies exactly between
    # bf16 1.0 (0x3F80) and 1 + 2^-7 (0x3F81) -> 0x3F80; scale 1 + 3 * 2^-8 (0x3C0C) lies between
    # 0x3F81 and 0x3F82 -> 0x3F82
    q1 = np.full((1, 16), 0x88, np.uint8)            # all codes 0
    q1[0, 0] = 0x89                                  # element 0: code +1
    assert oracle.dequant_bf16(q1, np.array([[0x3C04]], np.uint16))[0, 0] == 0x3F80
    assert oracle.dequant_bf16(q1, np.array([[0x3C0C]], np.uint16))[0, 0] == 0x3F82
