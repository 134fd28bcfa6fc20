"""Pins for the oracle's activation quantisation, the two GEMVs, the layer
walker and the routing rule (no GPU).

Fixed by the paper: s = amax / 127, q = round(x / s) clamped to [-127, 127]
(appendix "F16 -> Q8 Activation Quantization"); int32 accumulation and the
identity  sum (nib - 8) q = sum nib q - 8 sum q  (section on the W4A8 path);
the routing rule and its threshold counts (Algorithm 1, tables of per-layer
scores and of the threshold ablation).  Given the codes, both products have a
plain definition: a float64 dense mat-vec on the dequantised operands."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2604_21026_amd import synth
from tests import np_ref


def bf16(vals):
    t = torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16)
    assert torch.equal(t.float(), torch.tensor(vals, dtype=torch.float32)), "not exact in bf16"
    return t.view(torch.int16).numpy().astype(np.uint16)


def act(seed, M, K, outliers=True):
    return synth.bf16_bits(synth.make_activation(seed, M, K, outliers)).numpy().astype(np.uint16)


# ---- activation quantisation -------------------------------------------------
def test_act_hand_case_unit_scale_half_to_even():
    vals = [127.0, 0.5, 1.5, 2.5, -127.0, 3.5, -0.5, -1.5, -2.5, 126.5, 125.5] + [0.0] * 21
    want = [127, 0, 2, 2, -127, 4, 0, -2, -2, 126, 126] + [0] * 21
    xq, xs, gs = oracle.quant_act_i8(bf16([vals]))
    assert xs.tolist() == [1.0]
    assert xq[0].tolist() == want
    assert gs.tolist() == [[sum(want)]]


def test_act_per_token_vs_per_group_scales():
    row = [127.0] + [1.0] * 31 + [-254.0] + [2.0] * 31      # two groups
    x = bf16([row])
    xq, xs, gs = oracle.quant_act_i8(x, act_group=0)
    assert xs.tolist() == [2.0]
    # 127/2 = 63.5 -> 64 (even), 1/2 = 0.5 -> 0, -254/2 = -127, 2/2 = 1
    assert xq[0].tolist() == [64] + [0] * 31 + [-127] + [1] * 31
    assert gs.tolist() == [[64, -127 + 31]]
    xq, xs, gs = oracle.quant_act_i8(x, act_group=32)
    assert xs.tolist() == [[1.0, 2.0]]
    assert xq[0].tolist() == [127] + [1] * 31 + [-127] + [1] * 31
    assert gs.tolist() == [[127 + 31, -127 + 31]]


def test_act_zero_token():
    x = np.zeros((2, 64), np.uint16)
    x[1, 5] = bf16([3.0])[0]
    xq, xs, gs = oracle.quant_act_i8(x)
    assert xs[0] == 0.0 and not xq[0].any() and not gs[0].any()
    assert xq[1, 5] == 127 and xq[1].sum() == 127


@pytest.mark.parametrize("K,group", [(2048, 0), (3072, 0), (14336, 0), (4096, 32)])
def test_act_invariants(K, group):
    x = act(7 + K, 3, K)
    xq, xs, gs = oracle.quant_act_i8(x, group)
    xf = np_ref.bf16_bits_to_f64(x)
    assert xq.min() >= -127 and xq.max() <= 127
    s = xs.astype(np.float64).reshape(3, -1)
    s_el = np.repeat(s, K // s.shape[1], axis=1)
    # q = RNE(fl(x / s)) with |x / s| <= 127 and a relative division error of 2^-24:
    # |x / s - q| <= 1/2 + 127 * 2^-24 = (1/2) (1 + 1.52e-5)
    assert np.all(np.abs(xf - xq * s_el) <= s_el / 2 * (1 + 2e-5))
    # the absmax element of every scale span maps to +-127
    span = K // s.shape[1]
    am = np.abs(xf).reshape(3, -1, span).argmax(axis=2)
    qa = np.abs(xq.astype(np.int32)).reshape(3, -1, span)
    assert np.all(np.take_along_axis(qa, am[..., None], 2) == 127)
    assert np.array_equal(gs, xq.astype(np.int32).reshape(3, K // 32, 32).sum(axis=2))
    # against numpy float32 division + rint
    xf32 = xf.astype(np.float32)
    s32 = (np.abs(xf32).reshape(3, -1, span).max(axis=2) / np.float32(127)).astype(np.float32)
    assert np.array_equal(xs.reshape(3, -1), s32)
    q_np = np.clip(np.rint(xf32 / np.repeat(s32, span, axis=1)), -127, 127).astype(np.int8)
    assert np.array_equal(xq, q_np)


# ---- W4A8 ---------------------------------------------------------------------
def test_w4a8_extreme_accumulators_brute_force():
    # nibble 0 = code -8 everywhere against q = -127 gives +32*8*127 = 32512 per block;
    # nibble 15 = code 7 against +127 gives 32*7*127 = 28448
    N, K = 2, 64
    q = np.zeros((N, K // 2), np.uint8)
    q[1, :] = 0xFF
    s = np.full((N, K // 32), 0x3c00, np.uint16)        # scale 1.0
    xq = np.full((1, K), -127, np.int8)
    y, acc = oracle.gemv_w4a8(q, s, xq, np.array([1.0], np.float32), want_acc=True)
    assert acc.tolist() == [[[32512, 32512], [-28448, -28448]]]
    assert y.tolist() == [[65024.0, -56896.0]]


def test_w4a8_acc_python_triple_loop_and_deferred_identity():
    rng = np.random.default_rng(9)
    N, K, M = 4, 64, 2
    q = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    s = np.full((N, K // 32), 0x3c00, np.uint16)
    _, acc = oracle.gemv_w4a8(q, s, xq, np.ones(M, np.float32), want_acc=True)
    for m in range(M):
        for n in range(N):
            for g in range(K // 32):
                t = 0
                for j in range(32):
                    byte = int(q[n, g * 16 + j % 16])
                    nib = (byte & 15) if j < 16 else (byte >> 4)
                    t += (nib - 8) * int(xq[m, g * 32 + j])
                assert acc[m, n, g] == t
    gs = xq.astype(np.int32).reshape(M, K // 32, 32).sum(axis=2)
    assert np.array_equal(oracle.w4a8_acc_deferred(q, xq, gs), acc)


@pytest.mark.parametrize("N,K,M,group", [(24, 2048, 1, 0), (10, 3072, 3, 0), (6, 14336, 2, 0),
                                         (12, 4096, 2, 32)])
def test_w4a8_output_is_float64_matvec_of_dequantised_operands(N, K, M, group):
    W = synth.make_weight(100 + N, N, K).numpy()
    q, s = oracle.pack_int4(W)
    x = act(200 + K, M, K)
    xq, xs, gs = oracle.quant_act_i8(x, group)
    y, acc = oracle.gemv_w4a8(q, s, xq, xs, group, want_acc=True)
    Wd = np_ref.dequant(q, s)
    xs_el = np.repeat(xs.astype(np.float64).reshape(M, -1), K // xs.reshape(M, -1).shape[1], axis=1)
    xd = xq.astype(np.float64) * xs_el
    assert np_ref.rel_l2(y, xd @ Wd.T) < 1e-12
    codes = np_ref.unpack_codes(q).reshape(N, K // 32, 32)
    acc_np = np.einsum("ngj,mgj->mng", codes, xq.astype(np.int32).reshape(M, K // 32, 32))
    assert np.array_equal(acc, acc_np)
    assert np.abs(acc).max() <= 32512
    assert np.array_equal(oracle.w4a8_acc_deferred(q, xq, gs), acc)


# ---- W4A16 --------------------------------------------------------------------
@pytest.mark.parametrize("N,K,M", [(24, 2048, 1), (10, 3072, 3), (6, 14336, 2)])
def test_w4a16_output_is_float64_matvec_and_close_to_unquantised(N, K, M):
    W = synth.make_weight(300 + N, N, K).numpy()
    q, s = oracle.pack_int4(W)
    x = act(400 + K, M, K)
    y = oracle.gemv_w4a16(q, s, x)
    xf = np_ref.bf16_bits_to_f64(x)
    assert np_ref.rel_l2(y, xf @ np_ref.dequant(q, s).T) < 1e-12
    # quantisation error bound against the unquantised product
    sc = np.repeat(np_ref.half_bits_to_f64(s), 32, axis=1)            # [N,K]
    bound = np.abs(xf) @ (sc / 2).T
    assert np.all(np.abs(y - xf @ W.astype(np.float64).T) <= bound * (1 + 1e-6))


def test_w4a16_hand_case():
    # one row, K = 32, scale 2 (fp16 0x4000); codes 0..15 low half, -8..7 high half:
    # nibble j in both halves of byte j
    q = np.array([[(j + 8 if j < 8 else j - 8 + 8) | (j << 4) for j in range(16)]], np.uint8)
    codes = np_ref.unpack_codes(q)[0].tolist()
    assert codes == [0, 1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 3, 4, 5, 6, 7] + list(range(-8, 8))
    x = bf16([[1.0] * 16 + [0.5] * 16])
    y = oracle.gemv_w4a16(q, np.array([[0x4000]], np.uint16), x)
    assert y.tolist() == [[2.0 * (2 * 28 + 0.5 * (-8))]]


def test_batch_rows_equal_batch_one():
    N, K, M = 9, 2048, 4
    q, s = oracle.pack_int4(synth.make_weight(55, N, K).numpy())
    x = act(56, M, K)
    xq, xs, _ = oracle.quant_act_i8(x)
    y8, acc = oracle.gemv_w4a8(q, s, xq, xs, want_acc=True)
    y16 = oracle.gemv_w4a16(q, s, x)
    for m in range(M):
        xq1, xs1, _ = oracle.quant_act_i8(x[m:m + 1])
        y1, a1 = oracle.gemv_w4a8(q, s, xq1, xs1, want_acc=True)
        assert np.array_equal(a1[0], acc[m]) and np.array_equal(y1[0], y8[m])
        assert np.array_equal(oracle.gemv_w4a16(q, s, x[m:m + 1])[0], y16[m])


# ---- walker ---------------------------------------------------------------------
def test_decode_linears_equals_standalone_calls_and_respects_precision():
    shapes = [(16, 64), (8, 64), (8, 64), (16, 64), (40, 64), (40, 64), (16, 160)]
    layers = []
    for i, (N, K) in enumerate(shapes):
        q, s = oracle.pack_int4(synth.make_weight(600 + i, N, K).numpy())
        layers.append(dict(qweight=q, scales=s, x=act(700 + K, 2, K, False), precision=i % 2))
    ys = oracle.decode_linears(layers, 2)
    for L, y in zip(layers, ys):
        if L["precision"] == 1:
            ref = oracle.gemv_w4a16(L["qweight"], L["scales"], L["x"])
            other = None
        else:
            xq, xs, _ = oracle.quant_act_i8(L["x"])
            ref = oracle.gemv_w4a8(L["qweight"], L["scales"], xq, xs)
            other = oracle.gemv_w4a16(L["qweight"], L["scales"], L["x"])
        assert np.array_equal(y, ref)
        if other is not None:
            assert not np.array_equal(y, other)


# ---- routing rule -------------------------------------------------------------
def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "per_layer_scores.txt")
    scores, counts, l1 = None, [], None
    for line in open(path):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "scores":
            scores = [float(v) for v in t[1:]]
        elif t[0] == "l1_exact":
            l1 = float(t[1])
        elif t[0] == "count":
            counts.append((float(t[1]), int(t[2])))
    return scores, l1, counts


def test_routing_rule_reproduces_the_papers_threshold_counts():
    scores, l1, counts = _golden()
    assert len(scores) == 16
    scores[1] = l1                                   # the caption's unrounded value
    for tau, n16 in counts:
        bits, shat = oracle.precision_from_scores(scores, tau)
        assert int(bits.sum()) == n16, tau
    bits, shat = oracle.precision_from_scores(scores, 0.7)
    assert bits.tolist() == [0] * 15 + [1]          # only the last layer keeps W4A16
    assert np.allclose(shat, scores)                 # already normalised: min 0, max 1


def test_routing_normalisation_tie_and_degenerate_case():
    raw = np.array([61.0, 101.5, 142.0, 117.7])      # min-max: 0, 0.5, 1, 0.7
    bits, shat = oracle.precision_from_scores(raw, 0.5)
    assert shat.tolist() == [0.0, 0.5, 1.0, (117.7 - 61.0) / 81.0]
    assert bits.tolist() == [0, 1, 1, 1]             # a score equal to tau takes W4A16
    bits, shat = oracle.precision_from_scores(np.full(5, 3.25), 0.0001, eps=1e-9)
    assert bits.tolist() == [0] * 5 and not shat.any()
