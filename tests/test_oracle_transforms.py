"""Pins for the oracle's input transforms (RMSNorm, SiLU-multiply) and its one-step
double -> bf16 rounding.  The paper names the two kernels (kernel table) without restating
their formulas; the usual definitions are taken.  Pins: torch's own float64 routines with
a half-ulp bound, closed forms and invariants that a dropped term, a wrong power or a missing
rounding would break."""
import numpy as np
import torch

import oracle
from paper_2604_21026_amd import synth


def u16(t):
    return t.view(torch.int16).numpy().view(np.uint16)


def bf(u):
    return torch.from_numpy(u.view(np.int16)).view(torch.bfloat16)


def half_ulp(v):
    """Half a bf16 ulp at |v| (8 significand bits), float64."""
    e = np.floor(np.log2(np.maximum(np.abs(v), 1e-300)))
    return 2.0 ** (e - 7) / 2


def test_double_to_bf16_rounds_once():
    f = oracle.lib().orc_double_to_bf16
    assert f(1.0) == 0x3F80 and f(-2.5) == 0xC020
    assert f(1.0 + 2.0 ** -8) == 0x3F80                  # tie -> even
    assert f(1.0 + 3 * 2.0 ** -8) == 0x3F82              # tie -> even (up)
    # just above a tie: float32 rounding would land exactly on the tie and then go to even
    # (down); one-step rounding goes up
    assert f(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    assert f(1.0 + 2.0 ** -8 - 2.0 ** -40) == 0x3F80
    rng = np.random.default_rng(5)
    for v in rng.standard_normal(2000) * 10.0:
        got = float(bf(np.array([f(float(v))], np.uint16))[0])
        assert abs(got - v) <= half_ulp(v) * (1 + 1e-12)


def test_rms_norm_against_torch_float64_and_closed_forms():
    M, K = 3, 512
    x = synth.make_activation(41, M, K)
    gamma = (1.0 + 0.1 * torch.randn(K, generator=torch.Generator().manual_seed(7))).to(torch.bfloat16)
    eps = 1e-5
    out, h = oracle.rms_norm(u16(x), u16(gamma), eps)
    assert h is None
    want = torch.nn.functional.rms_norm(x.double(), (K,), gamma.double(), eps).numpy()
    got = bf(out).double().numpy()
    assert np.all(np.abs(got - want) <= half_ulp(want) * (1 + 1e-9))
    # a constant row c with eps = 0 normalises to sign(c): the output is gamma itself
    c = torch.full((1, K), -2.0).to(torch.bfloat16)
    out, _ = oracle.rms_norm(u16(c), u16(gamma), 0.0)
    assert np.array_equal(out[0], u16((-gamma).contiguous()))
    # scaling the input by a power of two changes nothing when eps = 0
    a, _ = oracle.rms_norm(u16(x), u16(gamma), 0.0)
    b, _ = oracle.rms_norm(u16((x.float() * 4).to(torch.bfloat16)), u16(gamma), 0.0)
    assert np.array_equal(a, b)
    # with gamma = 1 and eps = 0 the output has mean square 1 up to bf16 rounding
    ones = torch.ones(K).to(torch.bfloat16)
    o, _ = oracle.rms_norm(u16(x), u16(ones), 0.0)
    ms = (bf(o).double() ** 2).mean(dim=1)
    assert torch.all((ms - 1).abs() < 2e-3)
    # eps matters: a zero row stays zero (no 0/0), a tiny row is damped
    z = torch.zeros((1, K)).to(torch.bfloat16)
    o, _ = oracle.rms_norm(u16(z), u16(gamma), 1e-5)
    assert not o.any()


def test_rms_norm_residual_is_a_bf16_addition_first():
    M, K = 2, 256
    x = synth.make_activation(42, M, K)
    r = synth.make_activation(43, M, K)
    gamma = torch.ones(K).to(torch.bfloat16)
    out, h = oracle.rms_norm(u16(x), u16(gamma), 1e-6, res_bf16=u16(r))
    # torch adds bf16 tensors in float32 and rounds to nearest even: the library's addition
    assert np.array_equal(h, u16(x + r))
    # and the norm is the norm of that sum
    out2, _ = oracle.rms_norm(h, u16(gamma), 1e-6)
    assert np.array_equal(out, out2)


def test_silu_mul_against_torch_float64_and_closed_forms():
    M, K = 2, 1024
    g = synth.make_activation(44, M, K)
    u = synth.make_activation(45, M, K)
    out = oracle.silu_mul(u16(g), u16(u))
    want = (torch.nn.functional.silu(g.double()) * u.double()).numpy()
    got = bf(out).double().numpy()
    assert np.all(np.abs(got - want) <= half_ulp(want) * (1 + 1e-9))
    # silu(0) = 0; for large g silu(g) = g to double precision, so the result is the bf16 product
    g2 = torch.tensor([[0.0, 60.0, -60.0, 1.0]]).to(torch.bfloat16)
    u2 = torch.tensor([[3.0, 1.5, 2.0, 1.0]]).to(torch.bfloat16)
    o2 = bf(oracle.silu_mul(u16(g2), u16(u2))).float()[0]
    assert o2[0] == 0.0 and o2[1] == 90.0 and abs(float(o2[2])) < 1e-20
    assert o2[3] == torch.tensor(1.0 / (1.0 + np.exp(-1.0))).to(torch.bfloat16).float()
    # silu(g) - silu(-g) = g: with u = 1 the two outputs differ by g up to two roundings
    ones = torch.ones_like(g)
    a = bf(oracle.silu_mul(u16(g), u16(ones))).double()
    b = bf(oracle.silu_mul(u16((-g).contiguous()), u16(ones))).double()
    assert torch.all((a - b - g.double()).abs() <= (a.abs() + b.abs() + 1e-30) * 2.0 ** -8)


def test_walker_applies_the_transform_before_the_layer():
    M, N, K = 2, 24, 256
    W = synth.make_weight(46, N, K)
    q, s = oracle.pack_int4(W.numpy())
    x = synth.make_activation(47, M, K)
    r = synth.make_activation(48, M, K)
    gamma = (1.0 + 0.1 * torch.randn(K, generator=torch.Generator().manual_seed(8))).to(torch.bfloat16)
    for prec in (0, 1):
        e = dict(qweight=q, scales=s, x=u16(x), precision=prec, in_op=oracle.IN_RMSNORM,
                 x2=u16(r), gamma=u16(gamma), eps=1e-5)
        y = oracle.decode_linears([e], M)[0]
        xn, h = oracle.rms_norm(u16(x), u16(gamma), 1e-5, res_bf16=u16(r))
        assert np.array_equal(e["h"], h)
        y2 = oracle.decode_linears([dict(qweight=q, scales=s, x=xn, precision=prec)], M)[0]
        assert np.array_equal(y, y2)
        e = dict(qweight=q, scales=s, x=u16(x), precision=prec, in_op=oracle.IN_SILU_MUL, x2=u16(r))
        y = oracle.decode_linears([e], M)[0]
        y2 = oracle.decode_linears([dict(qweight=q, scales=s, x=oracle.silu_mul(u16(x), u16(r)),
                                         precision=prec)], M)[0]
        assert np.array_equal(y, y2)
