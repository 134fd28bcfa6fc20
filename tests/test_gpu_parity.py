"""GPU parity: every entry point of libnvq, called through the C ABI, against
the CPU oracle on the same seeded inputs.

Bars: packed int4 bytes, fp16 scale bits, int8 activation codes, activation
scales, block sums and W4A8 int32 accumulators are bit-exact; floating-point
outputs are within 1e-3 relative L2 of the float64 oracle (fp32 accumulation;
the observed error is around 1e-6)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_21026_amd import nvq, synth
from tests import np_ref

pytestmark = pytest.mark.gpu

TOL = 1e-3
DEV = "cuda"


def say(*a):
    print(*a, flush=True)


def u16(t):
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


def packed(seed, N, K):
    W = synth.make_weight(seed, N, K)
    q, s = oracle.pack_int4(W.numpy())
    return W, q, s


def to_dev_packed(q, s):
    return (torch.from_numpy(q).to(DEV), torch.from_numpy(s.view(np.int16)).to(DEV))


def act(seed, M, K, outliers=True):
    return synth.make_activation(seed, M, K, outliers)


# ---- a1 pack -----------------------------------------------------------------
@pytest.mark.parametrize("N,K", [(5, 32), (64, 2048), (33, 3072), (257, 4096), (7, 14336),
                                 (1, 64), (1031, 1024)])
def test_pack_int4_bit_exact(N, K):
    say("pack", N, K)
    W, q_ref, s_ref = packed(1000 + N, N, K)
    q, s = nvq.pack_int4(W.to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(u16(s), s_ref)


def test_pack_int4_edge_values():
    say("pack edge")
    W = torch.zeros(4, 64)
    S7 = 2.0 ** -7
    W[0, :12] = torch.tensor([7, 2.5, 3.5, -0.5, 0.5, 1.5, -2.5, -3.5, 6.5, -6.5, 4.5, 5.5]) * S7
    W[1, 40] = 0.5                      # one zero group, one single-spike group
    W[2, :32] = 1e-7                    # scale in the fp16 subnormal range
    W[2, 32:] = -3e-6
    W[3, 5] = 7 * 65504.0               # largest finite fp16 scale
    q_ref, s_ref = oracle.pack_int4(W.numpy())
    q, s = nvq.pack_int4(W.to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(u16(s), s_ref)
    assert np_ref.unpack_codes(q.cpu().numpy())[0, :12].tolist() == [7, 2, 4, 0, 0, 2, -2, -4, 6, -6, 4, 6]


# ---- prefill path: dense bf16 weights ------------------------------------------
@pytest.mark.parametrize("N,K", [(3, 32), (70, 2048), (257, 4096), (5, 14336), (1031, 1024)])
def test_dequant_bf16_bit_exact(N, K):
    say("dequant", N, K)
    _, q, s = packed(1500 + N, N, K)
    qd, sd = to_dev_packed(q, s)
    out = nvq.dequant_bf16(qd, sd)
    torch.cuda.synchronize()
    assert np.array_equal(u16(out), oracle.dequant_bf16(q, s))


def test_dequant_bf16_every_nibble_and_extreme_scales():
    say("dequant extremes")
    rng = np.random.default_rng(19)
    N, K = 33, 1024
    q = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)      # includes nibble 0 = code -8
    s = rng.integers(0x0000, 0x7c00, (N, K // 32)).astype(np.uint16)   # subnormal .. 65504
    s[0, :4] = [0x0000, 0x0001, 0x7bff, 0x3c04]
    qd, sd = to_dev_packed(q, s)
    out = nvq.dequant_bf16(qd, sd)
    torch.cuda.synchronize()
    assert np.array_equal(u16(out), oracle.dequant_bf16(q, s))


# ---- a2 activation quantisation ----------------------------------------------
@pytest.mark.parametrize("M,K,group", [(1, 32, 0), (1, 2048, 0), (3, 3072, 0), (1, 4096, 0),
                                       (2, 8192, 0), (1, 14336, 0), (32, 4096, 0),
                                       (1, 4096, 32), (4, 14336, 32), (2, 96, 32)])
def test_quant_act_bit_exact(M, K, group):
    say("quant", M, K, group)
    x = act(2000 + K + M, M, K)
    xq_r, xs_r, gs_r = oracle.quant_act_i8(u16(x), group)
    xq, xs, gs = nvq.quant_act_i8(x.to(DEV), group)
    torch.cuda.synchronize()
    assert np.array_equal(xq.cpu().numpy(), xq_r)
    assert np.array_equal(xs.cpu().numpy().view(np.uint32), xs_r.view(np.uint32))
    assert np.array_equal(gs.cpu().numpy(), gs_r)


def test_quant_act_edge_values():
    say("quant edge")
    x = torch.zeros(3, 64)
    x[1, :11] = torch.tensor([127.0, 0.5, 1.5, 2.5, -127.0, 3.5, -0.5, -1.5, -2.5, 126.5, 125.5])
    x[2, 40] = -3.0
    xb = x.to(torch.bfloat16)
    for group in (0, 32):
        xq_r, xs_r, gs_r = oracle.quant_act_i8(u16(xb), group)
        xq, xs, gs = nvq.quant_act_i8(xb.to(DEV), group)
        torch.cuda.synchronize()
        assert np.array_equal(xq.cpu().numpy(), xq_r)
        assert np.array_equal(xs.cpu().numpy(), xs_r)
        assert np.array_equal(gs.cpu().numpy(), gs_r)
    assert xq_r[1, :11].tolist() == [127, 0, 2, 2, -127, 4, 0, -2, -2, 126, 126]


# ---- a3 W4A8 -------------------------------------------------------------------
W4A8_CASES = [
    # N, K, M, act_group: every lane/row decomposition of the batch-1 kernel, ragged row
    # tails, more rows than one grid pass, the generic kernel (M > 1, K > 16384)
    (3, 32, 1, 0), (37, 1024, 1, 0), (70, 2048, 1, 0), (45, 2080, 1, 0), (29, 3072, 1, 0),
    (61, 4096, 1, 0), (19, 6144, 1, 0), (23, 8192, 1, 0), (11, 10240, 1, 0), (9, 12288, 1, 0),
    (13, 14336, 1, 0), (7, 16384, 1, 0), (5, 16416, 1, 0),
    (20011, 2048, 1, 0), (9003, 4096, 1, 0), (2501, 14336, 1, 0), (3000, 3072, 1, 0),
    (33, 4096, 1, 32), (21, 14336, 1, 32), (18, 3072, 1, 32),
    (40, 4096, 2, 0), (40, 4096, 4, 0), (17, 3072, 5, 0), (24, 14336, 8, 0), (12, 2048, 32, 0),
    (20, 4096, 3, 32),
    # matrix-core kernel (2 <= M <= 32, K % 128 == 0): one and two token tiles, ragged row
    # and token tails, fewer K columns than waves, 1 / 2 / 4 row tiles per workgroup
    (5, 128, 2, 0), (100, 4096, 16, 0), (70, 3072, 17, 0), (33, 14336, 32, 0), (16, 512, 9, 0),
    (16400, 2048, 8, 0), (33000, 1024, 24, 0),
]


@pytest.mark.parametrize("N,K,M,group", W4A8_CASES)
def test_gemv_w4a8_acc_bit_exact_and_output(N, K, M, group):
    say("w4a8", N, K, M, group)
    _, q, s = packed(3000 + N, N, K)
    x = act(3100 + K, M, K)
    xq_r, xs_r, gs_r = oracle.quant_act_i8(u16(x), group)
    y_r, acc_r = oracle.gemv_w4a8(q, s, xq_r, xs_r, group, want_acc=True)
    qd, sd = to_dev_packed(q, s)
    xq, xs, gs = nvq.quant_act_i8(x.to(DEV), group)
    y, acc = nvq.gemv_w4a8(qd, sd, xq, xs, gs, group, want_acc=True)
    y2 = nvq.gemv_w4a8(qd, sd, xq, xs, gs, group)            # the non-debug kernel
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_r)
    assert np_ref.rel_l2(y.cpu().numpy(), y_r) < TOL
    assert torch.equal(y, y2)
    assert np_ref.rel_l2(y.cpu().numpy(), y_r) < 1e-5        # what fp32 accumulation gives


@pytest.mark.parametrize("M", [1, 20])
def test_gemv_w4a8_accepts_every_nibble_and_extreme_codes(M):
    say("w4a8 extremes", M)
    rng = np.random.default_rng(17)
    N, K = 50, 4096
    q = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)      # includes nibble 0 = code -8
    q[0, :] = 0x00
    q[1, :] = 0xFF
    s = rng.integers(0x1400, 0x2c00, (N, K // 32)).astype(np.uint16)
    xq = rng.integers(-127, 128, (M, K)).astype(np.int8)
    xq[0, :64] = -127
    xq[M - 1, 64:128] = 127
    xs = np.linspace(0.03125, 0.0625, M).astype(np.float32)
    gs = xq.astype(np.int32).reshape(M, K // 32, 32).sum(axis=2).astype(np.int32)
    y_r, acc_r = oracle.gemv_w4a8(q, s, xq, xs, want_acc=True)
    assert acc_r.max() == 32512
    qd, sd = to_dev_packed(q, s)
    y, acc = nvq.gemv_w4a8(qd, sd, torch.from_numpy(xq).to(DEV), torch.from_numpy(xs).to(DEV),
                           torch.from_numpy(gs).to(DEV), want_acc=True)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_r)
    assert np_ref.rel_l2(y.cpu().numpy(), y_r) < TOL


def test_batched_w4a8_rows_equal_the_single_token_results():
    say("w4a8 batch rows")
    # the matrix-core kernel and the batch-1 kernel compute the same int32 accumulators
    N, K, M = 48, 4096, 19
    _, q, s = packed(3500, N, K)
    x = act(3501, M, K).to(DEV)
    qd, sd = to_dev_packed(q, s)
    xq, xs, gs = nvq.quant_act_i8(x, 0)
    y, acc = nvq.gemv_w4a8(qd, sd, xq, xs, gs, 0, want_acc=True)
    for m in (0, 7, 16, 18):
        y1, acc1 = nvq.gemv_w4a8(qd, sd, xq[m:m + 1].contiguous(), xs[m:m + 1].contiguous(),
                                 gs[m:m + 1].contiguous(), 0, want_acc=True)
        torch.cuda.synchronize()
        assert torch.equal(acc[m], acc1[0])
        assert np_ref.rel_l2(y[m].cpu().numpy(), y1[0].cpu().numpy()) < 1e-5


# ---- a4 W4A16 ------------------------------------------------------------------
W4A16_CASES = [(n, k, m) for (n, k, m, g) in W4A8_CASES if g == 0]


@pytest.mark.parametrize("N,K,M", W4A16_CASES)
def test_gemv_w4a16_output(N, K, M):
    say("w4a16", N, K, M)
    _, q, s = packed(4000 + N, N, K)
    x = act(4100 + K, M, K)
    y_r = oracle.gemv_w4a16(q, s, u16(x))
    qd, sd = to_dev_packed(q, s)
    y = nvq.gemv_w4a16(qd, sd, x.to(DEV))
    torch.cuda.synchronize()
    err = np_ref.rel_l2(y.cpu().numpy(), y_r)
    say("  rel_l2", err)
    assert err < TOL and err < 1e-5
    # per output (a norm over the whole output would let one row lose a whole group
    # unnoticed): every product code * scale * x is exact in fp32, so the GPU differs from
    # the float64 sum only by the roundings of its partial sums.  The kernel adds 136 to
    # every code and takes 136 * sum(x) away again, so a partial sum inside a group is at
    # most 279 * sum_j |x_j|; a few roundings of 2^-24 of that per group:
    sw = np_ref.half_bits_to_f64(s)                                               # [N][G]
    xa = np.abs(np_ref.bf16_bits_to_f64(u16(x))).reshape(M, K // 32, 32).sum(axis=2)   # [M][G]
    bound = 4 * 279 * 2.0 ** -24 * (xa @ sw.T)                                    # [M][N]
    diff = np.abs(y.cpu().numpy().astype(np.float64) - y_r)
    assert (diff <= bound + 1e-30).all(), float((diff / (bound + 1e-30)).max())


@pytest.mark.parametrize("M", [1, 20])
def test_gemv_w4a16_accepts_every_nibble(M):
    say("w4a16 nibbles", M)
    rng = np.random.default_rng(18)
    N, K = 40, 3072
    q = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    s = rng.integers(0x1400, 0x2c00, (N, K // 32)).astype(np.uint16)
    x = act(77, M, K)
    y_r = oracle.gemv_w4a16(q, s, u16(x))
    qd, sd = to_dev_packed(q, s)
    y = nvq.gemv_w4a16(qd, sd, x.to(DEV))
    torch.cuda.synchronize()
    assert np_ref.rel_l2(y.cpu().numpy(), y_r) < TOL


@pytest.mark.parametrize("prec", [nvq.W4A8, nvq.W4A16])
def test_bf16_output_is_the_rounded_fp32_output(prec):
    say("bf16 out", prec)
    N, K = 100, 4096
    _, q, s = packed(5000, N, K)
    x = act(5001, 1, K).to(DEV)
    qd, sd = to_dev_packed(q, s)
    if prec == nvq.W4A16:
        y32 = nvq.gemv_w4a16(qd, sd, x)
        y16 = nvq.gemv_w4a16(qd, sd, x, out_dtype=torch.bfloat16)
    else:
        xq, xs, gs = nvq.quant_act_i8(x)
        y32 = nvq.gemv_w4a8(qd, sd, xq, xs, gs)
        y16 = nvq.gemv_w4a8(qd, sd, xq, xs, gs, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(y16, y32.to(torch.bfloat16))


# ---- a5 walker -------------------------------------------------------------------
def tiny_model_entries(M, seed=6000, hidden=256, kv=64, ffn=704, blocks=3, bits=(0, 1, 0)):
    """Three transformer-block-shaped groups of seven linears; K = 256 and 704
    (22 groups: a ragged lane tail)."""
    entries, host = [], []
    for b in range(blocks):
        xs = [act(seed + 10 * b + p, M, k, True) for p, k in enumerate([hidden, hidden, hidden, ffn])]
        shapes = [(hidden, hidden, 0), (kv, hidden, 0), (kv, hidden, 0), (hidden, hidden, 1),
                  (ffn, hidden, 2), (ffn, hidden, 2), (hidden, ffn, 3)]
        for slot, (N, K, p) in enumerate(shapes):
            _, q, s = packed(seed + 100 * b + slot, N, K)
            host.append(dict(qweight=q, scales=s, x=u16(xs[p]), precision=bits[b]))
            qd, sd = to_dev_packed(q, s)
            entries.append(dict(qweight=qd, scales=sd, x=None, xkey=(b, p), xhost=xs[p],
                                y=torch.zeros((M, N), dtype=torch.float32, device=DEV),
                                precision=bits[b]))
    # entries of one phase must share one device buffer (the walker keys on the pointer)
    bufs = {}
    for e in entries:
        if e["xkey"] not in bufs:
            bufs[e["xkey"]] = e["xhost"].to(DEV)
        e["x"] = bufs[e["xkey"]]
    return entries, host


@pytest.mark.parametrize("M,group", [(1, 0), (1, 32), (3, 0)])
def test_decode_linears_matches_oracle_walker_and_standalone_calls(M, group):
    say("walker", M, group)
    entries, host = tiny_model_entries(M)
    ys_ref = oracle.decode_linears(host, M, group)
    nvq.decode_linears(entries, M, group)
    torch.cuda.synchronize()
    for e, h, y_r in zip(entries, host, ys_ref):
        got = e["y"].cpu().numpy()
        assert np_ref.rel_l2(got, y_r) < TOL
        # same result (up to fp32 summation order) as the standalone entry point
        if e["precision"] == nvq.W4A16:
            alone = nvq.gemv_w4a16(e["qweight"], e["scales"], e["x"])
            other = None
        else:
            xq, xs, gs = nvq.quant_act_i8(e["x"], group)
            alone = nvq.gemv_w4a8(e["qweight"], e["scales"], xq, xs, gs, group)
            other = nvq.gemv_w4a16(e["qweight"], e["scales"], e["x"])
        assert np_ref.rel_l2(e["y"].cpu().numpy(), alone.cpu().numpy()) < 1e-5
        if other is not None:                      # the precision bit was respected
            assert np_ref.rel_l2(e["y"].cpu().numpy(), other.cpu().numpy()) > 1e-4


def test_decode_linears_runs_in_order_on_chained_buffers():
    say("walker chain")
    # entry 1 reads what entry 0 wrote (bf16 output feeding the next input)
    M, K0, N0, N1 = 1, 2048, 4096, 512
    _, q0, s0 = packed(7000, N0, K0)
    W1 = synth.make_weight(7001, N1, N0)
    q1, s1 = oracle.pack_int4(W1.numpy())
    x0 = act(7002, M, K0)
    q0d, s0d = to_dev_packed(q0, s0)
    q1d, s1d = to_dev_packed(q1, s1)
    mid = torch.zeros((M, N0), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((M, N1), dtype=torch.float32, device=DEV)
    for p0, p1 in [(1, 0), (0, 1)]:
        mid.zero_(); out.zero_()
        nvq.decode_linears([dict(qweight=q0d, scales=s0d, x=x0.to(DEV), y=mid, precision=p0),
                            dict(qweight=q1d, scales=s1d, x=mid, y=out, precision=p1)], M)
        torch.cuda.synchronize()
        # oracle on the GPU's own intermediate (bf16 rounding of entry 0 is checked above)
        mid_h = u16(mid)
        ys = oracle.decode_linears([dict(qweight=q1, scales=s1, x=mid_h, precision=p1)], M)
        assert np_ref.rel_l2(out.cpu().numpy(), ys[0]) < TOL
        y0 = oracle.decode_linears([dict(qweight=q0, scales=s0, x=u16(x0), precision=p0)], M)[0]
        assert np_ref.rel_l2(mid.float().cpu().numpy(), y0) < 4e-3   # bf16 output rounding


def test_measurement_helpers():
    say("stream helpers")
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros_like(src)
    sink = torch.zeros(1, dtype=torch.int64, device=DEV)
    nvq.stream_copy(dst, src)
    nvq.stream_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    w = src.cpu().numpy().view(np.uint32).reshape(-1, 4)
    want = int((w[:, 0] ^ w[:, 1] ^ w[:, 2] ^ w[:, 3]).astype(np.uint64).sum())
    # per-lane sums wrap at 32 bits before the 64-bit atomic; compare modulo 2^32
    assert int(sink.item()) % (1 << 32) == want % (1 << 32)


# ---- persistent streaming walker (batch 1) ------------------------------------------
def model_entries(shapes_per_block, bits, M=1, seed=8000):
    """shapes_per_block: list of (N, K, phase-in-block); one x buffer per (block, phase)."""
    entries, host = [], []
    for b, bit in enumerate(bits):
        bufs = {}
        for slot, (N, K, p) in enumerate(shapes_per_block):
            if p not in bufs:
                xh = act(seed + 50 * b + p, M, K)
                bufs[p] = (xh, xh.to(DEV))
            _, q, s = packed(seed + 100 * b + slot, N, K)
            qd, sd = to_dev_packed(q, s)
            entries.append(dict(qweight=qd, scales=sd, x=bufs[p][1], precision=bit,
                                y=torch.zeros((M, N), dtype=torch.float32, device=DEV)))
            host.append(dict(qweight=q, scales=s, x=u16(bufs[p][0]), precision=bit))
    return entries, host


STREAM_MODELS = {
    # llama-1b block shapes, two blocks, one of each precision
    "1b": ([(2048, 2048, 0), (512, 2048, 0), (512, 2048, 0), (2048, 2048, 1),
            (8192, 2048, 2), (8192, 2048, 2), (2048, 8192, 3)], (0, 1)),
    # ragged: rows that do not divide over the waves, K with a partial last chunk (G = 66, 98)
    "ragged": ([(1000, 2112, 0), (37, 2112, 0), (3, 2112, 1), (2500, 3136, 2), (777, 3136, 2),
                (64, 14336, 3)], (1, 0, 0)),
    # 8b block shapes, one W4A8 block
    "8b": ([(4096, 4096, 0), (1024, 4096, 0), (1024, 4096, 0), (4096, 4096, 1),
            (14336, 4096, 2), (14336, 4096, 2), (4096, 14336, 3)], (0,)),
    # llama-3b block shapes (rows of 96 groups go to the waves in pairs), one block of
    # each precision; in the third, layers with an odd number of rows (no pairs there)
    "3b": ([(3072, 3072, 0), (1024, 3072, 0), (1024, 3072, 0), (3072, 3072, 1),
            (8192, 3072, 2), (8192, 3072, 2), (3072, 8192, 3)], (0, 1)),
    "3b odd": ([(3071, 3072, 0), (1024, 3072, 0), (8190, 3072, 1), (12294, 3072, 1),
                (2, 3072, 2)], (1, 0)),
}


@pytest.mark.parametrize("name,group,ordered", [("1b", 0, False), ("1b", 0, True),
                                                ("ragged", 0, False), ("ragged", 32, True),
                                                ("8b", 0, False), ("8b", 32, False),
                                                ("8b", 0, True),
                                                ("3b", 0, False), ("3b", 0, True),
                                                ("3b", 32, False), ("3b odd", 0, False)])
def test_streaming_plan_matches_oracle_on_repeated_runs(name, group, ordered):
    say("stream plan", name, group, ordered)
    shapes, bits = STREAM_MODELS[name]
    entries, host = model_entries(shapes, bits)
    ys_ref = oracle.decode_linears(host, 1, group)
    dl = nvq.DecodeList(entries, 1, group, ordered=ordered)
    info = dl.plan_info()
    say("  plan", info)
    assert info["streaming"], "batch-1 walk should use the persistent kernel"
    # independent buffers: no phase has to wait unless ordering is forced
    assert info["waits"] == (info["phases"] - 1 if ordered else 0)
    for rep in range(3):
        for e in entries:
            e["y"].zero_()
        dl.run_plan()
        assert not dl.plan_timed_out()
        for e, y_r in zip(entries, ys_ref):
            err = np_ref.rel_l2(e["y"].cpu().numpy(), y_r)
            assert err < TOL, (rep, err)
            assert err < 1e-5, (rep, err)
    dl.close()


@pytest.mark.parametrize("seed", range(4))
def test_streaming_plan_of_random_lists_matches_oracle(seed):
    """Random phases (1 to 3 layers on one input; rows from 1 to 9000; K with whole, ragged and
    one-and-a-half-chunk rows), both precisions, with and without forced ordering."""
    rng = np.random.default_rng(7300 + seed)
    entries, host = [], []
    for ph in range(int(rng.integers(4, 14))):
        K = int(rng.choice([96, 1024, 2048, 2112, 3072, 4096, 8192]))
        xh = act(7400 + 100 * seed + ph, 1, K)
        xd = xh.to(DEV)
        bit = int(rng.integers(0, 2))
        for k in range(int(rng.integers(1, 4))):
            N = int(rng.choice([1, 2, 7, 40, 96, 511, 1024, 3072, 4097, 9000]))
            _, q, s = packed(7500 + 1000 * seed + 10 * ph + k, N, K)
            qd, sd = to_dev_packed(q, s)
            entries.append(dict(qweight=qd, scales=sd, x=xd, precision=bit,
                                y=torch.zeros((1, N), dtype=torch.float32, device=DEV)))
            host.append(dict(qweight=q, scales=s, x=u16(xh), precision=bit))
    ordered = bool(seed & 1)
    say("stream plan, random list", seed, len(entries), "layers, ordered", ordered)
    ys_ref = oracle.decode_linears(host, 1, 0)
    dl = nvq.DecodeList(entries, 1, 0, ordered=ordered)
    assert dl.plan_info()["streaming"]
    for rep in range(2):
        for e in entries:
            e["y"].zero_()
        dl.run_plan()
        assert not dl.plan_timed_out()
        for i, (e, y_r) in enumerate(zip(entries, ys_ref)):
            err = np_ref.rel_l2(e["y"].cpu().numpy(), y_r)
            # (a handful of outputs can be small against their terms: the bar only)
            assert err < (1e-5 if y_r.size >= 96 else TOL), (rep, i, err)
    dl.close()


def test_streaming_plan_of_many_tiny_phases():
    """300 independent layers of 40 rows: nearly every wave has no rows in more than 255 phases
    in a row (the skip table's cap), a few work in one phase in a hundred."""
    say("stream plan, 300 tiny phases")
    entries, host = [], []
    for i in range(300):
        N, K = 40, 2048
        xh = act(9100 + i, 1, K)
        _, q, s = packed(9500 + i, N, K)
        qd, sd = to_dev_packed(q, s)
        entries.append(dict(qweight=qd, scales=sd, x=xh.to(DEV), precision=i % 2,
                            y=torch.zeros((1, N), dtype=torch.float32, device=DEV)))
        host.append(dict(qweight=q, scales=s, x=u16(xh), precision=i % 2))
    ys_ref = oracle.decode_linears(host, 1, 0)
    dl = nvq.DecodeList(entries, 1, 0)
    info = dl.plan_info()
    assert info["streaming"] and info["phases"] == 300 and info["waits"] == 0
    skips = nvq.plan_describe_skips([dl.arr[i] for i in range(dl.n)], 1,
                                    workgroups=torch.cuda.get_device_properties(0).multi_processor_count)
    assert skips.max() == 255 and skips.shape[0] % 13 == 0
    for rep in range(2):
        for e in entries:
            e["y"].zero_()
        dl.run_plan()
        assert not dl.plan_timed_out()
        for e, y_r in zip(entries, ys_ref):
            assert np_ref.rel_l2(e["y"].cpu().numpy(), y_r) < 1e-5
    dl.close()


def test_streaming_plan_orders_dependent_phases():
    say("stream chain")
    # four phases, each reading the bf16 output of the one before it
    dims = [2048, 4096, 1024, 6144, 512]
    hostW = [oracle.pack_int4(synth.make_weight(8800 + i, dims[i + 1], dims[i]).numpy())
             for i in range(4)]
    x0 = act(8899, 1, dims[0])
    bufs = [x0.to(DEV)] + [torch.zeros((1, d), dtype=torch.bfloat16, device=DEV) for d in dims[1:]]
    entries = []
    for i, (q, s) in enumerate(hostW):
        qd, sd = to_dev_packed(q, s)
        entries.append(dict(qweight=qd, scales=sd, x=bufs[i], y=bufs[i + 1], precision=i % 2))
    dl = nvq.DecodeList(entries, 1)
    info = dl.plan_info()
    assert info["streaming"] and info["waits"] == 3      # the analysis found the chain
    for rep in range(3):
        for b in bufs[1:]:
            b.zero_()
        dl.run_plan()
        assert not dl.plan_timed_out()
        # each stage against the oracle applied to the GPU's own previous stage
        for i, (q, s) in enumerate(hostW):
            y_r = oracle.decode_linears([dict(qweight=q, scales=s, x=u16(bufs[i]),
                                              precision=i % 2)], 1)[0]
            assert np_ref.rel_l2(bufs[i + 1].float().cpu().numpy(), y_r) < 4e-3, (rep, i)
    dl.close()


# ---- grouped small-batch walker (2..32 tokens on the matrix cores) -------------------
@pytest.mark.parametrize("name,M,ordered", [("1b", 5, False), ("1b", 20, True), ("8b", 16, False),
                                            ("8b", 32, False)])
def test_grouped_plan_matches_oracle_on_repeated_runs(name, M, ordered):
    say("grouped plan", name, M, ordered)
    shapes, bits = STREAM_MODELS[name]
    entries, host = model_entries(shapes, bits, M=M, seed=8300)
    ys_ref = oracle.decode_linears(host, M, 0)
    dl = nvq.DecodeList(entries, M, 0, ordered=ordered)
    info = dl.plan_info()
    say("  plan", info)
    assert not info["streaming"]
    assert info["persistent_grouped"]              # every K of these models is a multiple of 512
    # "waits" counts the batch boundaries: independent buffers make one batch of all phases
    assert info["waits"] == (info["phases"] - 1 if ordered else 0)
    for rep in range(3):
        for e in entries:
            e["y"].zero_()
        dl.run_plan()
        torch.cuda.synchronize()
        assert not dl.plan_timed_out()
        for e, y_r in zip(entries, ys_ref):
            err = np_ref.rel_l2(e["y"].cpu().numpy(), y_r)
            assert err < TOL, (rep, err)
            assert err < 1e-5, (rep, err)
    # the one-call entry point takes the same path
    for e in entries:
        e["y"].zero_()
    nvq.decode_linears(entries, M, 0)
    torch.cuda.synchronize()
    for e, y_r in zip(entries, ys_ref):
        assert np_ref.rel_l2(e["y"].cpu().numpy(), y_r) < 1e-5
    dl.close()


# The persistent small-batch kernel (loader wave + LDS rings) serves lists with every K a
# multiple of 512; these shapes exercise what its bookkeeping has to get right:
# row counts that end inside a unit of 32 rows and inside a 16-row tile, phases of several
# matrices whose boundaries fall inside a unit, a phase with fewer units than teams next to
# long ones (team ranges that cross phases), K from one step (512) to 28 steps, both
# precisions, and token counts from 2 to 32 (one or two token tiles).
RING_SHAPES = [(1000, 1536, 0), (37, 1536, 0), (3, 1536, 1), (2500, 3072, 2), (777, 3072, 2),
               (64, 14336, 3), (48, 512, 4), (4100, 512, 4), (16, 1024, 5)]


@pytest.mark.parametrize("M,bits", [(2, (0, 1)), (7, (1, 0)), (16, (0, 1, 1)), (17, (0, 1)),
                                    (32, (1, 0))])
def test_ring_plan_matches_oracle(M, bits):
    say("ring plan", M, bits)
    entries, host = model_entries(RING_SHAPES, bits, M=M, seed=8600)
    ys_ref = oracle.decode_linears(host, M, 0)
    dl = nvq.DecodeList(entries, M, 0)
    info = dl.plan_info()
    say("  plan", info)
    assert info["grouped"] and info["persistent_grouped"]
    for rep in range(3):
        for e in entries:
            e["y"].zero_()
        dl.run_plan()
        torch.cuda.synchronize()
        assert not dl.plan_timed_out()
        for e, y_r in zip(entries, ys_ref):
            assert np_ref.rel_l2(e["y"].cpu().numpy(), y_r) < 1e-5, rep
    dl.close()


def test_ring_plan_needs_k_multiple_of_512():
    say("ring plan fallback")
    M = 4
    entries, host = model_entries([(96, 1536, 0), (200, 640, 1)], (0, 1), M=M, seed=8700)
    ys_ref = oracle.decode_linears(host, M, 0)
    dl = nvq.DecodeList(entries, M, 0)
    info = dl.plan_info()
    assert info["grouped"] and not info["persistent_grouped"]   # K = 640: the per-tile grid
    dl.run_plan()
    torch.cuda.synchronize()
    for e, y_r in zip(entries, ys_ref):
        assert np_ref.rel_l2(e["y"].cpu().numpy(), y_r) < 1e-5
    dl.close()


def test_grouped_plan_orders_dependent_phases():
    say("grouped chain")
    # four phases, each reading the bf16 output of the one before it: four batches
    M = 6
    dims = [2048, 4096, 1024, 6144, 512]
    hostW = [oracle.pack_int4(synth.make_weight(8900 + i, dims[i + 1], dims[i]).numpy())
             for i in range(4)]
    x0 = act(8999, M, dims[0])
    bufs = [x0.to(DEV)] + [torch.zeros((M, d), dtype=torch.bfloat16, device=DEV) for d in dims[1:]]
    entries = []
    for i, (q, s) in enumerate(hostW):
        qd, sd = to_dev_packed(q, s)
        entries.append(dict(qweight=qd, scales=sd, x=bufs[i], y=bufs[i + 1], precision=i % 2))
    dl = nvq.DecodeList(entries, M)
    info = dl.plan_info()
    assert not info["streaming"] and info["waits"] == 3      # the analysis found the chain
    for rep in range(2):
        for b in bufs[1:]:
            b.zero_()
        dl.run_plan()
        torch.cuda.synchronize()
        for i, (q, s) in enumerate(hostW):
            y_r = oracle.decode_linears([dict(qweight=q, scales=s, x=u16(bufs[i]),
                                              precision=i % 2)], M)[0]
            assert np_ref.rel_l2(bufs[i + 1].float().cpu().numpy(), y_r) < 4e-3, (rep, i)
    dl.close()


# ---- input transforms: RMSNorm (+ residual) and SiLU-multiply ------------------------
def ulp_report(got_u16, want_u16):
    """(fraction of differing elements, largest difference in bf16 units of last place)."""
    a = got_u16.astype(np.int32)
    b = want_u16.astype(np.int32)
    # order-preserving integer view of the sign-magnitude patterns
    a = np.where(a & 0x8000, -(a & 0x7fff), a)
    b = np.where(b & 0x8000, -(b & 0x7fff), b)
    d = np.abs(a - b)
    return float((d != 0).mean()), int(d.max())


@pytest.mark.parametrize("M,K,with_res", [(1, 4096, False), (1, 4096, True), (3, 2048, True),
                                          (16, 14336, True), (2, 96, False), (32, 8192, False)])
def test_rms_norm_matches_oracle(M, K, with_res):
    say("rms_norm", M, K, with_res)
    x = act(9100 + K, M, K)
    r = act(9200 + K, M, K) if with_res else None
    gamma = (1.0 + 0.1 * torch.randn(K, generator=torch.Generator().manual_seed(K))).to(torch.bfloat16)
    out_r, h_r = oracle.rms_norm(u16(x), u16(gamma), 1e-5, res_bf16=u16(r) if with_res else None)
    out, h = nvq.rms_norm(x.to(DEV), gamma.to(DEV), 1e-5, r.to(DEV) if with_res else None)
    torch.cuda.synchronize()
    if with_res:
        assert np.array_equal(u16(h), h_r)            # the bf16 addition is exact-rounded
    frac, worst = ulp_report(u16(out), out_r)
    say("  differing %.2e, worst %d ulp" % (frac, worst))
    assert worst <= 1 and frac < 2e-3


@pytest.mark.parametrize("M,K", [(1, 14336), (5, 8192), (32, 4096), (2, 64)])
def test_silu_mul_matches_oracle(M, K):
    say("silu_mul", M, K)
    g = act(9300 + K, M, K)
    u = act(9400 + K, M, K)
    want = oracle.silu_mul(u16(g), u16(u))
    out = nvq.silu_mul(g.to(DEV), u.to(DEV))
    torch.cuda.synchronize()
    frac, worst = ulp_report(u16(out), want)
    say("  differing %.2e, worst %d ulp" % (frac, worst))
    assert worst <= 1 and frac < 2e-3


def block_with_transforms(M, hidden, kv, ffn, seed, bits):
    """One transformer block's linears with their neighbours fused in: RMSNorm in front of
    q/k/v, the attention output (its own buffer) into o, residual add + RMSNorm in front of
    gate/up, SiLU-multiply in front of down.  Returns (entries, buffers, host weights)."""
    g1 = (1.0 + 0.1 * torch.randn(hidden, generator=torch.Generator().manual_seed(seed))).to(torch.bfloat16)
    g2 = (1.0 + 0.1 * torch.randn(hidden, generator=torch.Generator().manual_seed(seed + 1))).to(torch.bfloat16)
    B = dict(h0=act(seed + 2, M, hidden).to(DEV), attn=act(seed + 3, M, hidden).to(DEV),
             g1=g1.to(DEV), g2=g2.to(DEV),
             o=torch.zeros((M, hidden), dtype=torch.bfloat16, device=DEV),
             h1=torch.zeros((M, hidden), dtype=torch.bfloat16, device=DEV),
             gate=torch.zeros((M, ffn), dtype=torch.bfloat16, device=DEV),
             up=torch.zeros((M, ffn), dtype=torch.bfloat16, device=DEV))
    shapes = [("q", hidden, hidden), ("k", kv, hidden), ("v", kv, hidden), ("o", hidden, hidden),
              ("gate", ffn, hidden), ("up", ffn, hidden), ("down", hidden, ffn)]
    W, entries = {}, []
    for i, (name, N, K) in enumerate(shapes):
        _, q, s = packed(seed + 10 + i, N, K)
        W[name] = (q, s)
        qd, sd = to_dev_packed(q, s)
        e = dict(qweight=qd, scales=sd, precision=bits[0] if i < 4 else bits[1])
        if name in ("q", "k", "v"):
            e.update(x=B["h0"], in_op=nvq.IN_RMSNORM, gamma=B["g1"], eps=1e-5,
                     y=torch.zeros((M, N), dtype=torch.float32, device=DEV))
        elif name == "o":
            e.update(x=B["attn"], y=B["o"])
        elif name in ("gate", "up"):
            e.update(x=B["h0"], x2=B["o"], in_op=nvq.IN_RMSNORM, gamma=B["g2"], eps=1e-5,
                     h_out=B["h1"], y=B[name])
        else:
            e.update(x=B["gate"], x2=B["up"], in_op=nvq.IN_SILU_MUL,
                     y=torch.zeros((M, N), dtype=torch.float32, device=DEV))
        entries.append(e)
    return entries, B, W


def check_block_against_oracle(entries, B, W, M):
    """Every stage against the oracle applied to the GPU's own inputs of that stage."""
    names = ["q", "k", "v", "o", "gate", "up", "down"]
    for e, name in zip(entries, names):
        q, s = W[name]
        h = dict(qweight=q, scales=s, x=u16(e["x"]), precision=e["precision"],
                 in_op=e.get("in_op", 0))
        if e.get("x2") is not None:
            h["x2"] = u16(e["x2"])
        if e.get("gamma") is not None:
            h["gamma"], h["eps"] = u16(e["gamma"]), e["eps"]
        y_r = oracle.decode_linears([h], M)[0]
        got = e["y"].float().cpu().numpy()
        err = np_ref.rel_l2(got, y_r)
        # fp32 outputs: the bar (rare one-ulp differences of a transformed bf16 input move them
        # by ~1e-4); bf16 outputs add their own rounding, 2^-9 relative per value at most
        assert err < (TOL if e["y"].dtype == torch.float32 else 4e-3), (name, err)
        if name == "gate":
            assert np.array_equal(u16(B["h1"]), h["h"])       # the updated residual stream


@pytest.mark.parametrize("M", [1, 3])
@pytest.mark.parametrize("bits", [(0, 1), (1, 0)])
def test_decode_linears_with_input_transforms(M, bits):
    say("walker with transforms", M, bits)
    entries, B, W = block_with_transforms(M, 2048, 512, 8192, 9500, bits)
    dl = nvq.DecodeList(entries, M, 0)
    info = dl.plan_info()
    say("  plan", info)
    if M == 1:
        # one launch; gate/up wait for o (their residual operand), down waits for gate/up
        assert info["streaming"] and info["phases"] == 4 and info["waits"] == 2
    for rep in range(2):
        for k in ("o", "h1", "gate", "up"):
            B[k].zero_()
        dl.run_plan()
        torch.cuda.synchronize()
        assert not dl.plan_timed_out()
        check_block_against_oracle(entries, B, W, M)
    dl.close()


def test_chain_of_blocks_with_transforms_in_one_launch():
    say("block chain with transforms")
    # two blocks at the 1B shapes, the second fed by the first (the residual add of the first
    # block's down projection happens in front of the second block's q/k/v), W4A8 then W4A16
    M, hidden, kv, ffn = 1, 2048, 512, 8192
    e0, B0, W0 = block_with_transforms(M, hidden, kv, ffn, 9600, (0, 0))
    e1, B1, W1 = block_with_transforms(M, hidden, kv, ffn, 9700, (1, 1))
    down0 = torch.zeros((M, hidden), dtype=torch.bfloat16, device=DEV)
    e0[6]["y"] = down0
    h2 = torch.zeros((M, hidden), dtype=torch.bfloat16, device=DEV)
    for e in e1[:3]:                      # q/k/v of block 1: RMSNorm(h1 + down0), sum -> h2
        e.update(x=B0["h1"], x2=down0, h_out=h2)
    for e in e1[4:6]:                     # gate/up of block 1: RMSNorm(h2 + o1), sum -> h1'
        e.update(x=h2)
    entries = e0 + e1
    dl = nvq.DecodeList(entries, M, 0)
    info = dl.plan_info()
    say("  plan", info)
    assert info["streaming"] and info["phases"] == 8 and info["waits"] == 5
    for rep in range(3):
        for t in (B0["o"], B0["h1"], B0["gate"], B0["up"], down0, h2, B1["o"], B1["h1"],
                  B1["gate"], B1["up"]):
            t.zero_()
        dl.run_plan()
        torch.cuda.synchronize()
        assert not dl.plan_timed_out(), (rep, hex(dl.status_code))
        check_block_against_oracle(e0, B0, W0, M)
        check_block_against_oracle(e1, B1, W1, M)
        # the residual stream entering block 1 is the exact bf16 sum
        assert torch.equal(h2, B0["h1"] + down0)
    dl.close()


# ---- exact sums: int32 accumulators and fused int8 codes of the kernels that are timed ----
def exact_layer(rng, N, K, M, per_group):
    """Weights c * 2^-7 with integer codes c in [-7, 7] (a 7 in every group: the scale is
    2^-7 exactly) and activations q * 2^e with integer q in [-127, 127] (a 127 in every token,
    or in every group of 32: the activation scale is 2^e exactly and the codes are q).  Then
    every int32 accumulator is the plain integer sum, every fp32 partial sum of the output
    is an integer multiple of a power of two below 2^24 of it, hence exact in any order:
    the fp32 output of a correct kernel equals the float64 oracle's to the bit, and a single
    wrong code or accumulator shows."""
    c = rng.integers(-7, 8, (N, K)).astype(np.float32)
    pos = rng.integers(0, 32, (N, K // 32))
    c.reshape(N, K // 32, 32)[np.arange(N)[:, None], np.arange(K // 32)[None, :], pos] = \
        rng.choice([-7.0, 7.0], (N, K // 32))
    W = c * np.float32(2.0 ** -7)
    q = rng.integers(-127, 128, (M, K)).astype(np.float32)
    if per_group:
        pos = rng.integers(0, 32, (M, K // 32))
        q.reshape(M, K // 32, 32)[np.arange(M)[:, None], np.arange(K // 32)[None, :], pos] = \
            rng.choice([-127.0, 127.0], (M, K // 32))
        e = rng.integers(-2, 3, (M, K // 32)).astype(np.float32)
        x = (q.reshape(M, K // 32, 32) * (2.0 ** e)[:, :, None]).reshape(M, K)
    else:
        q[np.arange(M), rng.integers(0, K, M)] = rng.choice([-127.0, 127.0], M)
        x = q * (2.0 ** rng.integers(-3, 4, (M, 1)).astype(np.float32))
    xb = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16)
    assert torch.equal(xb.float(), torch.from_numpy(x.astype(np.float32)))      # exact in bf16
    qw, sc = oracle.pack_int4(W)
    assert (sc == 0x2000).all()                                               # fp16 2^-7
    return qw, sc, xb


def exact_list(seed, shapes, M, per_group):
    """shapes: (N, K, phase); one input per phase; precisions alternate by phase."""
    rng = np.random.default_rng(seed)
    entries, host, xs = [], [], {}
    for N, K, ph in shapes:
        qw, sc, xb = exact_layer(rng, N, K, M, per_group)
        if ph not in xs:
            xs[ph] = xb
        qd, sd = to_dev_packed(qw, sc)
        prec = ph % 2
        entries.append(dict(qweight=qd, scales=sd, x=xs[ph].to(DEV), precision=prec,
                            y=torch.zeros((M, N), dtype=torch.float32, device=DEV)))
        host.append(dict(qweight=qw, scales=sc, x=u16(xs[ph]), precision=prec))
    # (entries of a phase must share the device buffer to be grouped)
    by_phase = {}
    for e, (_, _, ph) in zip(entries, shapes):
        e["x"] = by_phase.setdefault(ph, e["x"])
    return entries, host


EXACT_SHAPES = [(4096, 4096, 0), (1024, 4096, 0), (1031, 4096, 1), (640, 14336, 2), (96, 14336, 2),
                (2500, 2048, 3), (77, 8192, 4), (3000, 1024, 5)]


@pytest.mark.parametrize("M,group,ordered", [(1, 0, False), (1, 0, True), (1, 32, False),
                                             (1, 32, True), (2, 0, False), (5, 0, False),
                                             (16, 0, False), (17, 0, False), (32, 0, False),
                                             (3, 32, False)])
def test_exact_sums_are_bit_equal_on_the_timed_kernels(M, group, ordered):
    """Batch 1: the persistent streaming kernel with its fused quantiser, images prepared in
    the prologue (independent phases) and built after a wait (forced ordering).  2 to 32
    tokens: the persistent matrix-core kernel (every K a multiple of 512).  A scale per 32
    activations at several tokens: launches per phase."""
    say("exact sums", M, group, ordered)
    entries, host = exact_list(9000 + M + group, EXACT_SHAPES, M, group == 32)
    ys_ref = oracle.decode_linears(host, M, group)
    dl = nvq.DecodeList(entries, M, group, ordered=ordered)
    info = dl.plan_info()
    say("  plan", info)
    assert info["streaming"] == (M == 1)
    assert info["persistent_grouped"] == (M > 1 and group == 0)
    for rep in range(2):
        for e in entries:
            e["y"].zero_()
        dl.run_plan()
        assert not dl.plan_timed_out()
        for i, (e, y_r) in enumerate(zip(entries, ys_ref)):
            want = y_r.astype(np.float32)
            assert np.array_equal(want.astype(np.float64), y_r)        # the oracle's sum is exact
            got = e["y"].cpu().numpy()
            assert np.array_equal(got, want), (rep, i, int((got != want).sum()))
    dl.close()


def test_exact_sums_are_bit_equal_on_the_per_tile_matrix_core_kernel():
    """K = 640 (no multiple of 512): the grouped per-tile grid with its own quantiser."""
    say("exact sums, per-tile grid")
    M = 7
    entries, host = exact_list(9100, [(200, 640, 0), (96, 1536, 1), (333, 640, 2)], M, False)
    ys_ref = oracle.decode_linears(host, M, 0)
    dl = nvq.DecodeList(entries, M, 0)
    info = dl.plan_info()
    assert info["grouped"] and not info["persistent_grouped"]
    dl.run_plan()
    torch.cuda.synchronize()
    for e, y_r in zip(entries, ys_ref):
        assert np.array_equal(e["y"].cpu().numpy(), y_r.astype(np.float32))
    dl.close()


# ---- mail: an operand that is exactly an earlier layer's bf16 output ---------------------
def stage_reference(e, q, s, M=1):
    """The oracle on the GPU's own inputs of one layer."""
    h = dict(qweight=q, scales=s, x=u16(e["x"]), precision=e["precision"], in_op=e.get("in_op", 0))
    if e.get("x2") is not None:
        h["x2"] = u16(e["x2"])
    if e.get("gamma") is not None:
        h["gamma"], h["eps"] = u16(e["gamma"]), e["eps"]
    return oracle.decode_linears([h], M)[0]


@pytest.mark.parametrize("widths,group", [
    ((2048, 96, 2112, 4096, 64), 0),            # one ragged piece, a part of a piece, whole pieces
    ((4096, 14336, 3072, 1024, 8192, 32), 0),   # the widest input; rows streamed in pairs
    ((1024, 3136, 2048, 512), 32),              # a scale per 32 activations
])
def test_mail_chain_of_plain_layers(widths, group):
    """x0 -> L0 -> L1 -> ...: every layer reads the bf16 output of the one before it, so every
    operand but the first arrives by mail; precisions alternate; several walks (one tag each)."""
    say("mail chain", widths, group)
    entries, W = [], []
    x = act(9900 + widths[0], 1, widths[0]).to(DEV)
    for i in range(len(widths) - 1):
        K, N = widths[i], widths[i + 1]
        _, q, s = packed(9910 + 7 * i + N, N, K)
        qd, sd = to_dev_packed(q, s)
        y = torch.zeros((1, N), dtype=torch.bfloat16, device=DEV)
        entries.append(dict(qweight=qd, scales=sd, x=x, y=y, precision=(i + group // 32) % 2))
        W.append((q, s))
        x = y
    dl = nvq.DecodeList(entries, 1, group)
    info = dl.plan_info()
    _, phases = nvq.plan_describe([dl.arr[i] for i in range(dl.n)], 1, group)
    say("  plan", info, [ph["mail"] for ph in phases])
    assert info["streaming"] and info["waits"] == len(entries) - 1
    assert [ph["mail"] & 3 for ph in phases] == [0] + [1] * (len(entries) - 1)
    assert all(ph["wait"] < 0 for ph in phases)          # nobody waits for flags
    for rep in range(4):
        for e in entries:
            e["y"].zero_()
        if rep == 2:                                      # new data under the next tag
            entries[0]["x"].copy_(act(9950, 1, widths[0]).to(DEV))
        dl.run_plan()
        assert not dl.plan_timed_out()
        for e, (q, s) in zip(entries, W):
            y_r = oracle.decode_linears([dict(qweight=q, scales=s, x=u16(e["x"]),
                                              precision=e["precision"])], 1, group)[0]
            err = np_ref.rel_l2(e["y"].float().cpu().numpy(), y_r)
            assert err < 4e-3, (rep, err)                 # bf16 outputs
            # to the bit once the oracle's value is rounded to bf16 as well, but for sums that
            # fall next to a rounding boundary
            want = torch.from_numpy(y_r.astype(np.float32)).to(torch.bfloat16)
            differing = int((e["y"].cpu() != want).sum())
            assert differing <= max(1, int(5e-3 * want.numel())), (rep, differing)
    dl.close()


def test_mail_and_flags_in_one_list():
    """A buffer that is written twice and read in between: the reader takes the first
    writer's mail, the second writer waits for the first through the flags (it overwrites its
    bytes), and a last layer reads the second writer's mail."""
    say("mail and flags")
    K = 2048
    x0, x1 = act(9960, 1, K).to(DEV), act(9961, 1, K).to(DEV)
    y = torch.zeros((1, K), dtype=torch.bfloat16, device=DEV)
    outs = [torch.zeros((1, 640), dtype=torch.float32, device=DEV) for _ in range(2)]
    Ws = [packed(9970 + i, n, K) for i, n in enumerate((K, 640, K, 640))]
    dev = [to_dev_packed(q, s) for _, q, s in Ws]
    mk = lambda i, x, yy, prec: dict(qweight=dev[i][0], scales=dev[i][1], x=x, y=yy, precision=prec)
    entries = [mk(0, x0, y, 0), mk(1, y, outs[0], 1), mk(2, x1, y, 1), mk(3, y, outs[1], 0)]
    dl = nvq.DecodeList(entries, 1, 0)
    _, phases = nvq.plan_describe([dl.arr[i] for i in range(dl.n)], 1, 0)
    assert [ph["wait"] for ph in phases] == [-1, -1, 0, -1]
    assert [ph["mail"] & 3 for ph in phases] == [0, 1, 0, 1]
    for rep in range(3):
        for t in [y] + outs:
            t.zero_()
        dl.run_plan()
        assert not dl.plan_timed_out()
        # y holds the second writer's result; the first reader saw the first writer's
        y1 = oracle.decode_linears([dict(qweight=Ws[0][1], scales=Ws[0][2], x=u16(x0), precision=0)], 1)[0]
        y1b = torch.from_numpy(y1.astype(np.float32)).to(torch.bfloat16)
        r0 = oracle.decode_linears([dict(qweight=Ws[1][1], scales=Ws[1][2], x=u16(y1b), precision=1)], 1)[0]
        assert np_ref.rel_l2(outs[0].cpu().numpy(), r0) < 5e-3     # (y1b may differ by an ulp here and there)
        r2 = stage_reference(entries[2], Ws[2][1], Ws[2][2])
        assert np_ref.rel_l2(y.float().cpu().numpy(), r2) < 4e-3
        r3 = stage_reference(entries[3], Ws[3][1], Ws[3][2])
        assert np_ref.rel_l2(outs[1].cpu().numpy(), r3) < 1e-5
    dl.close()


def test_mail_tags_wrap_around():
    """A tag has 16 bits: 65535 walks later the same tag comes round again.  Between walks the
    input changes, so a consumer that took an old word for a new one would show."""
    say("mail tag wrap")
    K = 512
    _, q0, s0 = packed(9980, K, K)
    _, q1, s1 = packed(9981, 96, K)
    d0, d1 = to_dev_packed(q0, s0), to_dev_packed(q1, s1)
    x = act(9982, 1, K).to(DEV)
    mid = torch.zeros((1, K), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((1, 96), dtype=torch.float32, device=DEV)
    entries = [dict(qweight=d0[0], scales=d0[1], x=x, y=mid, precision=1),
               dict(qweight=d1[0], scales=d1[1], x=mid, y=out, precision=0)]
    dl = nvq.DecodeList(entries, 1, 0)
    dl.plan()
    xs = [act(9983 + i, 1, K).to(DEV) for i in range(3)]
    total = 65535 + 6
    for run in range(total):
        check = run < 3 or run >= 65535 - 3
        if check:
            x.copy_(xs[run % 3])
        dl.run_plan()
        if check:
            assert not dl.plan_timed_out()
            r = stage_reference(entries[1], q1, s1)
            assert np_ref.rel_l2(out.cpu().numpy(), r) < 1e-5, run
            m = oracle.decode_linears([dict(qweight=q0, scales=s0, x=u16(x), precision=1)], 1)[0]
            assert np_ref.rel_l2(mid.float().cpu().numpy(), m) < 4e-3, run
        elif run % 8192 == 0:
            torch.cuda.synchronize()
    assert not dl.plan_timed_out()
    dl.close()


# ---- prefill / large-batch product on the matrix cores --------------------------------
# Shapes: one tile, ragged tokens and rows inside a 256 x 128 workgroup tile and inside the
# 32 x 32 MFMA tiles, several workgroups in both directions, K from one group to many.
# The last two: many workgroups in both directions, ragged at both ends.
@pytest.mark.parametrize("M,N,K", [(32, 32, 32), (256, 128, 64), (77, 45, 96), (300, 200, 256),
                                   (513, 257, 2048), (1, 1, 32), (1024, 384, 4096),
                                   (4096, 4096, 64), (4000, 4300, 96)])
def test_gemm_w4a16_matches_oracle(M, N, K):
    say("gemm", M, N, K)
    _, q, s = packed(9100 + M + N, N, K)
    xh = act(9200 + K, M, K)
    want = oracle.gemm_w4a16_dense(q, s, u16(xh))
    qd, sd = to_dev_packed(q, s)
    y = nvq.gemm_w4a16(qd, sd, xh.to(DEV))
    torch.cuda.synchronize()
    err = np_ref.rel_l2(y.cpu().numpy(), want)
    say("  rel l2", err)
    assert err < 1e-5
    yb = nvq.gemm_w4a16(qd, sd, xh.to(DEV), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert np_ref.rel_l2(yb.float().cpu().numpy(), want) < 4e-3


# The kernel with 256 x 256 tiles (K % 256 == 0; chosen by itself from 96 tiles on, forced here
# so that small shapes reach it): one tile, ragged tokens and rows inside a tile and inside the
# MFMA tiles, a single row and token, several tiles in both directions, K from one block of four
# pairs of groups (no steady state in the loop) to many, K with an odd number of such blocks.
@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (300, 200, 512), (1, 1, 256), (33, 70, 1280),
                                   (513, 257, 2048), (1024, 384, 4096), (700, 1000, 2304)])
def test_gemm_w4a16_wide_tiles_match_oracle(M, N, K, monkeypatch):
    say("gemm wide", M, N, K)
    monkeypatch.setenv("NVQ_GEMM_TILE", "wide")
    _, q, s = packed(9150 + M + N, N, K)
    xh = act(9250 + K, M, K)
    want = oracle.gemm_w4a16_dense(q, s, u16(xh))
    qd, sd = to_dev_packed(q, s)
    y = nvq.gemm_w4a16(qd, sd, xh.to(DEV))
    torch.cuda.synchronize()
    err = np_ref.rel_l2(y.cpu().numpy(), want)
    say("  rel l2", err)
    assert err < 1e-5
    yb = nvq.gemm_w4a16(qd, sd, xh.to(DEV), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert np_ref.rel_l2(yb.float().cpu().numpy(), want) < 4e-3
    # both kernels add the same products in the same order
    monkeypatch.setenv("NVQ_GEMM_TILE", "narrow")
    yn = nvq.gemm_w4a16(qd, sd, xh.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(y, yn)


def test_gemm_w4a16_full_size_sampled():
    """A projection of the 8B block at 4096 tokens, as the benchmark launches it (the kernel with
    wide tiles, chosen by the library): sampled tokens and rows against the oracle."""
    say("gemm full size")
    M, N, K = 4096, 4096, 4096
    _, q, s = packed(9160, N, K)
    xh = act(9260, M, K)
    qd, sd = to_dev_packed(q, s)
    y = nvq.gemm_w4a16(qd, sd, xh.to(DEV))
    torch.cuda.synchronize()
    rng = np.random.default_rng(9161)
    toks = np.unique(np.concatenate([[0, 255, 256, M - 1], rng.integers(0, M, 28)]))
    rows = np.unique(np.concatenate([[0, 31, 32, 63, 64, 255, 256, N - 1], rng.integers(0, N, 56)]))
    want = oracle.gemm_w4a16_dense(q[rows], s[rows], u16(xh)[toks])
    got = y.cpu().numpy()[np.ix_(toks, rows)]
    err = np_ref.rel_l2(got, want)
    say("  rel l2", err)
    assert err < 1e-5


def test_gemm_w4a16_takes_every_code(monkeypatch):
    say("gemm codes")
    rng = np.random.default_rng(9300)
    M, N, K = 96, 64, 128
    q = rng.integers(0, 256, (N, K // 2)).astype(np.uint8)          # code -8 included
    s = (rng.random((N, K // 32)).astype(np.float32) * 0.1 + 0.01).astype(np.float16).view(np.uint16)
    xh = act(9301, M, K)
    want = oracle.gemm_w4a16_dense(q, s, u16(xh))
    qd, sd = to_dev_packed(q, s)
    y = nvq.gemm_w4a16(qd, sd, xh.to(DEV))
    torch.cuda.synchronize()
    assert np_ref.rel_l2(y.cpu().numpy(), want) < 1e-5
    # and with the wide tiles
    K = 256
    q = rng.integers(0, 256, (N, K // 2)).astype(np.uint8)
    s = (rng.random((N, K // 32)).astype(np.float32) * 0.1 + 0.01).astype(np.float16).view(np.uint16)
    xh = act(9302, M, K)
    want = oracle.gemm_w4a16_dense(q, s, u16(xh))
    qd, sd = to_dev_packed(q, s)
    monkeypatch.setenv("NVQ_GEMM_TILE", "wide")
    y = nvq.gemm_w4a16(qd, sd, xh.to(DEV))
    torch.cuda.synchronize()
    assert np_ref.rel_l2(y.cpu().numpy(), want) < 1e-5


# ---- calibration statistics (Algorithm 1) ----------------------------------------------
@pytest.mark.parametrize("M,Na,Nb,bf16", [(1, 5, 0, False), (7, 4096, 1024, False),
                                          (33, 4096, 0, True), (3, 1000, 37, True)])
def test_token_norms_match_oracle(M, Na, Nb, bf16):
    say("token norms", M, Na, Nb, bf16)
    g = torch.Generator().manual_seed(9400 + M)
    a = torch.randn((M, Na), generator=g) * 3
    b = torch.randn((M, Nb), generator=g) if Nb else None
    if bf16:
        a = a.to(torch.bfloat16)
        b = b.to(torch.bfloat16) if b is not None else None
        want = oracle.token_norms(u16(a), u16(b) if b is not None else None)
    else:
        want = oracle.token_norms(a.numpy(), b.numpy() if b is not None else None)
    got = nvq.token_norms(a.to(DEV), b.to(DEV) if b is not None else None)
    torch.cuda.synchronize()
    assert np.allclose(got.cpu().numpy(), want, rtol=2e-6, atol=0)
