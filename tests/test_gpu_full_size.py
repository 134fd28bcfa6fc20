"""GPU parity at the benchmark's full sizes: the Llama-shaped decode steps (8B: 225
linears, 7.5 G weights; 3B; 1B), built and launched exactly as bench.py does, with
sampled output rows checked one by one against the CPU oracle.

Per layer a few rows are sampled (first, last, two seeded); their fp32 weights
are copied to the host before the GPU packs the layer, the oracle packs and
multiplies them itself, and the GPU's packed bytes, scales and outputs of those
rows must match (bytes exactly, outputs within 1e-3 relative L2 per layer)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_21026_amd import nvq, synth
from tests import np_ref

pytestmark = pytest.mark.gpu

DEV = "cuda"
TOL = 1e-3


def u16(t):
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


def build_sampled_model(model, M, bits):
    """bench.py's build (same seeds, same generators), keeping sampled fp32 rows."""
    rng = np.random.default_rng(4242)
    layers, xbuf = [], {}
    for sp in synth.model_linears(model):
        seed = synth.tensor_seed(sp.block if sp.block >= 0 else 999, sp.slot)
        W = synth.make_weight(seed, sp.N, sp.K, device=DEV)
        rows = np.unique(np.concatenate([[0, sp.N - 1], rng.integers(0, sp.N, 2)]))
        w_rows = W[torch.from_numpy(rows).to(DEV)].cpu().numpy()
        q, s = nvq.pack_int4(W)
        torch.cuda.synchronize()
        del W
        if sp.phase not in xbuf:
            xbuf[sp.phase] = synth.make_activation(synth.activation_seed(sp.phase), M, sp.K, True,
                                                   device=DEV)
        prec = nvq.W4A16 if sp.block < 0 else bits[sp.block]
        layers.append(dict(spec=sp, qweight=q, scales=s, x=xbuf[sp.phase], precision=prec,
                           y=torch.zeros((M, sp.N), dtype=torch.float32, device=DEV),
                           rows=rows, w_rows=w_rows))
    return layers


@pytest.mark.parametrize("model,M", [("llama-8b", 1), ("llama-8b", 16), ("llama-8b", 32),
                                     ("llama-1b", 1), ("llama-3b", 1)])
def test_full_step_sampled_rows_match_oracle(model, M):
    """The benchmark's workloads as bench.py builds and launches them: the 8B step at 1, 16 and
    32 tokens (one and two token tiles of the matrix-core kernel), and the whole 1B and 3B
    steps at batch 1 (64 and 112 phases: thin phases dealt in larger units, rows of one and a
    half chunks streamed in pairs, the skip table)."""
    import bench
    print("full size step,", model, "M =", M, flush=True)
    bits = bench.block_bits(model, "mixed", synth)
    layers = build_sampled_model(model, M, bits)
    dl = nvq.DecodeList(layers, M, 0)
    dl.plan()
    info = dl.plan_info()
    assert info["streaming"] == (M == 1)       # batch 1 is the one-launch persistent kernel
    for _ in range(2):                          # the second walk reuses flags and images
        dl.run_plan()
    torch.cuda.synchronize()
    assert not dl.plan_timed_out()
    worst = 0.0
    for L in layers:
        sp, rows = L["spec"], L["rows"]
        q_r, s_r = oracle.pack_int4(L["w_rows"])
        idx = torch.from_numpy(rows).to(DEV)
        assert np.array_equal(L["qweight"][idx].cpu().numpy(), q_r), sp.name
        assert np.array_equal(u16(L["scales"][idx]), s_r), sp.name
        xh = u16(L["x"])
        if L["precision"] == nvq.W4A16:
            y_r = oracle.gemv_w4a16(q_r, s_r, xh)
        else:
            xq, xs, _ = oracle.quant_act_i8(xh, 0)
            y_r = oracle.gemv_w4a8(q_r, s_r, xq, xs, 0)
        got = L["y"][:, idx].cpu().numpy()
        err = np_ref.rel_l2(got, y_r)
        worst = max(worst, err)
        assert err < TOL, (sp.name, err)
    print("  worst per-layer relative L2 over sampled rows:", worst, flush=True)
    dl.close()


@pytest.mark.parametrize("model", ["llama-8b", "llama-1b", "llama-3b"])
def test_full_decode_chain_sampled_rows_match_oracle(model):
    """The same linears wired up as bench.py's dependent decode step (norms, residual adds and
    SiLU-multiply fused in, bf16 between the layers; every operand that is an earlier layer's
    output arrives by mail): sampled rows of every layer against the oracle applied to the
    GPU's own inputs of that layer, and the residual stream to the bit."""
    import bench
    print("full size decode chain,", model, flush=True)
    nb = synth.MODELS[model][0]
    bits = bench.block_bits(model, "mixed", synth)
    layers = build_sampled_model(model, 1, bits)
    entries = bench.chain_entries(layers, bits, model, torch, nvq, synth, DEV)
    assert len(entries) == len(layers)
    dl = nvq.DecodeList(entries, 1, 0)
    info = dl.plan_info()
    _, phases = nvq.plan_describe([dl.arr[i] for i in range(dl.n)], 1, 0)
    print("  plan", info, flush=True)
    assert info["streaming"] and info["waits"] == 3 * nb - 1 + (1 if len(layers) % 7 else 0)
    assert all(ph["wait"] < 0 for ph in phases)             # all of it by mail, none by flags
    for _ in range(3):
        dl.run_plan()
    torch.cuda.synchronize()
    assert not dl.plan_timed_out()
    worst32 = worst16 = 0.0
    for L, e in zip(layers, entries):
        sp, rows = L["spec"], L["rows"]
        q_r, s_r = oracle.pack_int4(L["w_rows"])
        h = dict(qweight=q_r, scales=s_r, x=u16(e["x"]), precision=e["precision"],
                 in_op=e.get("in_op", 0))
        if e.get("x2") is not None:
            h["x2"] = u16(e["x2"])
        if e.get("gamma") is not None:
            h["gamma"], h["eps"] = u16(e["gamma"]), e["eps"]
        y_r = oracle.decode_linears([h], 1)[0]
        idx = torch.from_numpy(rows).to(DEV)
        got = e["y"][:, idx].float().cpu().numpy()
        err = np_ref.rel_l2(got, y_r)
        if e["y"].dtype == torch.float32:
            worst32 = max(worst32, err)
            assert err < TOL, (sp.name, err)
        else:
            worst16 = max(worst16, err)
            assert err < 4e-3, (sp.name, err)               # one bf16 rounding per value
        if e.get("h_out") is not None and e.get("x2") is not None:
            assert torch.equal(e["h_out"], e["x"] + e["x2"]), sp.name   # exact bf16 sum
    print("  worst relative L2 over sampled rows: fp32 outputs %.3g, bf16 outputs %.3g"
          % (worst32, worst16), flush=True)
    dl.close()
