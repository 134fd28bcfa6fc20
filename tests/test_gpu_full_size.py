"""GPU parity at the benchmark's full size: the Llama-3.1-8B-shaped decode step
(225 linears, 7.5 G weights), built and launched exactly as bench.py does, with
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


@pytest.mark.parametrize("M", [1, 16])
def test_full_8b_step_sampled_rows_match_oracle(M):
    print("full size 8B step, M =", M, flush=True)
    model = "llama-8b"
    nb = synth.MODELS[model][0]
    bits = synth.make_precision_map(nb, nb // 2)
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
