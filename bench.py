#!/usr/bin/env python3
"""Benchmark of the decode-linear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--model llama-8b]
                    [--map mixed|w4a8|w4a16] [--leg all|step|roofline|cpu]

A step is one nvq_decode_linears walk over every linear layer of one decode
step (batch 1) of the named Llama-shaped model: activation quantisation for
the W4A8 layers, all GEMVs, lm_head included where the model has one.  All
weights and activations are resident in HBM before the timed region.  Prints
one JSON line (see the design doc for the fields).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--model", default="llama-8b", choices=["llama-1b", "llama-3b", "llama-8b"])
    ap.add_argument("--map", default="mixed", choices=["mixed", "w4a8", "w4a16"])
    ap.add_argument("--leg", default="all", choices=["all", "step", "roofline", "cpu"])
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--act-group", type=int, default=0, choices=[0, 32])
    ap.add_argument("--extra-maps", action="store_true",
                    help="also time the all-W4A8 and all-W4A16 maps (reported under config)")
    return ap.parse_args()


def block_bits(model, which, synth):
    nb = synth.MODELS[model][0]
    if which == "w4a8":
        return [0] * nb
    if which == "w4a16":
        return [1] * nb
    # seeded map: 1B 50% W4A8, 3B 25% W4A16, 8B 50/50
    n16 = {"llama-1b": nb // 2, "llama-3b": nb // 4, "llama-8b": nb // 2}[model]
    return synth.make_precision_map(nb, n16)


def build_model(model, M, torch, nvq, synth, dev):
    """Pack every layer on the GPU (one fp32 tensor alive at a time)."""
    specs = synth.model_linears(model)
    layers = []
    xbuf = {}
    for sp in specs:
        seed = synth.tensor_seed(sp.block if sp.block >= 0 else 999, sp.slot)
        W = synth.make_weight(seed, sp.N, sp.K, device=dev)
        q, s = nvq.pack_int4(W)
        torch.cuda.synchronize()
        del W
        if sp.phase not in xbuf:
            xbuf[sp.phase] = synth.make_activation(synth.activation_seed(sp.phase), M, sp.K,
                                                   True, device=dev)
        y = torch.zeros((M, sp.N), dtype=torch.float32, device=dev)
        layers.append(dict(spec=sp, qweight=q, scales=s, x=xbuf[sp.phase], y=y))
    return layers


def entries_for(layers, bits, nvq):
    out = []
    for L in layers:
        sp = L["spec"]
        prec = nvq.W4A16 if sp.block < 0 else bits[sp.block]
        out.append(dict(qweight=L["qweight"], scales=L["scales"], x=L["x"], y=L["y"],
                        precision=prec))
    return out


def time_steps(dl, steps, warmup, torch):
    """K walks of the prepared plan, bracketed by device synchronisation."""
    dl.plan()
    for _ in range(warmup):
        dl.run_plan()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        dl.run_plan()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    if dl.plan_timed_out():
        raise RuntimeError("a wait inside the streaming kernel timed out; results invalid")
    return sec


def roofline_leg(layers, torch, nvq, synth, reps=5):
    """The dominant kernel in isolation: the batch-1 W4A8 GEMV on the largest
    per-block matrix shape, rotating over every block's copy so that no launch
    finds its weights in cache.  Timed with HIP events on the launch stream."""
    cand = [L for L in layers if L["spec"].block >= 0]
    big = max(L["spec"].N * L["spec"].K for L in cand)
    mats = [L for L in cand if L["spec"].N * L["spec"].K == big and L["spec"].slot in (4, 6)]
    slot = mats[0]["spec"].slot
    mats = [L for L in mats if L["spec"].slot == slot]
    sp = mats[0]["spec"]
    xq, xs, gs = nvq.quant_act_i8(mats[0]["x"][:1].contiguous())
    for L in mats:
        nvq.gemv_w4a8(L["qweight"], L["scales"], xq, xs, gs, out=L["y"][:1])
    torch.cuda.synchronize()
    st = torch.cuda.current_stream()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(reps):
        for L in mats:
            nvq.gemv_w4a8(L["qweight"], L["scales"], xq, xs, gs, out=L["y"][:1])
    e1.record(st)
    torch.cuda.synchronize()
    n = reps * len(mats)
    avg_s = e0.elapsed_time(e1) * 1e-3 / n
    bytes_per_launch = synth.weight_bytes(sp.N, sp.K)
    gbs = bytes_per_launch / avg_s / 1e9
    G = sp.K // 32
    kernel = "gemv_w4a8_m1_kernel<%d, 64, false, false>" % ((G + 63) // 64)
    return {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None, "kernel": kernel,
            "shape": "N=%d K=%d M=1" % (sp.N, sp.K), "launches": n,
            "avg_launch_us": round(avg_s * 1e6, 2), "bytes_per_launch": bytes_per_launch}


def cpu_leg(model, bits, M, synth, budget_s=20.0):
    """The oracle's walker on a bounded sample of the same workload: the first
    blocks of the model (as many as fit the time budget, at least one), inputs
    generated and packed on the CPU by the oracle itself."""
    import numpy as np
    import torch
    import oracle
    specs = [s for s in synth.model_linears(model) if s.block >= 0]
    nb = synth.MODELS[model][0]
    total_w = sum(s.N * s.K for s in synth.model_linears(model))
    host, sample_w, t_gen0 = [], 0, time.perf_counter()
    blocks = 0
    for b in range(nb):
        for sp in [s for s in specs if s.block == b]:
            W = synth.make_weight(synth.tensor_seed(sp.block, sp.slot), sp.N, sp.K)
            q, s = oracle.pack_int4(W.numpy())
            x = synth.make_activation(synth.activation_seed(sp.phase), M, sp.K)
            host.append(dict(qweight=q, scales=s, x=x.view(torch.int16).numpy().view(np.uint16),
                             precision=bits[b]))
            sample_w += sp.N * sp.K
        blocks += 1
        if time.perf_counter() - t_gen0 > budget_s * 0.4 or blocks >= 4:
            break
    oracle.decode_linears(host, M)                       # warm caches / thread pool
    reps, t0 = 0, time.perf_counter()
    while reps < 3 or (time.perf_counter() - t0 < budget_s * 0.4 and reps < 50):
        oracle.decode_linears(host, M)
        reps += 1
    t = (time.perf_counter() - t0) / reps
    step_s = t * total_w / sample_w
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": round(M / step_s, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "oracle walker over the first %d of %d blocks (%d of %d weights), %d reps, "
                      "step time scaled by weight count" % (blocks, nb, sample_w, total_w, reps),
            "gbs": round(total_w * 0.5625 / step_s / 1e9, 2)}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path is a single-GPU decode "
              "step); --gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_21026_amd import nvq, synth

    M = a.batch
    bits = block_bits(a.model, a.map, synth)
    specs = synth.model_linears(a.model)
    step_bytes = sum(synth.weight_bytes(s.N, s.K) for s in specs)
    out = {
        "metric": "decode linear-layer tokens/s + achieved HBM GB/s (% of peak), 8B shapes, batch 1",
        "value": None, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 weights; int8 x int4 -> int32 (W4A8) and bf16 x int4 -> f32 (W4A16)",
        "data": "synthetic",
        "config": {"workload": "%s-shaped decode step, batch %d, %d linears, precision map %s "
                               "(%d of %d blocks W4A16%s)" %
                               (a.model, M, len(specs), a.map, sum(bits), len(bits),
                                ", lm_head W4A16" if specs[-1].block < 0 else ""),
                   "act_group": a.act_group, "weight_bytes_per_step": step_bytes},
    }
    if a.leg in ("all", "step", "roofline"):
        if not torch.cuda.is_available():
            print("bench.py: no GPU visible", file=sys.stderr)
            sys.exit(3)
        dev = "cuda:0"
        torch.cuda.set_device(0)
        nvq.lib()
        layers = build_model(a.model, M, torch, nvq, synth, dev)
        if a.leg in ("all", "step"):
            dl = nvq.DecodeList(entries_for(layers, bits, nvq), M, a.act_group)
            sec = time_steps(dl, a.steps, a.warmup, torch)
            out["value"] = round(M / sec, 2)
            out["ms_per_step"] = round(sec * 1e3, 4)
            gbs = step_bytes / sec / 1e9
            out["config"]["step_hbm_gbs"] = round(gbs, 1)
            out["config"]["step_frac_of_peak"] = round(gbs / HBM_PEAK_GBS, 4)
            if a.extra_maps:
                for name in ("w4a8", "w4a16"):
                    b2 = block_bits(a.model, name, synth)
                    d2 = nvq.DecodeList(entries_for(layers, b2, nvq), M, a.act_group)
                    s2 = time_steps(d2, max(a.steps // 2, 1), max(a.warmup // 2, 1), torch)
                    out["config"]["tokens_per_s_all_" + name] = round(M / s2, 2)
        if a.leg in ("all", "roofline"):
            out["roofline"] = roofline_leg(layers, torch, nvq, synth)
        del layers
        torch.cuda.empty_cache()
    if a.leg in ("all", "cpu"):
        out["cpu_baseline"] = cpu_leg(a.model, bits, M, synth)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
