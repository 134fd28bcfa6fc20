#!/usr/bin/env python3
"""Benchmark of the decode-linear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--model llama-8b]
                    [--map mixed|w4a8|w4a16] [--leg all|step|cpu|calib|prefill] [--extra]
                    [--batch M] [--act-group 0|32] [--prefill-tokens T]

A step is one walk (one run of a prepared nvq plan = one launch of the
persistent streaming kernel) over every linear layer of one decode step at
batch 1 of the named Llama-shaped model: activation quantisation for the W4A8
layers, all GEMVs, lm_head (W4A16) where the model has one.  All weights and
activations are resident in HBM before the timed region; every layer reads its
own seeded input buffer.  Prints one JSON line (metric, value, roofline of the
persistent kernel from HIP events, cpu_baseline = the CPU oracle on a bounded sample).

--leg prefill is a separate measurement outside the headline metric: the seven linears of one
transformer block of the model for T tokens at once through nvq_gemm_w4a16 (dequantisation
fused into a bf16 matrix-core GEMM), reported in TFLOP/s against the dense bf16 MFMA peak.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
STREAM_KERNEL = "nvq::decode_stream_kernel"  # <per-group scales, paired rows>: one of three
GROUP_KERNEL = "nvq::gemv_mfma_group_kernel (+ nvq::quant_act_group_kernel)"
RING_KERNEL = ("nvq::gemv_mfma_ring_kernel (+ nvq::token_scale_group_kernel, "
               "nvq::operand_image_group_kernel)")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--model", default="llama-8b", choices=["llama-1b", "llama-3b", "llama-8b"])
    ap.add_argument("--map", default="mixed", choices=["mixed", "w4a8", "w4a16"])
    ap.add_argument("--prefill-tokens", type=int, default=4096)
    ap.add_argument("--leg", default="all", choices=["all", "step", "cpu", "calib", "prefill"],
                    help="calib: run only the plain copy kernel (1 GiB, for scaling profiler "
                         "byte counters)")
    ap.add_argument("--act-group", type=int, default=0, choices=[0, 32])
    ap.add_argument("--batch", type=int, default=1,
                    help="tokens per step (1 = the headline workload; 2..32 = the small-batch "
                         "variant on the matrix cores, one launch per phase)")
    ap.add_argument("--extra", action="store_true",
                    help="also time the all-W4A8 / all-W4A16 maps and the fully ordered chain")
    return ap.parse_args()


def block_bits(model, which, synth):
    nb = synth.MODELS[model][0]
    if which == "w4a8":
        return [0] * nb
    if which == "w4a16":
        return [1] * nb
    # seeded maps: 1B half W4A8, 3B a quarter W4A16, 8B half and half
    n16 = {"llama-1b": nb // 2, "llama-3b": nb // 4, "llama-8b": nb // 2}[model]
    return synth.make_precision_map(nb, n16)


def build_model(model, M, torch, nvq, synth, dev):
    """Generate and pack every layer on the GPU (one fp32 tensor alive at a time)."""
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


def chain_entries(layers, bits, model, torch, nvq, synth, dev):
    """The same linears wired up as a real decode step: RMSNorm in front of q/k/v and gate/up,
    the residual adds fused into those norms, SiLU(gate)*up in front of down, a final norm in
    front of lm_head; bf16 activations between the layers.  Attention itself is outside the
    path: o reads a seeded buffer of its own.  Every phase but o depends on its predecessor."""
    nb, hidden, kv, ffn, vocab = synth.MODELS[model]
    bf = dict(dtype=torch.bfloat16, device=dev)
    gen = torch.Generator().manual_seed(synth.BASE_SEED + 800_000)
    gam = lambda: (1.0 + 0.1 * torch.randn(hidden, generator=gen)).to(torch.bfloat16).to(dev)
    h = synth.make_activation(synth.activation_seed(10_000), 1, hidden, True, device=dev)
    down = None
    out = []
    by_block = {}
    for L in layers:
        by_block.setdefault(L["spec"].block, []).append(L)
    for b in range(nb):
        q, k, v, o, gate, up, dn = by_block[b]
        prec = bits[b]
        g1, g2 = gam(), gam()
        h_in = torch.zeros((1, hidden), **bf) if down is not None else None
        for L in (q, k, v):
            e = dict(qweight=L["qweight"], scales=L["scales"], precision=prec, x=h,
                     in_op=nvq.IN_RMSNORM, gamma=g1, eps=1e-5,
                     y=torch.zeros((1, L["spec"].N), **bf))
            if down is not None:
                e.update(x2=down, h_out=h_in)
            out.append(e)
        if down is not None:
            h = h_in
        attn = synth.make_activation(synth.activation_seed(20_000 + b), 1, hidden, True, device=dev)
        o_out = torch.zeros((1, hidden), **bf)
        out.append(dict(qweight=o["qweight"], scales=o["scales"], precision=prec, x=attn, y=o_out))
        h1 = torch.zeros((1, hidden), **bf)
        gbuf, ubuf = torch.zeros((1, ffn), **bf), torch.zeros((1, ffn), **bf)
        for L, y in ((gate, gbuf), (up, ubuf)):
            out.append(dict(qweight=L["qweight"], scales=L["scales"], precision=prec, x=h, x2=o_out,
                            in_op=nvq.IN_RMSNORM, gamma=g2, eps=1e-5, h_out=h1, y=y))
        h = h1
        down = torch.zeros((1, hidden), **bf)
        out.append(dict(qweight=dn["qweight"], scales=dn["scales"], precision=prec, x=gbuf, x2=ubuf,
                        in_op=nvq.IN_SILU_MUL, y=down))
    if -1 in by_block:
        (head,) = by_block[-1]
        out.append(dict(qweight=head["qweight"], scales=head["scales"], precision=nvq.W4A16, x=h,
                        x2=down, in_op=nvq.IN_RMSNORM, gamma=gam(), eps=1e-5,
                        y=torch.zeros((1, head["spec"].N), dtype=torch.float32, device=dev)))
    return out


def time_steps(dl, steps, warmup, torch):
    """K walks of the prepared plan.  Returns (wall seconds per step between two device
    synchronisations, seconds per launch from HIP events on the launch stream)."""
    dl.plan()
    for _ in range(warmup):
        dl.run_plan()
    st = torch.cuda.current_stream()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(st)
    for _ in range(steps):
        dl.run_plan()
    e1.record(st)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    if dl.plan_timed_out():
        raise RuntimeError("a wait inside the streaming kernel timed out; results invalid")
    return wall, e0.elapsed_time(e1) * 1e-3 / steps


def traffic_from_profile(model, which, batch, kind="group"):
    """HBM bytes per step measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a
    copy kernel of known size); read from the committed summary, None if it is not there."""
    name = ("decode_stream_%s_%s_pmc.md" % (model, which) if batch == 1 else
            "gemv_mfma_%s_%s_%s_batch%d_pmc.md" % (kind, model, which, batch))
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_leg(model, bits, M, synth, budget_s=20.0):
    """The oracle's walker on a bounded sample of the same workload: the first blocks of the
    model (as many as the time budget allows, at most four), inputs generated and packed on
    the CPU by the oracle itself."""
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
    oracle.decode_linears(host, M)                       # warm caches and the thread pool
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


MFMA_BF16_PEAK_TFLOPS = 2500.0


def prefill_leg(a, torch, nvq, synth):
    """One block's linears for T tokens through the fused-dequantisation GEMM."""
    dev = "cuda:0"
    torch.cuda.set_device(0)
    T = a.prefill_tokens
    specs = [sp for sp in synth.model_linears(a.model) if sp.block == 0]
    mats, xs = [], {}
    for sp in specs:
        W = synth.make_weight(synth.tensor_seed(0, sp.slot), sp.N, sp.K, device=dev)
        q, s = nvq.pack_int4(W)
        del W
        if sp.phase not in xs:
            xs[sp.phase] = synth.make_activation(synth.activation_seed(sp.phase), T, sp.K, True,
                                                 device=dev)
        mats.append((q, s, xs[sp.phase], torch.empty((T, sp.N), dtype=torch.bfloat16, device=dev)))
    flops = sum(2.0 * T * sp.N * sp.K for sp in specs)

    def block():
        for q, s, x, y in mats:
            nvq.gemm_w4a16(q, s, x, out=y)

    for _ in range(a.warmup // 10 + 2):
        block()
    torch.cuda.synchronize()
    reps = max(a.steps // 10, 5)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(reps):
        block()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / reps
    dev_s = e0.elapsed_time(e1) * 1e-3 / reps
    tf = flops / dev_s / 1e12
    print(json.dumps({
        "metric": "prefill linear-layer throughput, one %s block, %d tokens" % (a.model, T),
        "value": round(T / wall, 1), "unit": "tokens/s (one block's seven linears)", "n_gpus": 1,
        "steps": reps, "warmup": a.warmup // 10 + 2, "ms_per_step": round(wall * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 x bf16(int4 * fp16 scale) -> f32", "data": "synthetic",
        "config": {"workload": "%s block 0: q, k, v, o, gate, up, down as %d-token GEMMs with the "
                               "dequantisation fused in" % (a.model, T), "flop_per_step": flops},
        "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": None, "kernel": "nvq::gemm_w4a16_kernel", "launches": reps * len(mats),
                     "avg_launch_us": round(dev_s * 1e6 / len(mats), 2)}}))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path is a single-GPU decode "
              "step); --gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_21026_amd import nvq, synth

    if a.leg == "calib":
        torch.cuda.set_device(0)
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            nvq.stream_copy(dst, src)
        torch.cuda.synchronize()
        print(json.dumps({"calib": "nvq::stream_copy_kernel", "bytes_read": 1 << 30,
                          "bytes_written": 1 << 30, "launches": 5}))
        return
    if a.leg == "prefill":
        prefill_leg(a, torch, nvq, synth)
        return
    M = a.batch
    if not 1 <= M <= 32:
        print("bench.py: --batch must be 1..32", file=sys.stderr)
        sys.exit(2)
    bits = block_bits(a.model, a.map, synth)
    specs = synth.model_linears(a.model)
    step_bytes = sum(synth.weight_bytes(s.N, s.K) for s in specs)
    out = {
        "metric": "decode linear-layer tokens/s + achieved HBM GB/s (%% of peak), %s shapes, "
                  "batch %d" % (a.model.split("-")[1].upper(), M),
        "value": None, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 weights; int8 x int4 -> int32 (W4A8) and bf16 x int4 -> f32 (W4A16)",
        "data": "synthetic",
        "config": {"workload": "%s-shaped decode step, batch %d, %d linears in %s, precision map "
                               "%s (%d of %d blocks W4A16%s), own input buffer per layer" %
                               (a.model, M, len(specs),
                                "one launch" if M == 1 else "three launches", a.map,
                                sum(bits), len(bits),
                                ", lm_head W4A16" if specs[-1].block < 0 else ""),
                   "act_group": a.act_group, "weight_bytes_per_step": step_bytes},
    }
    if a.leg in ("all", "step"):
        if not torch.cuda.is_available():
            print("bench.py: no GPU visible", file=sys.stderr)
            sys.exit(3)
        dev = "cuda:0"
        torch.cuda.set_device(0)
        nvq.lib()
        layers = build_model(a.model, M, torch, nvq, synth, dev)
        dl = nvq.DecodeList(entries_for(layers, bits, nvq), M, a.act_group)
        info = dl.plan_info()
        wall, per_launch = time_steps(dl, a.steps, a.warmup, torch)
        out["value"] = round(M / wall, 2)
        out["ms_per_step"] = round(wall * 1e3, 4)
        out["config"]["plan"] = info
        gbs = step_bytes / per_launch / 1e9
        out["roofline"] = {
            "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4),
            "traffic": traffic_from_profile(a.model, a.map, M,
                                            "ring" if info["persistent_grouped"] else "group"),
            "kernel": (STREAM_KERNEL if info["streaming"] else
                       RING_KERNEL if info["persistent_grouped"] else
                       GROUP_KERNEL if info["grouped"] else "per-phase launches"),
            "launches": a.steps, "avg_launch_us": round(per_launch * 1e6, 2),  # per step
            "bytes_per_launch": step_bytes}
        dl.close()
        if a.extra:
            for name in ("w4a8", "w4a16"):
                d2 = nvq.DecodeList(entries_for(layers, block_bits(a.model, name, synth), nvq), M,
                                    a.act_group)
                w2, _ = time_steps(d2, max(a.steps // 2, 1), max(a.warmup // 2, 1), torch)
                out["config"]["tokens_per_s_all_" + name] = round(M / w2, 2)
                d2.close()
            # prefill helper: dense bf16 weights of the largest layer (reads 0.5625, writes 2 bytes
            # per weight)
            big = max(layers, key=lambda L: L["spec"].N * L["spec"].K)
            dense = nvq.dequant_bf16(big["qweight"], big["scales"])
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                nvq.dequant_bf16_into(big["qweight"], big["scales"], dense)
            e1.record()
            torch.cuda.synchronize()
            nw = big["spec"].N * big["spec"].K
            out["config"]["dequant_bf16_gbs"] = round(nw * 2.5625 * 20 / (e0.elapsed_time(e1) * 1e-3)
                                                      / 1e9, 1)
            del dense
            if M == 1:
                # the realistic dependent step: norms, residual adds and SiLU-multiply fused in
                d4 = nvq.DecodeList(chain_entries(layers, bits, a.model, torch, nvq, synth, dev), 1,
                                    a.act_group)
                w4, _ = time_steps(d4, max(a.steps // 2, 1), max(a.warmup // 2, 1), torch)
                out["config"]["tokens_per_s_block_chain"] = round(1 / w4, 2)
                out["config"]["block_chain_plan"] = d4.plan_info()
                d4.close()
            d3 = nvq.DecodeList(entries_for(layers, bits, nvq), M, a.act_group, ordered=True)
            w3, _ = time_steps(d3, max(a.steps // 2, 1), max(a.warmup // 2, 1), torch)
            out["config"]["tokens_per_s_ordered_chain"] = round(M / w3, 2)
            d3.close()
        del layers
        torch.cuda.empty_cache()
    if a.leg in ("all", "cpu"):
        out["cpu_baseline"] = cpu_leg(a.model, bits, M, synth)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
