#!/usr/bin/env python3
"""Benchmark of the decode-linear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--model llama-8b|llama-3b|llama-1b]
                    [--map mixed|w4a8|w4a16] [--batch M] [--act-group 0|32] [--copies C]
                    [--leg all|step|cpu|cpu-full|config1|ceiling|calib|prefill|trace]

A step is one walk (one run of a prepared nvq plan = one launch of the persistent streaming
kernel at batch 1) over every linear layer of one decode step of the named Llama-shaped model:
activation quantisation for the W4A8 layers, all GEMVs, lm_head (W4A16) where the model has one.
All weights and activations are resident in HBM before the timed region.  One JSON line:

  value / ms_per_step / roofline   the workload the benchmark's metric is quoted on: every layer
                                   reads its own seeded input buffer, phases in list order
  config.*_block_chain             the same linears wired up as a real decode step (norms,
                                   residual adds, SiLU-multiply fused in; 3 of 4 phases per block
                                   wait for the phase before them)
  config.*_ordered_chain           the independent buffers with every phase forced to wait for
                                   its predecessor
  config.*_all_w4a8 / _all_w4a16   the two uniform precision maps
  roofline.ceiling_gbs             a plain streaming read of 4 GiB on this machine, this run
  cpu_baseline                     the CPU oracle on a bounded sample of the same workload

Every launch of the timed region has its own pair of HIP events on the launch stream
(roofline.avg/min/median_launch_us); before the warm-up an untimed loop runs until the launch time
stops falling (config.clock_ramp), so a short run measures the machine at its clocks.

Other legs: `config1` = BASELINE configs[0] (one 2048 x 2048 layer, both precisions, rotated
over 512 copies, and the warm single-buffer figure); `cpu-full` = the oracle over the whole step
on all cores and on one; `prefill` = one block's linears for T tokens through nvq_gemm_w4a16;
`ceiling` = the streaming read alone; `calib` = a plain copy for scaling profiler byte counters.
"""
import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
STREAM_KERNEL = "nvq::decode_stream_kernel"  # <per-group scales, paired rows, mail>
GROUP_KERNEL = "nvq::gemv_mfma_group_kernel (+ nvq::quant_act_group_kernel)"
RING_KERNEL = ("nvq::gemv_mfma_ring_kernel (+ nvq::token_scale_group_kernel, "
               "nvq::operand_image_group_kernel)")
# model copies a step rotates over so that no weight byte is read out of the 256 MB
# Infinity Cache or the L2s (at least 1 GB of distinct bytes between two uses)
DEFAULT_COPIES = {"llama-1b": 3, "llama-3b": 2, "llama-8b": 1}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--model", default="llama-8b", choices=["llama-1b", "llama-3b", "llama-8b"])
    ap.add_argument("--map", default="mixed", choices=["mixed", "w4a8", "w4a16"])
    ap.add_argument("--prefill-tokens", type=int, default=4096)
    ap.add_argument("--leg", default="all",
                    choices=["all", "step", "cpu", "cpu-full", "config1", "ceiling", "calib", "trace",
                             "prefill"])
    ap.add_argument("--act-group", type=int, default=0, choices=[0, 32])
    ap.add_argument("--batch", type=int, default=1,
                    help="tokens per step (1 = the headline workload; 2..32 = the small-batch "
                         "variant on the matrix cores)")
    ap.add_argument("--copies", type=int, default=0,
                    help="model copies the timed steps rotate over (0 = enough for 1 GB of "
                         "distinct weight bytes between two uses of a byte)")
    ap.add_argument("--extra", action="store_true", help="(kept for older command lines: the "
                    "chain and uniform-map figures are now part of the default line)")
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


def build_model(model, M, torch, nvq, synth, dev, copy=0):
    """Generate and pack every layer on the GPU (one fp32 tensor alive at a time).  Copy c > 0
    is another model of the same shapes (other seeds): for rotating over more bytes than the
    caches hold."""
    specs = synth.model_linears(model)
    layers = []
    xbuf = {}
    for sp in specs:
        seed = synth.tensor_seed(sp.block if sp.block >= 0 else 999, sp.slot) + 7_000_000 * copy
        W = synth.make_weight(seed, sp.N, sp.K, device=dev)
        q, s = nvq.pack_int4(W)
        torch.cuda.synchronize()
        del W
        if sp.phase not in xbuf:
            xbuf[sp.phase] = synth.make_activation(synth.activation_seed(sp.phase) + 7_000 * copy,
                                                   M, sp.K, True, device=dev)
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


def clock_ramp(dls, torch, budget_s=0.25):
    """Untimed: walk until the time of a launch stops falling (the clocks of an idle GPU take
    some milliseconds of load to come up), for at most `budget_s`.  Returns what it saw."""
    st = torch.cuda.current_stream()
    t_end = time.perf_counter() + budget_s
    first = last = best = None
    launches = 0
    while time.perf_counter() < t_end:
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(9)]
        for i in range(8):
            ev[i].record(st)
            dls[launches % len(dls)].run_plan()
            launches += 1
        ev[8].record(st)
        torch.cuda.synchronize()
        cur = min(ev[i].elapsed_time(ev[i + 1]) for i in range(8)) * 1e3
        first = cur if first is None else first
        if best is not None and cur > best * 0.995 and launches >= 24:
            last = cur
            break
        best = cur if best is None else min(best, cur)
        last = cur
    return {"launches": launches, "first_us": round(first, 2), "last_us": round(last, 2)}


def time_steps(dls, steps, warmup, torch):
    """K walks of the prepared plans in `dls`, taken in turn (one plan: the same walk K times).
    Returns (wall seconds per step between two device synchronisations, list of seconds per
    launch from a HIP event pair per launch on the launch stream)."""
    if not isinstance(dls, (list, tuple)):
        dls = [dls]
    for d in dls:
        d.plan()
    for i in range(warmup):
        dls[i % len(dls)].run_plan()
    st = torch.cuda.current_stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i].record(st)
        dls[i % len(dls)].run_plan()
    ev[steps].record(st)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    for d in dls:
        if d.plan_timed_out():
            raise RuntimeError("a wait inside the persistent kernel gave up (code %#x); results "
                               "invalid" % d.status_code)
    per = [ev[i].elapsed_time(ev[i + 1]) * 1e-3 for i in range(steps)]
    return wall, per


def traffic_from_profile(model, which, batch, kind="group"):
    """HBM bytes per step measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by a
    copy kernel of known size); read from the committed summary, None if it is not there."""
    name = ("decode_stream_%s_%s_pmc.md" % (model, which) if batch == 1 else
            "gemv_mfma_%s_%s_%s_batch%d_pmc.md" % (kind, model, which, batch))
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read())
        return (float(m.group(1)) if m else None), "profiles/" + name
    except OSError:
        return None, None


def ceiling_gbs(torch, nvq, gib=4):
    """A plain streaming read (non-temporal 128-bit loads, nvq_stream_read) of `gib` GiB: what
    this machine's HBM delivers to a kernel that does nothing else.  Best of five launches."""
    buf = torch.empty(gib << 30, dtype=torch.uint8, device="cuda:0")
    buf.random_(0, 255)
    sink = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    for _ in range(3):
        nvq.stream_read(buf, sink)
    best = None
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        nvq.stream_read(buf, sink)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) * 1e-3
        best = t if best is None else min(best, t)
    del buf
    torch.cuda.empty_cache()
    return (gib << 30) / best / 1e9


def cpu_sample(model, bits, M, synth, budget_s=20.0):
    """The oracle's walker on a bounded sample of the same workload: the first blocks of the
    model (at most two) and, where the model has one, the first rows of lm_head, in the
    proportion of the whole step; inputs generated and packed on the CPU by the oracle itself."""
    import numpy as np
    import torch
    import oracle
    all_specs = synth.model_linears(model)
    specs = [s for s in all_specs if s.block >= 0]
    nb = synth.MODELS[model][0]
    total_w = sum(s.N * s.K for s in all_specs)
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
        if time.perf_counter() - t_gen0 > budget_s * 0.2 or blocks >= 2:
            break
    head_rows = 0
    heads = [s for s in all_specs if s.block < 0]
    if heads:
        sp = heads[0]
        # lm_head rows in the proportion blocks / nb of the whole matrix
        head_rows = max(256, sp.N * blocks // nb // 256 * 256)
        W = synth.make_weight(synth.tensor_seed(999, sp.slot), head_rows, sp.K)
        q, s = oracle.pack_int4(W.numpy())
        x = synth.make_activation(synth.activation_seed(sp.phase), M, sp.K)
        host.append(dict(qweight=q, scales=s, x=x.view(torch.int16).numpy().view(np.uint16),
                         precision=1))
        sample_w += head_rows * sp.K
    oracle.decode_linears(host, M)                       # warm caches and the thread pool
    reps, t0 = 0, time.perf_counter()
    while reps < 3 or (time.perf_counter() - t0 < budget_s * 0.5 and reps < 50):
        oracle.decode_linears(host, M)
        reps += 1
    t = (time.perf_counter() - t0) / reps
    step_s = t * total_w / sample_w
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": round(M / step_s, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "oracle walker over the first %d of %d blocks%s (%d of %d weights), %d reps, "
                      "step time scaled by weight count" %
                      (blocks, nb, " and the first %d rows of lm_head" % head_rows if head_rows
                       else "", sample_w, total_w, reps),
            "gbs": round(total_w * 0.5625 / step_s / 1e9, 2)}


def cpu_full(model, bits, M, synth):
    """The oracle over the whole step (every linear, lm_head included): best of three on all
    cores, and once on one core."""
    import numpy as np
    import torch
    import oracle
    host, total_w = [], 0
    t_gen = time.perf_counter()
    for sp in synth.model_linears(model):
        W = synth.make_weight(synth.tensor_seed(sp.block if sp.block >= 0 else 999, sp.slot),
                              sp.N, sp.K)
        q, s = oracle.pack_int4(W.numpy())
        del W
        x = synth.make_activation(synth.activation_seed(sp.phase), M, sp.K)
        host.append(dict(qweight=q, scales=s, x=x.view(torch.int16).numpy().view(np.uint16),
                         precision=1 if sp.block < 0 else bits[sp.block]))
        total_w += sp.N * sp.K
        if len(host) % 14 == 0:  # (a line a minute or so: the generation takes minutes)
            print("cpu-full: %d linears generated and packed, %.0f s" %
                  (len(host), time.perf_counter() - t_gen), file=sys.stderr, flush=True)
    t_gen = time.perf_counter() - t_gen
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    oracle.decode_linears(host, M)
    best = None
    for _ in range(3):
        t0 = time.perf_counter()
        oracle.decode_linears(host, M)
        t = time.perf_counter() - t0
        best = t if best is None else min(best, t)
    # one core: the OpenMP runtime the oracle's library is linked against is told so
    import ctypes
    gomp = ctypes.CDLL("libgomp.so.1")
    gomp.omp_set_num_threads(1)
    t0 = time.perf_counter()
    oracle.decode_linears(host, M)
    single = time.perf_counter() - t0
    gomp.omp_set_num_threads(threads)
    return {"value": round(M / best, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "oracle walker over all %d linears of the step (%d weights), best of 3"
                      % (len(host), total_w),
            "gbs": round(total_w * 0.5625 / best / 1e9, 2),
            "single_thread": {"value": round(M / single, 4), "unit": "tokens/s", "cores": 1,
                              "gbs": round(total_w * 0.5625 / single / 1e9, 3)},
            "generate_and_pack_s": round(t_gen, 1)}


MFMA_BF16_PEAK_TFLOPS = 2500.0


def trace_leg(a, torch, nvq, synth):
    """Where the time of the dependent decode chain goes: the timestamps nvq_plan_trace takes in
    every workgroup (100 MHz clock), per kind of phase, medians over the blocks."""
    import numpy as np
    dev = "cuda:0"
    torch.cuda.set_device(0)
    bits = block_bits(a.model, a.map, synth)
    layers = build_model(a.model, 1, torch, nvq, synth, dev)
    entries = chain_entries(layers, bits, a.model, torch, nvq, synth, dev)
    dl = nvq.DecodeList(entries, 1, a.act_group)
    P = dl.plan_info()["phases"]
    wall, per = time_steps(dl, a.steps, a.warmup, torch)
    _, phases = nvq.plan_describe([dl.arr[i] for i in range(dl.n)], 1, a.act_group)
    kinds = [layers[ph["first"]]["spec"].name.split(".")[-1] for ph in phases]
    kinds = ["qkv" if k == "q" else "gate/up" if k == "gate" else k for k in kinds]
    nwg = torch.cuda.get_device_properties(0).multi_processor_count
    buf = torch.zeros(nwg * P * 8, dtype=torch.int64, device=dev)
    dl.trace(buf)
    dl.run_plan()
    torch.cuda.synchronize()
    buf.zero_()
    dl.run_plan()
    torch.cuda.synchronize()
    dl.trace(None)
    t = buf.cpu().numpy().reshape(nwg, P, 8).astype(np.float64) * 0.01      # us
    t = np.where(t > 0, t, np.nan)
    with np.errstate(all="ignore"):
        import warnings
        warnings.simplefilter("ignore")
        here, staged, done = t[:, :, 3], t[:, :, 2], t[:, :, 6]
        med = lambda x: np.nanmedian(x, axis=0)
        last_done = np.nanmax(done, axis=0)
        rows = {}
        for p in range(2, P):
            rows.setdefault(kinds[p], []).append((
                med(here)[p] - last_done[p - 1],          # operands here after the last producer
                med(staged)[p] - med(here)[p],            # image built
                med(done)[p] - med(staged)[p],            # rows, median workgroup's last wave
                last_done[p] - med(done)[p],              # the slowest workgroup behind the median
                last_done[p] - last_done[p - 1]))         # the phase, end to end
        out = {"trace": "%s-shaped dependent chain (block chain), map %s" % (a.model, a.map),
               "ms_per_step": round(wall * 1e3, 4), "phases": P,
               "kernel_us": round(float(np.nanmax(done[:, -1]) - np.nanmin(t[:, 0, 5])), 1),
               "unit": "us, medians over the phases of a kind",
               "columns": ["operands_after_last_producer", "image_build", "rows_median_workgroup",
                           "slowest_workgroup_behind_median", "phase_end_to_end", "count"]}
        for k, v in rows.items():
            v = np.array(v)
            out[k] = [None if np.isnan(x) else round(float(x), 2)
                      for x in np.nanmedian(v, axis=0)] + [len(v)]
    print(json.dumps(out))


def prefill_leg(a, torch, nvq, synth):
    """One block's linears for T tokens through the fused-dequantisation GEMM: as four launches
    (the rows of q, k, v in one weight matrix, likewise gate and up: they read the same input) and
    as seven (one per projection)."""
    dev = "cuda:0"
    torch.cuda.set_device(0)
    T = a.prefill_tokens
    specs = [sp for sp in synth.model_linears(a.model) if sp.block == 0]
    packed, xs = {}, {}
    for sp in specs:
        W = synth.make_weight(synth.tensor_seed(0, sp.slot), sp.N, sp.K, device=dev)
        packed[sp.slot] = nvq.pack_int4(W) + (sp,)
        del W
        if sp.phase not in xs:
            xs[sp.phase] = synth.make_activation(synth.activation_seed(sp.phase), T, sp.K, True,
                                                 device=dev)
    flops = sum(2.0 * T * sp.N * sp.K for sp in specs)

    def launches(groups):
        out = []
        for g in groups:
            q = torch.cat([packed[slot][0] for slot in g], 0).contiguous()
            s = torch.cat([packed[slot][1] for slot in g], 0).contiguous()
            sp = packed[g[0]][2]
            assert all(packed[slot][2].phase == sp.phase for slot in g)
            out.append((q, s, xs[sp.phase], torch.empty((T, q.shape[0]), dtype=torch.bfloat16,
                                                        device=dev)))
        return out

    slots = [sp.slot for sp in specs]
    by_phase = {}
    for sp in specs:
        by_phase.setdefault(sp.phase, []).append(sp.slot)
    reps = max(a.steps // 10, 5)
    warm = a.warmup // 10 + 2

    def timed(mats):
        def block():
            for q, s, x, y in mats:
                nvq.gemm_w4a16(q, s, x, out=y)
        for _ in range(warm):
            block()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(reps):
            block()
        e1.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps, e0.elapsed_time(e1) * 1e-3 / reps

    fused = launches(list(by_phase.values()))
    wall, dev_s = timed(fused)
    single = launches([[slot] for slot in slots])
    wall7, dev7 = timed(single)
    tf, tf7 = flops / dev_s / 1e12, flops / dev7 / 1e12
    # For scale, the route of the paper's kernel table on this machine: the dequantisation kernel
    # (nvq_dequant_bf16) and the library's dense bf16 GEMM on its output, the same four launches;
    # with the dense weights made once beforehand (GEMM only) and made anew in every step.
    dense = [nvq.dequant_bf16(q, s) for q, s, _, _ in fused]

    def timed_fn(fn):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    def lib_only():
        for (q, s, x, y), w in zip(fused, dense):
            torch.matmul(x, w.t(), out=y)

    def lib_with_dequant():
        for (q, s, x, y), w in zip(fused, dense):
            nvq.dequant_bf16_into(q, s, w)
            torch.matmul(x, w.t(), out=y)

    lib_s, libd_s = timed_fn(lib_only), timed_fn(lib_with_dequant)
    print(json.dumps({
        "metric": "prefill linear-layer throughput, one %s block, %d tokens" % (a.model, T),
        "value": round(T / wall, 1), "unit": "tokens/s (one block's linears)", "n_gpus": 1,
        "steps": reps, "warmup": warm, "ms_per_step": round(wall * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 x bf16(int4 * fp16 scale) -> f32", "data": "synthetic",
        "config": {"workload": "%s block 0 as %d-token GEMMs with the dequantisation fused in: "
                               "q+k+v, o, gate+up, down (%d launches)" % (a.model, T, len(fused)),
                   "flop_per_step": flops},
        "roofline": {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": None, "kernel": "nvq::gemm_w4a16_wide_kernel",
                     "launches": reps * len(fused), "avg_launch_us": round(dev_s * 1e6 / len(fused), 2)},
        "one_launch_per_projection": {"launches": len(single), "ms_per_step": round(wall7 * 1e3, 4),
                                      "achieved": round(tf7, 1), "unit": "TFLOP/s",
                                      "frac": round(tf7 / MFMA_BF16_PEAK_TFLOPS, 4)},
        "dequantise_then_library_gemm": {
            "gemm_only_tflops": round(flops / lib_s / 1e12, 1),
            "with_dequantisation_each_step_tflops": round(flops / libd_s / 1e12, 1),
            "ms_per_step": [round(lib_s * 1e3, 4), round(libd_s * 1e3, 4)]}}))


def config1_leg(a, torch, nvq, synth):
    """BASELINE configs[0]: one 2048 x 2048 layer at batch 1, both precisions.  Cold: 512
    copies of the layer (1.2 GB: more than the caches hold), as single calls (a W4A8 call is the
    activation quantisation and the GEMV: two launches) and as one list of 512 layers in one
    launch of the persistent kernel.  Warm: the same call on one buffer over and over (2.4 MB:
    resident in the L2 / Infinity Cache; labelled so)."""
    dev = "cuda:0"
    torch.cuda.set_device(0)
    N = K = 2048
    copies = 512
    layer_bytes = synth.weight_bytes(N, K)
    W = synth.make_weight(synth.tensor_seed(0, 0), N, K, device=dev)
    q0, s0 = nvq.pack_int4(W)
    qs = torch.empty((copies,) + tuple(q0.shape), dtype=q0.dtype, device=dev)
    ss = torch.empty((copies,) + tuple(s0.shape), dtype=s0.dtype, device=dev)
    gen = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 31)
    # (the copies need not be valid quantisations of anything: random nibbles, the one real
    # layer's scales; every byte distinct memory)
    qs.random_(0, 256, generator=gen)
    ss[:] = s0
    qs[0], ss[0] = q0, s0
    x = synth.make_activation(synth.activation_seed(0), 1, K, False, device=dev)
    y = torch.empty((1, N), dtype=torch.float32, device=dev)
    res = {}

    def timed(fn, reps):
        for _ in range(3):
            fn(0)
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(reps):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / reps
            best = t if best is None else min(best, t)
        return best

    def w4a16(i):
        nvq.gemv_w4a16(qs[i % copies], ss[i % copies], x, out=y)

    codes = nvq.quant_act_i8(x)

    def w4a8(i):
        xq, xs, gs = nvq.quant_act_i8(x, out=codes)
        nvq.gemv_w4a8(qs[i % copies], ss[i % copies], xq, xs, gs, out=y)

    for name, fn in (("w4a16", w4a16), ("w4a8", w4a8)):
        cold = timed(fn, copies)
        warm = timed(lambda i: fn(0), copies)
        res[name] = {
            "single_calls_cold": {"gemv_per_s": round(1 / cold, 1), "us": round(cold * 1e6, 2),
                                  "gbs": round(layer_bytes / cold / 1e9, 1),
                                  "frac_of_hbm_peak": round(layer_bytes / cold / 1e9 / HBM_PEAK_GBS, 4)},
            "single_calls_warm_cache_resident": {"gemv_per_s": round(1 / warm, 1),
                                                 "us": round(warm * 1e6, 2),
                                                 "gbs": round(layer_bytes / warm / 1e9, 1)}}
    # one launch over the 512 copies (each its own output), both precisions
    ys = torch.empty((copies, 1, N), dtype=torch.float32, device=dev)
    for name, prec in (("w4a16", nvq.W4A16), ("w4a8", nvq.W4A8)):
        dl = nvq.DecodeList([dict(qweight=qs[i], scales=ss[i], x=x, y=ys[i], precision=prec)
                             for i in range(copies)], 1, a.act_group)
        wall, per = time_steps(dl, max(a.steps // 10, 5), max(a.warmup // 10, 2), torch)
        t = statistics.median(per) / copies
        res[name]["one_launch_512_layers_cold"] = {
            "gemv_per_s": round(1 / t, 1), "us_per_layer": round(t * 1e6, 3),
            "gbs": round(layer_bytes / t / 1e9, 1),
            "frac_of_hbm_peak": round(layer_bytes / t / 1e9 / HBM_PEAK_GBS, 4)}
        dl.close()
    print(json.dumps({
        "metric": "single linear layer 2048 x 2048, batch 1: GEMV/s and HBM GB/s",
        "value": res["w4a8"]["one_launch_512_layers_cold"]["gemv_per_s"], "unit": "GEMV/s",
        "n_gpus": 1, "higher_is_better": True, "vs_baseline": None, "data": "synthetic",
        "dtype": "int4 weights; int8 x int4 -> int32 (W4A8) and bf16 x int4 -> f32 (W4A16)",
        "config": {"workload": "one 2048 x 2048 layer (%d bytes), batch 1, N(0,1) input without "
                               "outliers; cold = rotated over %d copies (%.2f GB)" %
                               (layer_bytes, copies, copies * layer_bytes / 1e9),
                   "results": res}}))


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
    if a.leg == "ceiling":
        torch.cuda.set_device(0)
        g = ceiling_gbs(torch, nvq)
        print(json.dumps({"ceiling": "nvq::stream_read_kernel, 4 GiB, best of 5",
                          "gbs": round(g, 1), "frac_of_hbm_peak": round(g / HBM_PEAK_GBS, 4)}))
        return
    if a.leg == "prefill":
        prefill_leg(a, torch, nvq, synth)
        return
    if a.leg == "config1":
        config1_leg(a, torch, nvq, synth)
        return
    if a.leg == "trace":
        trace_leg(a, torch, nvq, synth)
        return
    M = a.batch
    if not 1 <= M <= 32:
        print("bench.py: --batch must be 1..32", file=sys.stderr)
        sys.exit(2)
    bits = block_bits(a.model, a.map, synth)
    specs = synth.model_linears(a.model)
    step_bytes = sum(synth.weight_bytes(s.N, s.K) for s in specs)
    copies = a.copies if a.copies > 0 else DEFAULT_COPIES[a.model]
    out = {
        "metric": "decode linear-layer tokens/s + achieved HBM GB/s (%% of peak), %s shapes, "
                  "batch %d" % (a.model.split("-")[1].upper(), M),
        "value": None, "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 weights; int8 x int4 -> int32 (W4A8) and bf16 x int4 -> f32 (W4A16)",
        "data": "synthetic",
        "config": {"workload": "%s-shaped decode step, batch %d, %d linears in %s, precision map "
                               "%s (%d of %d blocks W4A16%s), own input buffer per layer%s" %
                               (a.model, M, len(specs),
                                "one launch" if M == 1 else "three launches", a.map,
                                sum(bits), len(bits),
                                ", lm_head W4A16" if specs[-1].block < 0 else "",
                                ", steps rotate over %d model copies (%.2f GB)" %
                                (copies, copies * step_bytes / 1e9) if copies > 1 else ""),
                   "act_group": a.act_group, "weight_bytes_per_step": step_bytes,
                   "model_copies": copies},
    }
    if a.leg in ("all", "step"):
        if not torch.cuda.is_available():
            print("bench.py: no GPU visible", file=sys.stderr)
            sys.exit(3)
        dev = "cuda:0"
        torch.cuda.set_device(0)
        nvq.lib()
        models = [build_model(a.model, M, torch, nvq, synth, dev, c) for c in range(copies)]
        layers = models[0]
        dls = [nvq.DecodeList(entries_for(m, bits, nvq), M, a.act_group) for m in models]
        for d in dls:
            d.plan()
        info = dls[0].plan_info()
        out["config"]["clock_ramp"] = clock_ramp(dls, torch)
        wall, per = time_steps(dls, a.steps, a.warmup, torch)
        per_launch = sum(per) / len(per)
        out["value"] = round(M / wall, 2)
        out["ms_per_step"] = round(wall * 1e3, 4)
        out["config"]["plan"] = info
        gbs = step_bytes / per_launch / 1e9
        traffic, traffic_src = traffic_from_profile(
            a.model, a.map, M, "ring" if info["persistent_grouped"] else "group")
        out["roofline"] = {
            "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4),
            "traffic": traffic, "traffic_source": traffic_src,
            "kernel": (STREAM_KERNEL if info["streaming"] else
                       RING_KERNEL if info["persistent_grouped"] else
                       GROUP_KERNEL if info["grouped"] else "per-phase launches"),
            "launches": a.steps, "avg_launch_us": round(per_launch * 1e6, 2),  # per step
            "min_launch_us": round(min(per) * 1e6, 2),
            "median_launch_us": round(statistics.median(per) * 1e6, 2),
            "bytes_per_launch": step_bytes}
        if copies > 1:
            # the same walk on one copy over and over: partly out of the caches
            w1, p1 = time_steps(dls[0], a.steps, a.warmup, torch)
            out["config"]["single_copy_cache_resident"] = {
                "tokens_per_s": round(M / w1, 2),
                "frac_of_hbm_peak": round(step_bytes / statistics.median(p1) / 1e9 / HBM_PEAK_GBS, 4)}
        for d in dls[1:]:
            d.close()
        del dls[1:], models[1:]

        def side(entries, ordered=False):
            d = nvq.DecodeList(entries, M, a.act_group, ordered=ordered)
            w, p = time_steps(d, a.steps, a.warmup, torch)
            inf = d.plan_info()
            d.close()
            med = statistics.median(p)
            return {"tokens_per_s": round(M / w, 2), "ms_per_step": round(w * 1e3, 4),
                    "median_launch_us": round(med * 1e6, 2),
                    "frac_of_hbm_peak": round(step_bytes / med / 1e9 / HBM_PEAK_GBS, 4),
                    "waits": inf["waits"]}

        if a.leg == "all":
            if M == 1:
                r = side(chain_entries(layers, bits, a.model, torch, nvq, synth, dev))
                out["config"]["tokens_per_s_block_chain"] = r["tokens_per_s"]
                out["config"]["block_chain_frac"] = r["frac_of_hbm_peak"]
                out["config"]["block_chain"] = r
            r = side(entries_for(layers, bits, nvq), ordered=True)
            out["config"]["tokens_per_s_ordered_chain"] = r["tokens_per_s"]
            out["config"]["ordered_chain_frac"] = r["frac_of_hbm_peak"]
            out["config"]["ordered_chain"] = r
            if a.map == "mixed":
                for name in ("w4a8", "w4a16"):
                    r = side(entries_for(layers, block_bits(a.model, name, synth), nvq))
                    out["config"]["tokens_per_s_all_" + name] = r["tokens_per_s"]
                    out["config"]["all_%s_frac" % name] = r["frac_of_hbm_peak"]
        dls[0].close()
        del layers, models, dls
        torch.cuda.empty_cache()
        if a.leg == "all":
            g = ceiling_gbs(torch, nvq)
            out["roofline"]["ceiling_gbs"] = round(g, 1)
            out["roofline"]["frac_of_ceiling"] = round(gbs / g, 4)
    if a.leg in ("all", "cpu"):
        out["cpu_baseline"] = cpu_sample(a.model, bits, M, synth)
    if a.leg == "cpu-full":
        out["cpu_baseline"] = cpu_full(a.model, bits, M, synth)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
