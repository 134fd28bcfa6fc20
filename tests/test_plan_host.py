"""Host-side planning of the decode walk, checked without a GPU through
nvq_plan_describe: phase grouping, dependency analysis, the dealing of rows to the
streaming waves and the placement of activation images in the circular LDS area.
The pointers in the layer list are made up (they are compared, never followed)."""
import numpy as np
import pytest

from paper_2604_21026_amd import nvq, synth

AREA = 59392          # bytes of the LDS image area (decode_stream.h)


class Arena:
    """Hands out made-up, 256-byte aligned device addresses."""

    def __init__(self):
        self.at = 1 << 20

    def take(self, nbytes):
        p = self.at
        self.at += (int(nbytes) + 255) // 256 * 256
        return p


def linear(a, N, K, x, y=None, prec=0, y_f32=True, M=1, **kw):
    y = y if y is not None else a.take(M * N * 4)
    return nvq.Linear(a.take(N * K // 2), a.take(N * (K // 32) * 2), N, K, x, y,
                      nvq.F32 if y_f32 else nvq.BF16, prec, kw.get("in_op", 0),
                      kw.get("eps", 0.0), kw.get("x2"), kw.get("gamma"), kw.get("h_out"))


def model_list(model, bits):
    a = Arena()
    xs, out = {}, []
    for sp in synth.model_linears(model):
        if sp.phase not in xs:
            xs[sp.phase] = a.take(sp.K * 2)
        out.append(linear(a, sp.N, sp.K, xs[sp.phase], prec=1 if sp.block < 0 else bits[sp.block]))
    return out


def rows_of_wave(ph, j, waves):
    """First row and row count of wave j as the kernel computes them."""
    k = (j - ph["rows_rot"]) % waves
    more = min(k, ph["rows_extra"])
    u = ph["row_unit"]
    first, count = u * (k * ph["rows_base"] + more), u * (ph["rows_base"] + (1 if k < ph["rows_extra"] else 0))
    return first, max(0, min(count, ph["rows"] - first))        # the last unit may be short


@pytest.mark.parametrize("model", ["llama-1b", "llama-3b", "llama-8b"])
def test_rows_are_dealt_once_each_and_evenly(model):
    nb = synth.MODELS[model][0]
    layers = model_list(model, synth.make_precision_map(nb, nb // 2))
    waves, phases = nvq.plan_describe(layers, 1)
    assert waves == 256 * 12
    specs = synth.model_linears(model)
    assert len(phases) == len({s.phase for s in specs})
    load = np.zeros(waves)
    biggest_unit = 0
    for ph in phases:
        assert ph["wait"] == -1 and ph["publish"] == 0          # every phase reads its own buffer
        K = layers[ph["first"]].K
        # rows of 96 groups (K = 3072) are streamed in pairs; a phase too short to give
        # every wave 12 chunks deals its rows in larger units to fewer waves
        assert ph["pair_stream"] == (2 if K == 3072 else 0)
        u, gpl = ph["row_unit"], (K // 32 + 63) // 64
        chunks_per_row = 1.5 if K == 3072 else gpl
        step = max(ph["pair_stream"], 1)
        want = step
        while want * chunks_per_row < 12:
            want += step
        assert u == (want if ph["rows"] < want * waves else step)
        assert ph["rows_base"] * waves + ph["rows_extra"] == -(-ph["rows"] // u)
        assert 0 <= ph["rows_rot"] < waves
        K = layers[ph["first"]].K
        covered = np.zeros(ph["rows"], np.int32)
        for j in range(waves):
            first, count = rows_of_wave(ph, j, waves)
            covered[first:first + count] += 1
            load[j] += count * (K // 32) * 18
        assert covered.min() == 1 and covered.max() == 1         # every row exactly once
        biggest_unit = max(biggest_unit, u * (K // 32) * 18)
    # the heaviest wave (it ends the step) carries at most 3 % more than the average, the
    # lightest at most 12 % less
    assert biggest_unit > 0
    assert load.max() <= 1.03 * load.mean() and load.min() >= 0.88 * load.mean()


@pytest.mark.parametrize("model,ordered", [("llama-1b", False), ("llama-3b", False),
                                           ("llama-8b", False), ("llama-1b", True)])
def test_skip_table_passes_exactly_the_phases_without_rows_and_barriers(model, ordered):
    nb = synth.MODELS[model][0]
    layers = model_list(model, synth.make_precision_map(nb, nb // 2))
    waves, phases = nvq.plan_describe(layers, 1, ordered=ordered)
    table = nvq.plan_describe_skips(layers, 1, ordered=ordered)
    P = len(phases)
    assert table.shape[0] == waves + waves // 12 and table.shape[1] >= P + 4 and table.shape[1] % 4 == 0
    skips, wg_passes = table[:waves], table[waves:]
    assert not skips[:, P:].any()                       # the padding reads as "do not pass"
    # which wave works in which phase, from the dealing alone
    nwg = waves // 12
    active = np.zeros((P, waves), bool)
    for p, ph in enumerate(phases):
        for j in range(waves):
            _, count = rows_of_wave(ph, j, waves)
            g = (j % nwg) * 12 + j // nwg if ph["spread"] else j
            active[p, g] = (count > 0 or ph["wait"] >= 0 or ph["publish"] == 1 or
                            (ph["mail"] & 3) != 0)
    # a workgroup leaves a phase's image alone exactly if none of its 12 waves works in it
    assert np.array_equal(wg_passes[:, :P].T, ~active.reshape(P, nwg, 12).any(axis=2))
    assert not wg_passes[:, P:].any()
    if ordered:
        assert not skips.any() and not wg_passes.any()  # every phase has barriers
        return
    assert skips.any()
    for g in range(0, waves, 37):                       # a sample of the waves
        for p in range(P):
            run = 0
            while p + run < P and not active[p + run, g]:
                run += 1
            assert skips[g, p] == min(run, 255)
    # a wave that follows its row of the table visits exactly the phases it works in
    for g in (0, 1, 11, 12, 1000, waves - 1):
        p, seen = 0, []
        while p < P:
            p += int(skips[g, p])
            if p < P:
                seen.append(p)
                p += 1
        assert seen == [p for p in range(P) if active[p, g]]


@pytest.mark.parametrize("seed", range(12))
def test_random_lists_deal_every_row_once_and_skip_only_idle_phases(seed):
    """Random shapes (rows from 1 to 40000, K any multiple of 32 the kernel takes, several
    layers per phase, chained and independent phases, 64 to 304 workgroups)."""
    rng = np.random.default_rng(4200 + seed)
    a = Arena()
    layers, prev_y, prev_n = [], None, 0
    for _ in range(int(rng.integers(3, 40))):
        K = int(rng.choice([32, 96, 1024, 2048, 2112, 3072, 4096, 8192, 14336]))
        chained = prev_y is not None and prev_n == K and rng.random() < 0.5
        x = prev_y if chained else a.take(K * 2)
        for _ in range(int(rng.integers(1, 4))):          # layers sharing the input: one phase
            N = int(rng.choice([1, 2, 7, 40, 96, 511, 1024, 2048, 3072, 4096, 4097, 40000]))
            y_bf16 = rng.random() < 0.4
            y = a.take(N * 4)
            layers.append(linear(a, N, K, x, y=y, prec=int(rng.integers(0, 2)), y_f32=not y_bf16))
            prev_y, prev_n = (y, N) if y_bf16 else (None, 0)   # only bf16 outputs can feed a layer
    nwg = int(rng.choice([64, 256, 304]))
    ordered = bool(rng.random() < 0.25)
    waves, phases = nvq.plan_describe(layers, 1, ordered=ordered, workgroups=nwg)
    assert waves == nwg * 12
    table = nvq.plan_describe_skips(layers, 1, ordered=ordered, workgroups=nwg)
    P = len(phases)
    skips, wg_passes = table[:waves], table[waves:]
    active = np.zeros((P, waves), bool)
    for p, ph in enumerate(phases):
        covered = np.zeros(ph["rows"], np.int32)
        # a barrier: the phase waits (through flags, or for mail) or publishes through flags
        barrier = ph["wait"] >= 0 or ph["publish"] == 1 or (ph["mail"] & 3) != 0
        waited_for = barrier or (ph["mail"] & 4) != 0      # ... or posts mail
        assert ph["spread"] == int(waited_for)
        if waited_for:
            assert ph["row_unit"] == max(ph["pair_stream"], 1)
        for j in range(waves):
            first, count = rows_of_wave(ph, j, waves)
            covered[first:first + count] += 1
            g = (j % nwg) * 12 + j // nwg if ph["spread"] else j
            active[p, g] = count > 0 or barrier
        assert covered.min() == 1 and covered.max() == 1
    for g in range(0, waves, 53):
        p, seen = 0, []
        while p < P:
            p += int(skips[g, p])
            if p < P:
                seen.append(p)
                p += 1
        # a visited phase is one the wave works in, or where a run of 255 passes ended
        assert set(p for p in range(P) if active[p, g]) <= set(seen)
        assert all(active[p, g] or skips[g, max(p - 255, 0)] == 255 for p in seen)
    assert np.array_equal(wg_passes[:, :P].T, ~active.reshape(P, nwg, 12).any(axis=2))


def test_image_regions_never_overwrite_an_image_that_may_still_be_read():
    layers = model_list("llama-8b", synth.make_precision_map(32, 16))
    _, phases = nvq.plan_describe(layers, 1)
    for p, ph in enumerate(phases):
        lo, hi = ph["img_lds"], ph["img_lds"] + ph["img_bytes"]
        assert 0 <= lo and hi <= AREA and ph["img_bytes"] % 1024 == 0 and ph["img_prepared"] == 1
        assert ph["img_need"] < p
        assert p == 0 or ph["img_need"] >= phases[p - 1]["img_need"]     # images load in order
        # the image may be loaded once every wave has finished phase img_need: the image of
        # every later phase (img_need < q < p) may still be read and must be disjoint from it
        for q in range(ph["img_need"] + 1, p):
            qlo, qhi = phases[q]["img_lds"], phases[q]["img_lds"] + phases[q]["img_bytes"]
            assert qhi <= lo or hi <= qlo, (p, q)
    # the area is really reused (the requirement is not vacuous) and the loader can run ahead
    assert max(ph["img_need"] for ph in phases) > 100
    assert all(p - ph["img_need"] >= 2 for p, ph in enumerate(phases) if ph["img_need"] >= 0)


def test_dependencies_follow_the_buffers():
    a = Arena()
    K = 2048
    x0, y0, y1 = a.take(K * 2), a.take(K * 2), a.take(K * 2)
    other, other2 = a.take(K * 2), a.take(K * 2)
    layers = [
        linear(a, K, K, x0, y0, y_f32=False),        # 0
        linear(a, K, K, y0, y1, y_f32=False),        # 1 reads what 0 wrote
        linear(a, K, K, other),                      # 2 independent
        linear(a, K, K, other2, y0, y_f32=False),    # 3 writes what 1 read and 0 wrote
        linear(a, K, K, x0, in_op=nvq.IN_RMSNORM, x2=y1, gamma=a.take(K * 2), eps=1e-5,
               h_out=a.take(K * 2)),                 # 4 reads y1 through its second operand
    ]
    waves, phases = nvq.plan_describe(layers, 1)
    # layer 1 reads what its predecessor writes and layer 2 conflicts with neither: 2 goes
    # first, so that the wait has passed when the waves get to 1
    assert [ph["first"] for ph in phases] == [0, 2, 1, 3, 4]
    # 1 and 4 take y0 / y1 by mail (exactly one earlier layer's bf16 output): no flags, and 1
    # never reads y0's memory, so 3 only has to wait for the phase that wrote it before
    assert waves and [ph["wait"] for ph in phases] == [-1, -1, -1, 0, -1]
    assert [ph["mail"] & 3 for ph in phases] == [0, 0, 1, 0, 2]
    assert [ph["mail"] >> 2 for ph in phases] == [1, 0, 1, 0, 0]      # who posts mail
    assert [ph["publish"] for ph in phases] == [1, 0, 0, 0, 0]
    # a phase whose input must be rebuilt after a wait has no prepared image
    assert [ph["img_prepared"] for ph in phases] == [1, 1, 0, 0, 0]
    # who waits or is waited for is dealt rows across the compute units
    assert [ph["spread"] for ph in phases] == [1, 0, 1, 1, 1]
    # forced ordering: everybody waits for the one before, through the flags
    _, ordered = nvq.plan_describe(layers, 1, ordered=True)
    assert [ph["first"] for ph in ordered] == [0, 1, 2, 3, 4]
    assert [ph["wait"] for ph in ordered] == [-1, 0, 1, 2, 3]
    assert [ph["mail"] for ph in ordered] == [0] * 5


def test_an_independent_phase_goes_before_the_phase_that_waits():
    """Where a phase reads what its predecessor writes and the phase after it conflicts with
    neither, the two change places (the results cannot differ: they do not touch each other's
    buffers); a forced order and batches above 1 keep the list's order."""
    a = Arena()
    K = 2048
    x0, xa, xb = a.take(K * 2), a.take(K * 2), a.take(K * 2)
    y = [a.take(K * 2) for _ in range(6)]
    layers = [
        linear(a, K, K, x0, y[0], y_f32=False),      # 0
        linear(a, K, K, y[0], y[1], y_f32=False),    # 1 waits for 0
        linear(a, K, K, xa, y[2], y_f32=False),      # 2 independent: before 1
        linear(a, K, K, y[1], y[3], y_f32=False),    # 3 waits for 1
        linear(a, K, K, xb, y[4], y_f32=False),      # 4 independent: before 3
        linear(a, K, K, y[3], y[5], y_f32=False),    # 5 waits for 3, nothing behind it
    ]
    _, phases = nvq.plan_describe(layers, 1)
    assert [ph["first"] for ph in phases] == [0, 2, 1, 4, 3, 5]
    assert [ph["mail"] & 3 for ph in phases] == [0, 0, 1, 0, 1, 1]
    _, ordered = nvq.plan_describe(layers, 1, ordered=True)
    assert [ph["first"] for ph in ordered] == [0, 1, 2, 3, 4, 5]
    # a phase that reads the waiting phase's output, or writes what it reads, stays behind it
    layers[2] = linear(a, 64, K, y[1], y[2], y_f32=False)
    _, phases = nvq.plan_describe(layers[:3], 1)
    assert [ph["first"] for ph in phases] == [0, 1, 2]
    layers[2] = linear(a, K, K, xa, y[0], y_f32=False)
    _, phases = nvq.plan_describe(layers[:3], 1)
    assert [ph["first"] for ph in phases] == [0, 1, 2]


def test_mail_needs_exactly_one_earlier_bf16_output():
    a = Arena()
    K = 2048

    def waits_and_mail(layers):
        _, phases = nvq.plan_describe(layers, 1)
        return [ph["wait"] for ph in phases], [ph["mail"] & 3 for ph in phases]

    x0 = a.take(K * 2)
    # an fp32 output read back as bf16 input: bytes overlap, no link
    yf = a.take(K * 4)
    assert waits_and_mail([linear(a, K, K, x0, yf), linear(a, 64, K, yf)]) == ([-1, 0], [0, 0])
    # two half-length outputs side by side make up the input: flags
    yh = a.take(K * 2)
    assert waits_and_mail([linear(a, K // 2, K, x0, yh, y_f32=False),
                           linear(a, K // 2, K, x0, yh + K, y_f32=False),
                           linear(a, 64, K, yh)]) == ([-1, 0], [0, 0])
    # the input is part of a longer output: flags
    yl = a.take(2 * K * 2)
    assert waits_and_mail([linear(a, 2 * K, K, x0, yl, y_f32=False),
                           linear(a, 64, K, yl + 64)]) == ([-1, 0], [0, 0])
    # written twice: the later writer is the one that sends the mail (and waits for the
    # earlier one, whose bytes it overwrites)
    y = a.take(K * 2)
    w, m = waits_and_mail([linear(a, K, K, x0, y, y_f32=False),
                           linear(a, K, K, a.take(K * 2), y, y_f32=False),
                           linear(a, 64, K, y)])
    assert (w, m) == ([-1, 0, -1], [0, 0, 1])
    # the latest writer only touched a part of it: flags for the reader
    w, m = waits_and_mail([linear(a, K, K, x0, y, y_f32=False),
                           linear(a, 8, K, a.take(K * 2), y + 32, y_f32=False),
                           linear(a, 64, K, y)])
    assert (w, m) == ([-1, 0, 1], [0, 0, 0])
    # both operands of a SiLU-multiply from the two layers of one phase, and the residual sum
    # of a norm phase into the next norm: the links of a decode block
    xg, xu, h0, h1, o, g = (a.take(K * 2) for _ in range(6))
    block = [linear(a, K, K, x0, o, y_f32=False),                                    # 0 "o"
             linear(a, K, K, h0, xg, y_f32=False, in_op=nvq.IN_RMSNORM, x2=o, gamma=g,
                    eps=1e-5, h_out=h1),                                             # 1 gate
             linear(a, K, K, h0, xu, y_f32=False, in_op=nvq.IN_RMSNORM, x2=o, gamma=g,
                    eps=1e-5, h_out=h1),                                             #   up
             linear(a, K, K, xg, a.take(K * 2), y_f32=False, in_op=nvq.IN_SILU_MUL, x2=xu),  # 2 down
             ]
    down = block[-1].y
    block.append(linear(a, 64, K, h1, in_op=nvq.IN_RMSNORM, x2=down, gamma=g, eps=1e-5,
                        h_out=a.take(K * 2)))                                        # 3 next q
    w, m = waits_and_mail(block)
    assert (w, m) == ([-1, -1, -1, -1], [0, 2, 3, 3])
    # at more than one token there is no persistent batch-1 kernel and no mail
    _, phases = nvq.plan_describe([linear(a, K, K, a.take(4 * K * 2), a.take(4 * K * 2), y_f32=False, M=4)], 4)
    assert phases[0]["mail"] == 0


def test_grouping_needs_the_same_input_precision_and_transform():
    a = Arena()
    K = 1024
    x, g = a.take(K * 2), a.take(K * 2)
    layers = [linear(a, 64, K, x), linear(a, 64, K, x), linear(a, 64, K, x, prec=1),
              linear(a, 64, K, x, prec=1, in_op=nvq.IN_RMSNORM, gamma=g, eps=1e-5),
              linear(a, 64, K, x, prec=1, in_op=nvq.IN_RMSNORM, gamma=g, eps=1e-5),
              linear(a, 64, K, x, prec=1, in_op=nvq.IN_RMSNORM, gamma=g, eps=1e-6)]
    _, phases = nvq.plan_describe(layers, 1)
    assert [(ph["first"], ph["count"]) for ph in phases] == [(0, 2), (2, 1), (3, 2), (5, 1)]
    # at most four matrices per phase
    many = [linear(a, 64, K, x) for _ in range(6)]
    _, phases = nvq.plan_describe(many, 1)
    assert [(ph["first"], ph["count"]) for ph in phases] == [(0, 4), (4, 2)]


def test_lists_the_persistent_kernel_does_not_take():
    a = Arena()
    big = [linear(a, 8, 16384, a.take(16384 * 2))]           # wider than an image holds
    waves, phases = nvq.plan_describe(big, 1)
    assert waves == 0 and len(phases) == 1 and phases[0]["wait"] == -1
    waves, _ = nvq.plan_describe(model_list_m("llama-1b", [0] * 16, 4), 4)   # batch 4: not batch 1
    assert waves == 0


# ---- grouped small-batch launches: batches and the parts of the persistent kernel ----
def model_list_m(model, bits, M):
    a = Arena()
    xs, out = {}, []
    for sp in synth.model_linears(model):
        if sp.phase not in xs:
            xs[sp.phase] = a.take(M * sp.K * 2)
        out.append(linear(a, sp.N, sp.K, xs[sp.phase], prec=1 if sp.block < 0 else bits[sp.block],
                          M=M))
    return out


@pytest.mark.parametrize("model,M", [("llama-1b", 4), ("llama-8b", 16)])
def test_parts_of_a_batch_cover_its_units_with_equal_weight(model, M):
    nb = synth.MODELS[model][0]
    layers = model_list_m(model, synth.make_precision_map(nb, nb // 2), M)
    _, phases = nvq.plan_describe(layers, M)
    ring, batches = nvq.plan_describe_batches(layers, M)
    assert ring and len(batches) == 1              # independent inputs: one batch of all phases
    b = batches[0]
    assert (b["first_phase"], b["last_phase"]) == (0, len(phases) - 1)
    assert b["jobs"] == len(phases)                # every phase gets an operand image
    # units: pairs of 16-row tiles, phase after phase; a unit of a phase weighs its K
    unit_phase, weight = [], []
    for p, ph in enumerate(phases):
        first = layers[ph["first"]]
        rows = sum(layers[ph["first"] + i].N for i in range(ph["count"]))
        unit_phase += [p] * ((rows + 31) // 32)
        weight += [first.K] * ((rows + 31) // 32)
    assert b["units"] == len(unit_phase)
    assert b["grid"] == 256 and b["parts"] == 8    # one workgroup per compute unit, 8 XCDs
    cuts = b["cuts"]
    assert cuts[0] == 0 and cuts[-1] == b["units"] and cuts == sorted(cuts)
    for c, p in zip(cuts[:-1], b["cut_phases"][:-1]):
        assert p == unit_phase[c]                  # where a team starts looking for its phase
    w = np.array(weight, dtype=np.int64)
    part_weight = [int(w[cuts[i]:cuts[i + 1]].sum()) for i in range(8)]
    assert max(part_weight) - min(part_weight) <= 2 * int(w.max())


def test_a_chain_makes_one_batch_per_phase_and_small_batches_few_workgroups():
    a = Arena()
    M = 6
    dims = [2048, 4096, 1024, 6144, 512]
    bufs = [a.take(M * d * 2) for d in dims]
    layers = [linear(a, dims[i + 1], dims[i], bufs[i], y=bufs[i + 1], prec=i % 2, y_f32=False, M=M)
              for i in range(4)]
    ring, batches = nvq.plan_describe_batches(layers, M)
    assert ring and len(batches) == 4
    for i, b in enumerate(batches):
        units = (dims[i + 1] + 31) // 32
        assert (b["first_phase"], b["last_phase"], b["units"], b["jobs"]) == (i, i, units, 1)
        assert b["grid"] == min(256, (units + 8) // 9)       # 3 teams x bundles of 3 units
        assert b["parts"] == min(8, b["grid"])
        assert b["cuts"][0] == 0 and b["cuts"][-1] == units
        assert all(p == i for p in b["cut_phases"])


def test_lists_the_persistent_small_batch_kernel_does_not_take():
    a = Arena()
    x = a.take(32 * 4096 * 2)
    ring, batches = nvq.plan_describe_batches([linear(a, 128, 4096, x, M=32)], 32)
    assert ring and batches[0]["grid"] == 2        # 4 units, two teams per workgroup beyond 16 tokens
    ring, batches = nvq.plan_describe_batches([linear(a, 128, 640, x, M=4)], 4)
    assert not ring and len(batches) == 1          # K is no multiple of 512
    ring, batches = nvq.plan_describe_batches([linear(a, 128, 4128, x, M=4)], 4)
    assert not ring and batches == []              # K % 128 != 0: launches per phase
