"""Benchmark of the encoding-decomposition QNN hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input resident in HBM:
    qnn_encode_pack (fp32 activations -> a_bits planes)
 -> qnn_binary_gemm (M x K xor+bitcount branches, recombination, fused per-channel scale;
                     writes the int32 accumulators and the fp32 scaled outputs)
on the 4096 x 4096 x 4096 workload with 2-bit weights and 2-bit activations (weights are packed
once, offline).  Prints ONE JSON line: effective binary TOPS (2 * rows * cols * n * w_bits *
a_bits operations per step / step time), the roofline of the dominant kernel (the binary GEMM,
bound by plain VALU xor + bitcount issue) and the CPU oracle timed on the host as a baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# VALU roofline of the xor + bitcount pair on MI355X, from the chip's unit counts and its 2.4 GHz clock (256 CUs x 4
# SIMDs).  The published 157.3 TFLOP/s fp32 vector figure is 32 lanes per SIMD and clock (one FMA = 2 flops); a
# wave64 v_xor_b32 issues at that rate (2 cycles) and v_bcnt_u32_b32 at half of it (16 lanes per clock, 4 cycles).
# One plane pair per 32 bit-pairs costs one of each and counts as 2 binary operations per bit-pair (xnor and
# count, the 2 * MAC convention):   peak = 1024 SIMDs x 2.4e9 / 6 cycles x 64 lanes x 32 bits x 2 = 1677.7 binary TOP/s.
# This ONE figure is the denominator of every "frac" this file prints.  What the chip shows on register-only loops
# is reported next to it (roofline.probe: the clock it holds under that load, read inside the kernel, and the cost
# of the two instructions in real cycles -- about 2.25 and 4.2 -- so a SIMD sustains about 6.4 .. 6.6 cycles per
# pair at 2.3 .. 2.4 GHz, 0.87 .. 0.91 of the figure above).
CLOCK_HZ = 2.4e9
SIMDS = 256 * 4
PEAK_BINARY_TOPS = SIMDS * CLOCK_HZ / 6.0 * 64 * 32 * 2 / 1e12
PEAK_NOTE = ("v_xor_b32 at 32 lanes/clk/SIMD (2 cycles per wave64) + v_bcnt_u32_b32 at 16 lanes/clk/SIMD (4 cycles), "
             "256 CUs x 4 SIMDs x 2.4 GHz")

# HBM bytes of one default-workload GEMM launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (profiles/bgemm_2x2_4096_hbm_counters.txt); only valid for size 4096, 2x2 bit
GEMM_2X2_4096_TRAFFIC_BYTES = 206.1e6

# HIP event pairs are put around every EVENT_EVERY-th GEMM launch of a timed region
EVENT_EVERY = 5


VALU_PROBE_MODES = ((0, "v_xor_b32"), (1, "v_bcnt_u32_b32"), (2, "xor_bcnt_pair"), (3, "pair_back_to_back"),
                    (4, "pair_two_deep"), (5, "pair_groups_of_4"), (6, "pair_two_deep_nop"))


def valu_probe(torch):
    """The register-only issue-rate loops: per mode the time per wave64 instruction and SIMD in ns, and the two
    in-kernel counters across the loop (s_memtime and the constant 100 MHz s_memrealtime).  Where s_memtime
    follows the shader clock, their ratio is the clock the chip held under that very load, and the time per
    instruction becomes real cycles; where it does not (ratio 1: both constant-rate), cycles are left out
    rather than derived from a nominal clock."""
    from paper_1905_13389_amd import probe
    wgs, iters = 512, 20000          # 2 waves per SIMD, 64 VALU instructions per iteration
    buf = torch.empty(wgs * 256, dtype=torch.int32, device="cuda")
    clocks = torch.zeros((wgs * 4, 2), dtype=torch.int64, device="cuda")
    res = {"unit": "ns per wave64 instruction per SIMD, 2 waves per SIMD"}
    for mode, name in VALU_PROBE_MODES:
        probe.qnn_probe_valu(mode, wgs, iters // 10, buf)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        probe.qnn_probe_valu(mode, wgs, iters, buf, clocks)
        e1.record()
        torch.cuda.synchronize()
        instr_per_simd = 64.0 * iters * (wgs / 256)
        ns = e0.elapsed_time(e1) * 1e6 / instr_per_simd
        c = clocks.double().mean(dim=0).tolist()
        ratio = c[0] / c[1] if c[1] > 0 else 0.0
        entry = {"ns": round(ns, 4), "memtime_over_realtime": round(ratio, 4)}
        if ratio > 1.5:   # s_memtime counts shader cycles: clock = ratio x 100 MHz
            entry["clock_ghz"] = round(ratio * 0.1, 4)
            entry["cycles"] = round(c[0] / (64.0 * iters * 2), 3)   # per instruction of the SIMD's 2 waves
        res[name] = entry
    best = min(res[n]["ns"] for _, n in VALU_PROBE_MODES[2:])
    res["best_pair_order"] = [n for _, n in VALU_PROBE_MODES[2:] if res[n]["ns"] == best][0]
    res["pair_binary_tops"] = round(SIMDS / (2 * best * 1e-9) * 64 * 64 / 1e12, 1)
    return res


def mfma_probe(torch):
    """Sustained rate of the register-only MFMA loops, in TOP/s (int8) and TFLOP/s (fp4)."""
    from paper_1905_13389_amd import probe
    wgs, iters = 512, 20000          # 2 waves per SIMD, 16 MFMAs per wave and iteration
    buf = torch.empty(wgs * 256, dtype=torch.int32, device="cuda")
    res = {}
    for mode, name, ops in ((0, "int8", 65536.0), (1, "fp4", 131072.0)):
        probe.qnn_probe_mfma(mode, wgs, iters // 10, buf)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        probe.qnn_probe_mfma(mode, wgs, iters, buf)
        e1.record()
        torch.cuda.synchronize()
        res[name] = round(ops * 16.0 * iters * wgs * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    # the same loops on operands from memory: what they hold sets the power drawn and with it the clock
    gen = torch.Generator().manual_seed(190513389)
    n = 256 * 8 * 16
    clocks = torch.zeros((wgs * 4, 2), dtype=torch.int64, device="cuda")
    by_data = {}
    for mode, name, ops in ((0, "int8", 65536.0), (1, "fp4", 131072.0)):
        lv = 2 * torch.randint(0, 4, (n,), generator=gen) - 3                       # levels of 2-bit codes
        if mode == 1:
            nib = torch.tensor([0xD, 0xA, 0x2, 0x5], dtype=torch.uint8)              # E2M1 codes of -3, -1, 1, 3
            pick = torch.randint(0, 4, (n, 2), generator=gen)
            levels = nib[pick[:, 0]] | (nib[pick[:, 1]] << 4)
        else:
            levels = lv.to(torch.int8).view(torch.uint8)
        kinds = (("zeros", torch.zeros(n, dtype=torch.uint8)), ("levels_of_2bit_codes", levels),
                 ("random_bytes", torch.randint(0, 256, (n,), generator=gen).to(torch.uint8)))
        row = {}
        for kind, host in kinds:
            operands = host.cuda()
            probe.qnn_probe_mfma_operands(mode, wgs, iters // 10, operands, buf)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            probe.qnn_probe_mfma_operands(mode, wgs, iters, operands, buf, clocks)
            e1.record()
            torch.cuda.synchronize()
            c = clocks.double().mean(dim=0).tolist()
            entry = {"tops": round(ops * 16.0 * iters * wgs * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)}
            if c[1] > 0 and c[0] / c[1] > 1.5:    # s_memtime counts shader cycles
                ghz = c[0] / c[1] * 0.1
                entry["clock_ghz"] = round(ghz, 3)
                # kernel time x clock / MFMAs per SIMD (a wave's own span is shorter: of the two waves of a SIMD the
                # older one is served first and ends early)
                entry["cycles_per_mfma_and_simd"] = round(e0.elapsed_time(e1) * 1e-3 * ghz * 1e9 / (16.0 * iters * wgs * 4 / SIMDS), 2)
            row[kind] = entry
        by_data[name] = row
    res["by_operand_data"] = by_data
    return res


SETTLE_MS = 300.0
SETTLE_MAX_MS = 1500.0


def settle(torch, fn):
    """Call fn untimed, back to back (the clock only rises under load without gaps), in batches of about 20 ms with a
    device synchronisation after each, until at least SETTLE_MS have passed and a batch is no longer more than 1 %
    faster per call than the one before it (at most SETTLE_MAX_MS)."""
    if SETTLE_MS <= 0:          # --no-settle: counter-collection runs, where every launch is serialised anyway
        return
    n, prev, spent = 4, None, 0.0
    while spent < SETTLE_MAX_MS:
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) * 1e3
        spent += dt
        per = max(dt / n, 1e-4)
        if spent >= SETTLE_MS and prev is not None and per > 0.99 * prev:
            break
        prev = per if dt >= 10.0 else None      # only batches long enough to show the pace are compared
        n = min(max(4, int(20.0 / per) + 1), 20000)


def timed_ms(torch, fn, steps, warmup):
    """`warmup` untimed calls, then exactly `steps` calls bracketed by device synchronisations: ms per call.
    The chip raises its shader clock to the sustained value only under tens of milliseconds of continuous load (read
    inside the kernels: an 80 us convolution runs at 2.05 GHz after 50 back-to-back launches and at 2.37 GHz after
    500, where it takes 70 us; a process that starts from an idle device needs longer), so after the `warmup` calls the
    workload is called untimed until its pace is steady (settle): the timed region then sees the clock a stream of such
    steps sees."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    settle(torch, fn)       # the warm-up calls' wall time may be one-time set-up, not load: it is not counted
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--size", type=int, default=4096, help="rows = cols = n of the square GEMM")
    ap.add_argument("--w-bits", type=int, default=2)
    ap.add_argument("--a-bits", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="default workload only: leave out the summaries of configurations 1, 3, 4, 5")
    ap.add_argument("--no-settle", action="store_true",
                    help="skip the untimed calls that bring the clock to its sustained value before each timed region "
                         "(for counter-collection runs under rocprofv3, which serialise the launches)")
    ap.add_argument("--repeats", type=int, default=5, help="default workload: repetitions of the K timed steps (the median is reported)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--sweep", action="store_true", help="also print GEMM-only times for all 1..4 x 1..4 bits")
    ap.add_argument("--workload", default="gemm", choices=["gemm", "fc1", "conv3", "stack4", "stack5", "ssd", "trunk", "pool", "grad", "deconv", "probe", "timeline"],
                    help="gemm (default, the headline 4096^3 GEMM) or one of the convolution workloads: conv3 = "
                         "ResNet-18-shaped 3x3 conv batch 64 (2x2 bit), stack4 = ResNet-18-shaped 16-conv stack "
                         "batch 256 (3x3 bit), stack5 = VGG16-style detection stack batch 32 at 300x300 (4x4 bit)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch of a convolution workload")
    return ap.parse_args()


def cpu_baseline(cfg, w_bits, a_bits, target_s):
    """The oracle as it stands, on a bounded row sample of the same GEMM."""
    import numpy as np
    import oracle
    size = cfg["a"].shape[1]
    cols = cfg["w"].shape[0]
    rows = 64
    t0 = time.perf_counter()
    oracle.gemm(cfg["a"][:rows], cfg["w"])
    probe = time.perf_counter() - t0
    rows = int(min(cfg["a"].shape[0], max(64, rows * target_s / max(probe, 1e-4))))
    # the whole workload is repeated when one pass is shorter than the target, so that the figure
    # rests on several seconds of CPU work
    reps = 1
    if rows == cfg["a"].shape[0]:
        reps = int(max(1, min(100, target_s / max(probe * rows / 64, 1e-4))))
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.gemm(cfg["a"][:rows], cfg["w"])
    dt = (time.perf_counter() - t0) / reps
    ops = 2.0 * rows * cols * size * w_bits * a_bits
    return {"value": ops / dt / 1e12, "unit": "effective binary TOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": "%d of %d rows x %d cols x n=%d, %d pass(es) of %.2f s, %.2f GMAC/s" %
            (rows, cfg["a"].shape[0], cols, size, reps, dt, rows * cols * size / dt / 1e9)}


def cpu_baseline_conv(groups, target_s):
    """The oracle's layer chain as it stands on the first images of every resolution group."""
    import oracle
    total_macs = 0.0
    per_image = []
    for g in groups:
        B, H, W, _ = g["x"].shape
        m = 0.0
        for L in g["layers"]:
            H, W = (H + 2 * L["pad"] - 3) // L["stride"] + 1, (W + 2 * L["pad"] - 3) // L["stride"] + 1
            m += H * W * L["cout"] * 9.0 * L["cin"]
        per_image.append(m)
    t0 = time.perf_counter()
    for g in groups:
        oracle.conv_stack(g["x"][:1], g["layers"])
    one = time.perf_counter() - t0
    batch = groups[0]["x"].shape[0]
    images = int(max(1, min(batch, target_s / max(one, 1e-4))))
    reps = int(max(1, min(50, target_s / max(one * images, 1e-4)))) if images == batch else 1
    t0 = time.perf_counter()
    for _ in range(reps):
        for g in groups:
            oracle.conv_stack(g["x"][:images], g["layers"])
    dt = (time.perf_counter() - t0) / reps
    macs = images * sum(per_image)
    bits = groups[0]["layers"][0]
    ops = 2.0 * macs * bits["w_bits"] * bits["a_bits"]
    return {"value": ops / dt / 1e12, "unit": "effective binary TOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d of %d images through every layer, %d pass(es) of %.2f s, %.2f GMAC/s" %
                      (images, batch, reps, dt, macs / dt / 1e9)}


def cpu_baseline_fc(c, target_s):
    """The oracle's GEMM on the whole small layer, repeated to fill the time budget."""
    import oracle
    t0 = time.perf_counter()
    oracle.gemm(c["a"], c["w"])
    one = time.perf_counter() - t0
    reps = int(max(1, min(20000, target_s / max(one, 1e-6))))
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.gemm(c["a"], c["w"])
    dt = (time.perf_counter() - t0) / reps
    rows, n = c["a"].shape
    cols = c["w"].shape[0]
    return {"value": 2.0 * rows * cols * n * 4 / dt / 1e12, "unit": "effective binary TOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": "the whole %dx%d -> %d layer, %d passes of %.1f us" % (rows, n, cols, reps, dt * 1e6)}


def conv_workload(args):
    """Convolution workloads: encode the fp32 input on device, then every conv with the fused
    scale -> quantize -> plane-split epilogue feeding the next one (the last writes fp32)."""
    import numpy as np
    import torch
    import qnn_workloads as wl
    from paper_1905_13389_amd import qnn

    if args.workload == "conv3":
        c = wl.resnet_conv_2x2(batch=args.batch or 64)
        L = {"w": c["w"], "scale": c["scale"], "clip": c["clip"], "a_bits": 2, "w_bits": 2, "stride": 1,
             "pad": 1, "cin": 64, "cout": 64}
        groups = [{"x": c["x"], "layers": [L]}]
        name = "ResNet-18-shaped 3x3 conv 64->64 @56x56, batch %d, 2x2 bit, int32 acc + fp32 scaled out" % c["x"].shape[0]
    elif args.workload == "stack4":
        c = wl.resnet18_stack(batch=args.batch or 256)
        groups = [c]
        name = "ResNet-18-shaped stack of 16 quantized 3x3 convs, batch %d, 3x3 bit" % c["x"].shape[0]
    else:
        groups = wl.vgg_ssd_stack(batch=args.batch or 32)
        name = "VGG16-style detection stack of 12 quantized 3x3 convs @300x300, batch %d, 4x4 bit" \
            % groups[0]["x"].shape[0]

    single = args.workload == "conv3"
    plans, macs, binops = [], 0, 0.0
    for g in groups:
        B, H, W, C = g["x"].shape
        d_x = torch.from_numpy(g["x"]).cuda()
        steps = []
        planes = torch.empty((g["layers"][0]["a_bits"], B * H * W, (C + 31) // 32), dtype=torch.int32, device="cuda")
        first = planes
        for li, L in enumerate(g["layers"]):
            wp = qnn.qnn_encode_pack(torch.from_numpy(L["w"]).cuda(), 1.0, L["w_bits"]).view(
                L["w_bits"], L["cout"], 3, 3, -1)
            ho = (H + 2 * L["pad"] - 3) // L["stride"] + 1
            wo = (W + 2 * L["pad"] - 3) // L["stride"] + 1
            last = li + 1 == len(g["layers"])
            nxt = None if last else torch.empty((g["layers"][li + 1]["a_bits"], B * ho * wo, (L["cout"] + 31) // 32),
                                                dtype=torch.int32, device="cuda")
            out = torch.empty((B, ho, wo, L["cout"]), dtype=torch.float32, device="cuda") if last else None
            # the single-layer configuration hands out both results, int32 accumulators and fp32 scaled values
            acc = torch.empty((B, ho, wo, L["cout"]), dtype=torch.int32, device="cuda") if single else None
            steps.append((planes, wp, (B, H, W), L, torch.from_numpy(L["scale"]).cuda(), out, nxt,
                          None if last else g["layers"][li + 1], acc))
            m = B * ho * wo * L["cout"] * 9 * L["cin"]
            macs += m
            binops += 2.0 * m * L["w_bits"] * L["a_bits"]
            planes, H, W = nxt, ho, wo
        plans.append((d_x, g["layers"][0], first, steps))

    # one step as a flat list of launches: (label, binary operations, launch)
    calls = []
    for d_x, L0, first, steps in plans:
        calls.append(("encode", 0.0, lambda d_x=d_x, L0=L0, first=first: qnn.qnn_encode_pack(d_x, L0["clip"], L0["a_bits"], planes=first)))
        for planes, wp, shape, L, sc, out, nxt, Ln, acc in steps:
            label = "%d->%d@%dx%d%s" % (L["cin"], L["cout"], shape[1], shape[2], " s2" if L["stride"] == 2 else "")
            ho = (shape[1] + 2 * L["pad"] - 3) // L["stride"] + 1
            ops = 2.0 * shape[0] * ho * ho * L["cout"] * 9 * L["cin"] * L["w_bits"] * L["a_bits"]
            calls.append((label, ops, lambda planes=planes, wp=wp, shape=shape, L=L, sc=sc, out=out, nxt=nxt, Ln=Ln, acc=acc:
                          qnn.qnn_conv2d(planes, wp, shape, L["cin"], L["stride"], L["pad"], scale=sc, want_acc=False, acc=acc,
                                         want_out=out is not None, out=out, next_clip=None if Ln is None else Ln["clip"],
                                         next_bits=0 if Ln is None else Ln["a_bits"], next_planes=nxt)))

    def step():
        for _, _, launch in calls:
            launch()

    ms = timed_ms(torch, step, args.steps, args.warmup)
    tops = binops / (ms * 1e-3) / 1e12
    # The dominant kernel's own time: every convolution launch of a step between its own pair of HIP events on
    # torch's current stream (the stream the launches go to), over a few instrumented steps outside the timed region.
    # Each launch is issued `back_to_back` times between its events (the launches of a step are idempotent): a
    # single short kernel between two events also shows the device's latency from one dependent kernel to the
    # next (about 10 us here), which is not the kernel's own time.
    reps, back_to_back = 3, 4
    samples = [[] for _ in calls]
    for _ in range(reps):
        evs = []
        for _, _, launch in calls:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(back_to_back):
                launch()
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        for i, (e0, e1) in enumerate(evs):
            samples[i].append(e0.elapsed_time(e1) / back_to_back)
    per_launch = [sorted(v)[reps // 2] for v in samples]      # the median: one disturbed pass does not count
    conv_ms = sum(t for (label, ops, _), t in zip(calls, per_launch) if ops > 0)
    conv_tops = binops / (conv_ms * 1e-3) / 1e12
    layer_fracs = [(label, ops / (t * 1e-3) / 1e12 / PEAK_BINARY_TOPS, t) for (label, ops, _), t in zip(calls, per_launch) if ops > 0]
    worst = min(layer_fracs, key=lambda e: e[1])
    best = max(layer_fracs, key=lambda e: e[1])

    # the same chain on the matrix cores (comparison only): levels stay decoded as int8 from layer to
    # layer, qnn_encode_levels_i8 + qnn_level_conv2d_i8 with the fused scale -> quantize -> level epilogue
    mplans = []
    for g in groups:
        B, H, W, C = g["x"].shape
        d_x = torch.from_numpy(g["x"]).cuda()
        lv = torch.empty((B, H, W, C), dtype=torch.int8, device="cuda")
        first, msteps = lv, []
        for li, L in enumerate(g["layers"]):
            ho = (H + 2 * L["pad"] - 3) // L["stride"] + 1
            wo = (W + 2 * L["pad"] - 3) // L["stride"] + 1
            last = li + 1 == len(g["layers"])
            nxt = None if last else torch.empty((B, ho, wo, L["cout"]), dtype=torch.int8, device="cuda")
            out = torch.empty((B, ho, wo, L["cout"]), dtype=torch.float32, device="cuda") if last else None
            acc = torch.empty((B, ho, wo, L["cout"]), dtype=torch.int32, device="cuda") if single else None
            msteps.append((lv, torch.from_numpy(L["w"]).cuda(), L, torch.from_numpy(L["scale"]).cuda(), out, nxt,
                           None if last else g["layers"][li + 1], acc))
            lv, H, W = nxt, ho, wo
        mplans.append((d_x, g["layers"][0], first, msteps))

    def mfma_step():
        for d_x, L0, first, msteps in mplans:
            qnn.qnn_encode_levels_i8(d_x, L0["clip"], L0["a_bits"], levels=first)
            for lv, w, L, sc, out, nxt, Ln, acc in msteps:
                qnn.qnn_level_conv2d_i8(lv, w, L["stride"], L["pad"], L["a_bits"], L["w_bits"], scale=sc,
                                        want_acc=False, acc=acc, want_out=out is not None, out=out,
                                        next_clip=None if Ln is None else Ln["clip"],
                                        next_bits=0 if Ln is None else Ln["a_bits"], next_levels=nxt)

    m_ms = timed_ms(torch, mfma_step, args.steps, args.warmup)
    int8_tops = 2.0 * macs / (m_ms * 1e-3) / 1e12

    # 1- and 2-bit chains also run on the fp4 matrix-core path: two levels per byte, twice the products per clock
    fp4 = None
    if all(L["a_bits"] <= 2 and L["w_bits"] <= 2 for g in groups for L in g["layers"]):
        fplans = []
        for g in groups:
            B, H, W, C = g["x"].shape
            d_x = torch.from_numpy(g["x"]).cuda()
            lv = torch.empty((B, H, W, C // 2), dtype=torch.uint8, device="cuda")
            first, fsteps = lv, []
            for li, L in enumerate(g["layers"]):
                ho = (H + 2 * L["pad"] - 3) // L["stride"] + 1
                wo = (W + 2 * L["pad"] - 3) // L["stride"] + 1
                last = li + 1 == len(g["layers"])
                nxt = None if last else torch.empty((B, ho, wo, L["cout"] // 2), dtype=torch.uint8, device="cuda")
                out = torch.empty((B, ho, wo, L["cout"]), dtype=torch.float32, device="cuda") if last else None
                acc = torch.empty((B, ho, wo, L["cout"]), dtype=torch.int32, device="cuda") if single else None
                fsteps.append((lv, qnn.qnn_levels_to_fp4(torch.from_numpy(L["w"]).cuda()), L,
                               torch.from_numpy(L["scale"]).cuda(), out, nxt, None if last else g["layers"][li + 1], acc))
                lv, H, W = nxt, ho, wo
            fplans.append((d_x, g["layers"][0], first, fsteps))

        def fp4_step():
            for d_x, L0, first, fsteps in fplans:
                qnn.qnn_encode_levels_fp4(d_x, L0["clip"], L0["a_bits"], levels=first)
                for lv, w, L, sc, out, nxt, Ln, acc in fsteps:
                    qnn.qnn_level_conv2d_fp4(lv, w, L["stride"], L["pad"], L["a_bits"], L["w_bits"], scale=sc,
                                             want_acc=False, acc=acc, want_out=out is not None, out=out,
                                             next_clip=None if Ln is None else Ln["clip"],
                                             next_bits=0 if Ln is None else Ln["a_bits"], next_levels=nxt)

        f_ms = timed_ms(torch, fp4_step, args.steps, args.warmup)
        fp4_tops = 2.0 * macs / (f_ms * 1e-3) / 1e12
        fp4 = {"step": "qnn_encode_levels_fp4 + qnn_level_conv2d_fp4 per layer (fused scale/quantize epilogue)",
               "ms_per_step": round(f_ms, 4), "effective_binary_tops": round(binops / (f_ms * 1e-3) / 1e12, 1),
               "speedup_vs_xor_bitcount_step": round(ms / f_ms, 2),
               "roofline": {"bound": "mfma", "achieved": round(fp4_tops, 1), "peak": 10100.0, "unit": "fp4 TFLOP/s",
                            "frac": round(fp4_tops / 10100.0, 4), "note": "whole step, not a single kernel"}}

    result = {
        "metric": "effective binary TOPS (xnor+popcount) and % of VALU/HBM roofline, 1 MI355X", "value": round(tops, 2),
        "unit": "binary TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 bit-planes, int32 accumulate", "data": "synthetic",
        "fp4_variant": fp4,
        "config": {"workload": name, "macs": macs,
                   "step": "qnn_encode_pack + qnn_conv2d per layer (fused scale/quantize/pack epilogue)"},
        "roofline": {"bound": "alu", "kernel": "bconv_tile_kernel (%d launches per step)" % sum(1 for c in calls if c[1] > 0),
                     "achieved": round(conv_tops, 2), "peak": round(PEAK_BINARY_TOPS, 1),
                     "unit": "binary TOP/s", "frac": round(conv_tops / PEAK_BINARY_TOPS, 4), "traffic": None,
                     "kernel_ms": round(conv_ms, 4),
                     "kernel_ms_note": "sum over the step's convolution launches, each timed between its own HIP events as the average of 4 back-to-back launches (median of 3 passes)",
                     "step_frac": round(tops / PEAK_BINARY_TOPS, 4),
                     "slowest_layer": {"layer": worst[0], "frac": round(worst[1], 4), "ms": round(worst[2], 4)},
                     "fastest_layer": {"layer": best[0], "frac": round(best[1], 4), "ms": round(best[2], 4)},
                     "peak_note": PEAK_NOTE},
        "mfma_variant": {"step": "qnn_encode_levels_i8 + qnn_level_conv2d_i8 per layer (fused scale/quantize epilogue)",
                         "ms_per_step": round(m_ms, 4), "effective_binary_tops": round(binops / (m_ms * 1e-3) / 1e12, 1),
                         "speedup_vs_xor_bitcount_step": round(ms / m_ms, 2),
                         "roofline": {"bound": "mfma", "achieved": round(int8_tops, 1), "peak": 5000.0,
                                      "unit": "int8 TOP/s", "frac": round(int8_tops / 5000.0, 4),
                                      "note": "whole step, not a single kernel"}}}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline_conv(groups, args.cpu_seconds)
    return result


def trunk_workload(args):
    """The residual trunk of ResNet-18 (8 blocks: 16 3x3 convolutions, 3 1x1 shortcut convolutions, bias
    and shortcut terms fused into the epilogues), 3x3 bit, on both machine routes.  Between layers only
    planes (or int8 levels) exist; the three 1x1 shortcuts are handed over in fp32."""
    import torch
    import qnn_workloads as wl
    from paper_1905_13389_amd import qnn

    bits = 3
    net = wl.resnet18_trunk(batch=args.batch or 256, bits=bits)
    x, blocks = net["x"], net["blocks"]
    B, H0, W0, C0 = x.shape
    d_x = torch.from_numpy(x).cuda()
    up = lambda a: torch.from_numpy(a).cuda()
    macs = 0

    def build(route):
        nonlocal macs
        macs = 0
        H, W, C = H0, W0, C0
        if route == "planes":
            new = lambda h, w, c: torch.empty((bits, B * h * w, (c + 31) // 32), dtype=torch.int32, device="cuda")
            wt = lambda L, k: qnn.qnn_encode_pack(up(L["w"]), 1.0, bits).view(bits, L["cout"], k, k, -1)
        else:
            new = lambda h, w, c: torch.empty((B, h, w, c), dtype=torch.int8, device="cuda")
            wt = lambda L, k: up(L["w"])
        first = a = new(H, W, C)
        calls = []
        for bi, blk in enumerate(blocks):
            c1, c2, dn = blk["conv1"], blk["conv2"], blk["down"]
            st, cout = c1["stride"], c1["cout"]
            Ho, Wo = (H + 2 - 3) // st + 1, (W + 2 - 3) // st + 1
            last = bi + 1 == len(blocks)
            hq = new(Ho, Wo, cout)
            nxt = None if last else new(Ho, Wo, cout)
            y = torch.empty((B, Ho, Wo, cout), dtype=torch.float32, device="cuda") if last else None
            short = torch.empty((B, Ho, Wo, cout), dtype=torch.float32, device="cuda") if dn is not None else None
            nclip = None if last else blocks[bi + 1]["conv1"]["clip"]
            common = {"want_acc": False}
            calls.append((a, wt(c1, 3), (B, H, W), C, st, 1, up(c1["scale"]),
                          dict(common, bias=up(c1["bias"]), next_clip=c2["clip"], next_bits=bits), hq, None))
            macs += B * Ho * Wo * cout * 9 * C
            if dn is not None:
                calls.append((a, wt(dn, 1), (B, H, W), C, st, 0, up(dn["scale"]),
                              dict(common, bias=up(dn["bias"]), want_out=True), None, short))
                macs += B * Ho * Wo * cout * C
                res = {"res_f32": short}
            elif route == "planes":
                res = {"res_planes": a, "res_scale": blk["res_scale"]}
            else:
                res = {"res_levels": a, "res_bits": bits, "res_scale": blk["res_scale"]}
            calls.append((hq, wt(c2, 3), (B, Ho, Wo), cout, 1, 1, up(c2["scale"]),
                          dict(common, bias=up(c2["bias"]), want_out=last, next_clip=nclip,
                               next_bits=0 if last else bits, **res), nxt, y))
            macs += B * Ho * Wo * cout * 9 * cout
            a, H, W, C = nxt, Ho, Wo, cout
        return first, calls

    p_first, p_calls = build("planes")
    l_first, l_calls = build("levels")
    clip0 = blocks[0]["conv1"]["clip"]

    def step():
        qnn.qnn_encode_pack(d_x, clip0, bits, planes=p_first)
        for a, w, shape, cin, st, pad, sc, kw, nxt, out in p_calls:
            qnn.qnn_conv2d_block(a, w, shape, cin, st, pad, sc, next_planes=nxt, out=out, **kw)

    def mfma_step():
        qnn.qnn_encode_levels_i8(d_x, clip0, bits, levels=l_first)
        for a, w, shape, cin, st, pad, sc, kw, nxt, out in l_calls:
            qnn.qnn_level_conv2d_block_i8(a, w, st, pad, bits, bits, sc, next_levels=nxt, out=out, **kw)

    ms, m_ms = (timed_ms(torch, f, args.steps, args.warmup) for f in (step, mfma_step))

    # the unquantized ends around the trunk: image -> first convolution (fp32, planes out) -> 3x3 stride-2
    # pooling of the planes -> trunk -> global average pooling -> classifier
    ends = wl.resnet18_ends(batch=B)
    img, w0, s0, b0 = (up(ends[k]) for k in ("image", "stem_w", "stem_scale", "stem_shift"))
    fc_w, fc_b = up(ends["fc_w"]), up(ends["fc_b"])
    side = (img.shape[1] + 2 * 3 - 7) // 2 + 1
    stem_planes = torch.empty((bits, B * side * side, 2), dtype=torch.int32, device="cuda")
    y_last = p_calls[-1][-1]
    feat = torch.empty((B, y_last.shape[-1]), dtype=torch.float32, device="cuda")
    logits = torch.empty((B, fc_w.shape[0]), dtype=torch.float32, device="cuda")

    def stem():
        qnn.qnn_dense_conv2d_f32(img, w0, 2, 3, scale=s0, shift=b0, relu=True, want_out=False, next_clip=clip0,
                                 next_bits=bits, next_planes=stem_planes)
        qnn.qnn_maxpool_planes(stem_planes, (B, side, side), 64, 3, 2, 1, out=p_first)

    def head():
        qnn.qnn_global_avgpool_f32(y_last, out=feat)
        qnn.qnn_dense_fc_f32(feat, fc_w, fc_b, out=logits)

    def network():
        stem()
        for a, w, shape, cin, st, pad, sc, kw, nxt, out in p_calls:
            qnn.qnn_conv2d_block(a, w, shape, cin, st, pad, sc, next_planes=nxt, out=out, **kw)
        head()

    # the same graph on the matrix-core route: int8 levels from the first convolution on
    stem_levels = torch.empty((B, side, side, 64), dtype=torch.int8, device="cuda")
    ym_last = l_calls[-1][-1]

    def mfma_network():
        qnn.qnn_dense_conv2d_f32_levels(img, w0, 2, 3, clip0, bits, scale=s0, shift=b0, relu=True, next_levels=stem_levels)
        qnn.qnn_maxpool_levels_i8(stem_levels, 3, 2, 1, out=l_first)
        for a, w, shape, cin, st, pad, sc, kw, nxt, out in l_calls:
            qnn.qnn_level_conv2d_block_i8(a, w, st, pad, bits, bits, sc, next_levels=nxt, out=out, **kw)
        qnn.qnn_global_avgpool_f32(ym_last, out=feat)
        qnn.qnn_dense_fc_f32(feat, fc_w, fc_b, out=logits)

    assert side // 2 == H0, "the pooled stem output is the trunk's input"
    conv_only = lambda: qnn.qnn_dense_conv2d_f32(img, w0, 2, 3, scale=s0, shift=b0, relu=True, want_out=False,
                                                 next_clip=clip0, next_bits=bits, next_planes=stem_planes)
    stem_ms, conv_ms, head_ms, net_ms, mnet_ms = (timed_ms(torch, f, args.steps, args.warmup)
                                                  for f in (stem, conv_only, head, network, mfma_network))
    stem_tflops = 2.0 * B * side * side * 64 * 147 / (conv_ms * 1e-3) / 1e12
    binops = 2.0 * macs * bits * bits
    tops = binops / (ms * 1e-3) / 1e12
    int8_tops = 2.0 * macs / (m_ms * 1e-3) / 1e12
    return {
        "metric": "effective binary TOPS (xnor+popcount) and % of VALU/HBM roofline, 1 MI355X", "value": round(tops, 2),
        "unit": "binary TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 bit-planes, int32 accumulate", "data": "synthetic",
        "config": {"workload": "residual trunk of ResNet-18 (16 3x3 + 3 1x1 convolutions, shortcuts and folded "
                               "batch-norm shifts in the epilogues), batch %d, 3x3 bit" % B, "macs": macs,
                   "step": "qnn_encode_pack + qnn_conv2d_block per convolution"},
        "roofline": {"bound": "alu", "achieved": round(tops, 2), "peak": round(PEAK_BINARY_TOPS, 1),
                     "unit": "binary TOP/s", "frac": round(tops / PEAK_BINARY_TOPS, 4), "traffic": None,
                     "note": "whole step (encode + all conv launches), not a single kernel"},
        "network": {"step": "qnn_dense_conv2d_f32 (image -> planes) + qnn_maxpool_planes + trunk + "
                            "qnn_global_avgpool_f32 + qnn_dense_fc_f32: %dx%d images to %d logits" % (img.shape[1], img.shape[2], fc_w.shape[0]),
                    "ms_per_step": round(net_ms, 4), "images_per_s": round(B / (net_ms * 1e-3), 1),
                    "stem_ms": round(stem_ms, 4), "head_ms": round(head_ms, 4),
                    "matrix_core_route": {"step": "qnn_dense_conv2d_f32_levels + qnn_maxpool_levels_i8 + trunk on "
                                                  "qnn_level_conv2d_block_i8 + the same head",
                                          "ms_per_step": round(mnet_ms, 4), "images_per_s": round(B / (mnet_ms * 1e-3), 1)},
                    "stem_roofline": {"bound": "mfma", "kernel": "dense_conv_kernel", "achieved": round(stem_tflops, 1),
                                      "peak": 157.3, "unit": "fp32 TFLOP/s", "frac": round(stem_tflops / 157.3, 4),
                                      "kernel_ms": round(conv_ms, 4)}},
        "mfma_variant": {"step": "qnn_encode_levels_i8 + qnn_level_conv2d_block_i8 per convolution",
                         "ms_per_step": round(m_ms, 4), "effective_binary_tops": round(binops / (m_ms * 1e-3) / 1e12, 1),
                         "speedup_vs_xor_bitcount_step": round(ms / m_ms, 2),
                         "roofline": {"bound": "mfma", "achieved": round(int8_tops, 1), "peak": 5000.0,
                                      "unit": "int8 TOP/s", "frac": round(int8_tops / 5000.0, 4),
                                      "note": "whole step, not a single kernel"}}}


def graph_workload(args):
    """The detection network of configuration 5 as ONE chain on one input (wl.vgg_ssd_chained): the backbone's twelve
    convolutions joined by max-pooling of the planes, the SSD-style extra layers down to 1x1 and the heads on the
    six maps, 4x4 bit, on both machine routes.  Between layers only planes (or int8 levels) exist; the heads write
    fp32 scores."""
    import torch
    import qnn_workloads as wl
    from paper_1905_13389_amd import qnn

    B = args.batch or 32
    net = wl.vgg_ssd_chained(batch=B, bits=4)
    bits, nodes = net["bits"], net["nodes"]
    up = lambda a: torch.from_numpy(a).cuda()
    d_x = up(net["x"])
    _, H0, W0, C0 = net["x"].shape

    def build(route):
        planes = route == "planes"
        new = (lambda h, c: torch.empty((bits, B * h * h, (c + 31) // 32), dtype=torch.int32, device="cuda")) if planes \
            else (lambda h, c: torch.empty((B, h, h, c), dtype=torch.int8, device="cuda"))
        first = new(H0, C0)
        val = {"input": (first, H0, C0)}
        calls, macs = [], 0
        for nd in nodes:
            src, H, C = val[nd["src"]]
            if nd["kind"] == "pool":
                ho = qnn.qnn_pool_out_size(H, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"])
                dst = new(ho, C)
                if planes:
                    fn = lambda src=src, H=H, C=C, nd=nd, dst=dst: qnn.qnn_maxpool_planes(
                        src, (B, H, H), C, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"], out=dst)
                else:
                    fn = lambda src=src, nd=nd, dst=dst: qnn.qnn_maxpool_levels_i8(
                        src, nd["k"], nd["stride"], nd["pad"], nd["ceil_mode"], out=dst)
                calls.append((nd["name"], 0.0, fn))
                val[nd["name"]] = (dst, ho, C)
                continue
            k, head, dil = nd["k"], nd["head"], nd.get("dilation", 1)
            ho = (H + 2 * nd["pad"] - dil * (k - 1) - 1) // nd["stride"] + 1
            sc = up(nd["scale"])
            dst = None if head else new(ho, nd["cout"])
            out = torch.empty((B, ho, ho, nd["cout"]), dtype=torch.float32, device="cuda") if head else None
            m = B * ho * ho * nd["cout"] * k * k * nd["cin"]
            macs += m
            if planes:
                wp = qnn.qnn_encode_pack(up(nd["w"]), 1.0, bits).view(bits, nd["cout"], k, k, -1)
                fn = lambda src=src, wp=wp, H=H, C=C, nd=nd, sc=sc, dst=dst, out=out, head=head, dil=dil: qnn.qnn_conv2d_dilated(
                    src, wp, (B, H, H), C, nd["stride"], nd["pad"], dil, scale=sc, want_acc=False, want_out=head, out=out,
                    next_clip=None if head else nd["clip"], next_bits=0 if head else bits, next_planes=dst)
            else:
                wl_ = up(nd["w"])
                fn = lambda src=src, wl_=wl_, nd=nd, sc=sc, dst=dst, out=out, head=head, dil=dil: qnn.qnn_level_conv2d_dilated_i8(
                    src, wl_, nd["stride"], nd["pad"], dil, bits, bits, scale=sc, want_acc=False, want_out=head, out=out,
                    next_clip=None if head else nd["clip"], next_bits=0 if head else bits, next_levels=dst)
            calls.append(("%s %d->%d@%d k%d%s" % (nd["name"], nd["cin"], nd["cout"], H, k, " s2" if nd["stride"] == 2 else ""),
                          2.0 * m * bits * bits, fn))
            val[nd["name"]] = (dst, ho, nd["cout"])
        return first, calls, macs

    p_first, p_calls, macs = build("planes")
    l_first, l_calls, _ = build("levels")
    binops = 2.0 * macs * bits * bits

    def step():
        qnn.qnn_encode_pack(d_x, net["clip0"], bits, planes=p_first)
        for _, _, fn in p_calls:
            fn()

    def mfma_step():
        qnn.qnn_encode_levels_i8(d_x, net["clip0"], bits, levels=l_first)
        for _, _, fn in l_calls:
            fn()

    ms, m_ms = (timed_ms(torch, f, args.steps, args.warmup) for f in (step, mfma_step))
    tops = binops / (ms * 1e-3) / 1e12
    # every launch of the planes route between its own events, 4 back-to-back launches each (see conv_workload)
    evs = []
    for _ in range(2):                      # the first pass settles the clocks, the second is read
        evs = []
        for label, ops, fn in p_calls:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(4):
                fn()
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
    per = [(label, ops, e0.elapsed_time(e1) / 4) for (label, ops, _), (e0, e1) in zip(p_calls, evs)]
    conv_ms = sum(t for _, ops, t in per if ops > 0)
    pool_ms = sum(t for _, ops, t in per if ops == 0)
    conv_tops = binops / (conv_ms * 1e-3) / 1e12
    fr = [(label, ops / (t * 1e-3) / 1e12 / PEAK_BINARY_TOPS, t) for label, ops, t in per if ops > 0]
    worst = min((e for e in fr if e[2] > 0.01 * conv_ms), key=lambda e: e[1])   # among layers that matter
    int8_tops = 2.0 * macs / (m_ms * 1e-3) / 1e12
    return {
        "metric": "effective binary TOPS (xnor+popcount) and % of VALU/HBM roofline, 1 MI355X", "value": round(tops, 2),
        "unit": "binary TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32 bit-planes, int32 accumulate",
        "data": "synthetic",
        "config": {"workload": "VGG16 + SSD-style detection network as one chain: 12 backbone convolutions joined by max-pooling, "
                               "10 extra convolutions down to 1x1 (one with its taps 6 pixels apart), 12 head convolutions on six maps; batch %d, 300x300, 4x4 bit" % B,
                   "macs": macs, "images_per_s": round(B / (ms * 1e-3), 1),
                   "step": "qnn_encode_pack + qnn_conv2d_dilated (dilation 1 = qnn_conv2d; fused scale/quantize/pack epilogue) / qnn_maxpool_planes per node"},
        "roofline": {"bound": "alu", "kernel": "bconv_tile_kernel (%d launches per step)" % sum(1 for e in per if e[1] > 0),
                     "achieved": round(conv_tops, 2), "peak": round(PEAK_BINARY_TOPS, 1), "unit": "binary TOP/s",
                     "frac": round(conv_tops / PEAK_BINARY_TOPS, 4), "traffic": None, "kernel_ms": round(conv_ms, 4),
                     "pooling_ms": round(pool_ms, 4), "step_frac": round(tops / PEAK_BINARY_TOPS, 4),
                     "slowest_layer_above_1pct_of_time": {"layer": worst[0], "frac": round(worst[1], 4), "ms": round(worst[2], 4)},
                     "peak_note": PEAK_NOTE},
        "mfma_variant": {"step": "qnn_encode_levels_i8 + qnn_level_conv2d_dilated_i8 / qnn_maxpool_levels_i8 per node",
                         "ms_per_step": round(m_ms, 4), "images_per_s": round(B / (m_ms * 1e-3), 1),
                         "speedup_vs_xor_bitcount_step": round(ms / m_ms, 2),
                         "roofline": {"bound": "mfma", "achieved": round(int8_tops, 1), "peak": 5000.0, "unit": "int8 TOP/s",
                                      "frac": round(int8_tops / 5000.0, 4), "note": "whole step, not a single kernel"}}}


def probe_workload(args):
    """The register-only issue-rate loops of libqnn_probe over 1, 2, 3, 4 and 8 waves per SIMD: per order the cost of a
    wave64 instruction in real cycles (kernel time x the clock read inside the kernel / instructions per SIMD) and what
    a single wave sees (cycles between its own instructions).  The evidence behind the VALU roofline's notes."""
    import torch
    from paper_1905_13389_amd import probe
    names = {0: "v_xor_b32", 1: "v_bcnt_u32_b32", 2: "pair, s_nop after each", 3: "pair back to back", 4: "two deep, rotating temporaries",
             5: "4 xors then 4 counts", 6: "two deep + s_nop", 7: "count + s_nop", 8: "2 xors + s_nop", 9: "xor xor count count s_nop",
             10: "two pairs + s_nop", 11: "xor s_nop count", 12: "count xor s_nop"}
    iters = 10000
    table = {}
    for wps in (1, 2, 3, 4, 8):
        wgs = 256 * wps
        buf = torch.empty(wgs * 256, dtype=torch.int32, device="cuda")
        clk = torch.zeros((wgs * 4, 2), dtype=torch.int64, device="cuda")
        row = {}
        for mode, label in names.items():
            probe.qnn_probe_valu(mode, wgs, iters // 10, buf)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            probe.qnn_probe_valu(mode, wgs, iters, buf, clk)
            e1.record()
            torch.cuda.synchronize()
            c = clk.double()
            ghz = (c[:, 0].sum() / c[:, 1].sum()).item() * 0.1
            own = c[:, 0] / (64.0 * iters)
            row[label] = {"cycles_per_instruction_per_simd": round(e0.elapsed_time(e1) * 1e-3 * ghz * 1e9 / (64.0 * iters * wps), 3),
                          "clock_ghz": round(ghz, 3), "kernel_ms": round(e0.elapsed_time(e1), 3),
                          "wave_cycles_between_own_instructions": {"min": round(own.min().item(), 2), "mean": round(own.mean().item(), 2),
                                                                   "max": round(own.max().item(), 2)}}
        table["%d waves per SIMD" % wps] = row
    best = min(v["pair, s_nop after each"]["cycles_per_instruction_per_simd"] for v in table.values())
    return {"metric": "VALU issue cost of the binary dot product's instructions", "value": round(2 * best, 3),
            "unit": "cycles per xor + count pair per SIMD (best occupancy)", "n_gpus": 1, "steps": 1, "warmup": 1,
            "ms_per_step": None, "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
            "config": {"workload": "register-only loops of 64 VALU instructions x %d iterations per wave, 256 CUs" % iters},
            "probe_matrix": table, "mfma_probe": mfma_probe(torch)}


def timeline_workload(args):
    """Wave timestamps of the convolution kernel (libqnn_timeline.so: the same kernels compiled with s_memrealtime reads
    at wave start, after the prologue and at wave end), with and without the balance between the two workgroups of a CU:
    when the workgroups dispatched first / second end, how far the waves' ends are spread, the launch's span."""
    import torch
    from paper_1905_13389_amd import probe, qnn

    cases = [("config 3: 64->64 @56x56, batch 64, 2x2 bit, acc + out", 64, 56, 64, 64, 2, "acc+out"),
             ("64->64 @56x56, batch 64, 2x2 bit, next planes only", 64, 56, 64, 64, 2, "planes"),
             ("128->128 @28x28, batch 256, 3x3 bit, next planes", 256, 28, 128, 128, 3, "planes"),
             ("256->256 @14x14, batch 256, 3x3 bit, next planes", 256, 14, 256, 256, 3, "planes"),
             ("64->64 @300x300, batch 8, 4x4 bit, next planes", 8, 300, 64, 64, 4, "planes")]
    gen = torch.Generator(device="cuda").manual_seed(190513389)
    table = {}
    for label, B, HW, cin, cout, bits, outs in cases:
        ap = torch.randint(-2**31, 2**31 - 1, (bits, B * HW * HW, cin // 32), dtype=torch.int32, device="cuda", generator=gen)
        wp = torch.randint(-2**31, 2**31 - 1, (bits, cout, 3, 3, cin // 32), dtype=torch.int32, device="cuda", generator=gen)
        sc = (torch.rand(cout, device="cuda", generator=gen) + 0.5) / (3.0 * cin ** 0.5 * ((1 << bits) - 1) ** 2 / 3)
        d = qnn.qnn_conv_desc(B, HW, HW, cin, cout, 3, 3, 1, 1, bits, bits)
        # the product library's results are what the instrumented kernels must reproduce
        if outs == "acc+out":
            r_acc, r_out, _ = qnn.qnn_conv2d(ap, wp, (B, HW, HW), cin, 1, 1, scale=sc, want_out=True)
            acc, out, nxt, ref = torch.empty_like(r_acc), torch.empty_like(r_out), None, (r_acc, r_out)
        else:
            _, _, r_nxt = qnn.qnn_conv2d(ap, wp, (B, HW, HW), cin, 1, 1, scale=sc, want_acc=False, next_clip=3.0, next_bits=bits)
            acc, out, nxt, ref = None, None, torch.empty_like(r_nxt), (r_nxt,)
        row = {}
        for hint in (False, True):
            buf = torch.zeros((512 * 8, 5), dtype=torch.int64, device="cuda")
            probe.qnn_timeline_set(buf, pair_hint=hint)
            launch = lambda: probe.timeline_conv2d(d, ap, wp, sc, acc, out, nxt, 3.0, bits if nxt is not None else 0)  # noqa: E731
            settle(torch, launch)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                launch()
            e1.record()
            torch.cuda.synchronize()
            same = all(torch.equal(a, b) for a, b in zip(ref, [t for t in (acc, out, nxt) if t is not None]))
            t = buf.cpu().numpy()
            t = t[t[:, 0] > 0]
            waves = len(t)
            wpw = waves // 512 if waves % 512 == 0 else 0     # waves per workgroup when the grid is 2 per CU
            base = t[:, 0].min()
            end = (t[:, 2] - base) * 0.01
            entry = {"us_per_launch_10_back_to_back": round(e0.elapsed_time(e1) * 100, 1), "waves": waves,
                     "results_equal_libqnn": bool(same),
                     "start_spread_us": round(float((t[:, 0] - base).max()) * 0.01, 2),
                     "prologue_us_mean": round(float((t[:, 1] - t[:, 0]).mean()) * 0.01, 2),
                     "wave_end_us": {"mean": round(float(end.mean()), 1), "p10": round(float(sorted(end)[waves // 10]), 1),
                                     "p90": round(float(sorted(end)[waves * 9 // 10]), 1), "max": round(float(end.max()), 1)}}
            ratio = float(t[:, 4].sum()) / float((t[:, 2] - t[:, 0]).sum())
            if ratio > 1.5:      # s_memtime counts shader cycles
                entry["clock_ghz"] = round(ratio * 0.1, 3)
                entry["wave_life_cycles_mean"] = round(float(t[:, 4].mean()))
            if wpw:
                half = 256 * wpw
                entry["first_dispatched_workgroups_end_us_mean"] = round(float(end[:half].mean()), 1)
                entry["second_dispatched_workgroups_end_us_mean"] = round(float(end[half:].mean()), 1)
                cu = ((t[:, 3] >> 32) & 15) * 4096 + ((t[:, 3] >> 8) & 0xff)         # XCC id, SE / SH / CU id fields of HW_ID
                pairs = sum(1 for b in range(256) if cu[b * wpw] == cu[(b + 256) * wpw])
                entry["workgroups_b_and_b_plus_256_on_one_cu"] = "%d of 256" % pairs
            row["pair balance on" if hint else "pair balance off"] = entry
        probe.qnn_timeline_set(None)
        table[label] = row
    return {"metric": "wave timeline of the convolution kernel", "value": None, "unit": "us", "n_gpus": 1, "steps": 10, "warmup": 0,
            "settle_ms": SETTLE_MS, "ms_per_step": None, "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "u32 bit-planes",
            "data": "synthetic", "config": {"workload": "qnn_conv2d of libqnn_timeline.so, 3x3 stride 1 pad 1"}, "timeline": table,
            "level_gemm_timeline": level_gemm_timeline(torch)}


def level_gemm_timeline(torch):
    """Wave timestamps of the matrix-core GEMM at 4096^3 (libqnn_timeline.so): how long prologue, reduction loop and
    epilogue take, how many shader cycles the loop takes against the 65,536 that its 2048 MFMAs per SIMD need at the
    instruction's published rate, and the clock the chip holds in the loop -- on zeros, on the levels of 2-bit codes
    and on random bytes, since the power the matrix cores draw depends on what they multiply."""
    from paper_1905_13389_amd import probe, qnn
    size = 4096
    gen = torch.Generator(device="cuda").manual_seed(190513389)
    sc = torch.rand(size, device="cuda", generator=gen) + 0.5
    acc = torch.empty((size, size), dtype=torch.int32, device="cuda")
    out = torch.empty((size, size), dtype=torch.float32, device="cuda")
    table = {}
    for fp4 in (False, True):
        nb = qnn.qnn_fp4_row_bytes(size) if fp4 else qnn.qnn_level_row_bytes(size)
        nib = torch.tensor([0xD, 0xA, 0x2, 0x5], dtype=torch.uint8, device="cuda")      # E2M1 codes of -3, -1, 1, 3
        kinds = [("zeros", lambda: torch.zeros((size, nb), dtype=torch.uint8, device="cuda"))]
        if fp4:
            kinds.append(("levels of 2-bit codes", lambda: nib[torch.randint(0, 4, (size, nb), device="cuda", generator=gen)]
                          | (nib[torch.randint(0, 4, (size, nb), device="cuda", generator=gen)] << 4)))
        else:
            kinds.append(("levels of 2-bit codes", lambda: (2 * torch.randint(0, 4, (size, nb), device="cuda", generator=gen) - 3)
                          .to(torch.int8).view(torch.uint8)))
            kinds.append(("random bytes", lambda: torch.randint(0, 256, (size, nb), device="cuda", generator=gen).to(torch.uint8)))
        for kind, make in kinds:
            a, w = make().contiguous(), make().contiguous()
            view = (lambda t: t) if fp4 else (lambda t: t.view(torch.int8))
            ref = (qnn.qnn_level_gemm_fp4 if fp4 else qnn.qnn_level_gemm_i8)(view(a), view(w), size, scale=sc)
            for outs, pa, po in (("acc + out", acc, out), ("acc only", acc, None)):
                buf = torch.zeros((256 * 8, 6), dtype=torch.int64, device="cuda")
                probe.qnn_level_gemm_timeline_set(buf)
                launch = lambda: probe.timeline_level_gemm(a, w, size, size, size, pa, sc, po, fp4=fp4)  # noqa: E731
                settle(torch, launch)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(10):
                    launch()
                e1.record()
                torch.cuda.synchronize()
                same = torch.equal(ref[0], acc) and (po is None or torch.equal(ref[1], out))
                t = buf.cpu().numpy().astype("float64")
                base = t[:, 0].min()
                loop_us = (t[:, 2] - t[:, 1]) * 0.01
                ratio = t[:, 4].sum() / (t[:, 2] - t[:, 1]).sum()
                entry = {"us_per_launch_10_back_to_back": round(e0.elapsed_time(e1) * 100, 1), "results_equal_libqnn": bool(same),
                         "start_spread_us": round(float((t[:, 0] - base).max()) * 0.01, 2),
                         "prologue_us_mean": round(float((t[:, 1] - t[:, 0]).mean()) * 0.01, 2),
                         "loop_us": {"mean": round(float(loop_us.mean()), 1), "max": round(float(loop_us.max()), 1)},
                         "epilogue_us_mean": round(float((t[:, 3] - t[:, 2]).mean()) * 0.01, 2),
                         "last_wave_ends_us": round(float((t[:, 3] - base).max()) * 0.01, 1)}
                if ratio > 1.5:          # s_memtime counts shader cycles
                    entry["clock_in_loop_ghz"] = round(float(ratio) * 0.1, 3)
                    entry["loop_cycles_mean"] = round(float(t[:, 4].mean()))
                    mf = 65536.0 / (2 if fp4 else 1)    # 2048 (fp4: 1024) MFMAs per SIMD, 32 cycles each
                    entry["mfma_cycles_needed"] = round(mf)
                    entry["matrix_core_busy_in_loop"] = round(mf / float(t[:, 4].mean()), 3)
                table["%s, %s, %s" % ("fp4" if fp4 else "int8", kind, outs)] = entry
    probe.qnn_level_gemm_timeline_set(None)
    return table


def fc_workload(args):
    """Config 1: one FC layer, 2 x 2 bit, A [64][512] x W [256][512]: 6.7e7 binary operations, far too
    little to load the chip -- the figure of interest is the latency of the two launches."""
    import torch
    import qnn_workloads as wl
    from paper_1905_13389_amd import qnn

    c = wl.fc_2x2()
    d_a = torch.from_numpy(c["a"]).cuda()
    w_planes = qnn.qnn_encode_pack(torch.from_numpy(c["w"]).cuda(), 1.0, 2)
    d_scale = torch.from_numpy(c["scale"]).cuda()
    a_planes = torch.empty((2, 64, 16), dtype=torch.int32, device="cuda")
    acc = torch.empty((64, 256), dtype=torch.int32, device="cuda")
    out = torch.empty((64, 256), dtype=torch.float32, device="cuda")

    def step():
        qnn.qnn_encode_pack(d_a, 1.0, 2, planes=a_planes)
        qnn.qnn_binary_gemm(a_planes, w_planes, 512, acc=acc, scale=d_scale, out=out)

    steps = max(args.steps, 200)
    for _ in range(max(args.warmup, 20)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    # 20 steps captured once into a HIP graph and replayed: what is left of a step when the host side of its
    # launches (Python, ctypes, the runtime's argument marshalling, one graph launch) is shared by 20 steps
    ref_acc, ref_out = acc.clone(), out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    per_graph = 20
    with torch.cuda.graph(graph):
        for _ in range(per_graph):
            step()
    acc.zero_(), out.zero_()
    for _ in range(20):
        graph.replay()
    torch.cuda.synchronize()
    if not (torch.equal(acc, ref_acc) and torch.equal(out, ref_out)):
        raise SystemExit("bench.py: graph replay of the FC step differs from the eager step")
    t0 = time.perf_counter()
    for _ in range(steps // per_graph):
        graph.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) / (steps // per_graph * per_graph) * 1e3
    # the whole layer in one launch (qnn_fc_fused): same acc and out
    acc.zero_(), out.zero_()
    fused = lambda: qnn.qnn_fc_fused(d_a, 1.0, 2, w_planes, acc=acc, scale=d_scale, out=out)
    for _ in range(20):
        fused()
    torch.cuda.synchronize()
    if not (torch.equal(acc, ref_acc) and torch.equal(out, ref_out)):
        raise SystemExit("bench.py: qnn_fc_fused differs from the two-launch step")
    t0 = time.perf_counter()
    for _ in range(steps):
        fused()
    torch.cuda.synchronize()
    fused_ms = (time.perf_counter() - t0) / steps * 1e3
    ops = 2.0 * 64 * 256 * 512 * 4
    tops = ops / (ms * 1e-3) / 1e12
    # the GEMM launch between its own HIP events (the dominant kernel of the two-launch step)
    evs = []
    for _ in range(20):
        qnn.qnn_encode_pack(d_a, 1.0, 2, planes=a_planes)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        qnn.qnn_binary_gemm(a_planes, w_planes, 512, acc=acc, scale=d_scale, out=out)
        e1.record()
        evs.append((e0, e1))
    torch.cuda.synchronize()
    gemm_ms = sorted(a.elapsed_time(b) for a, b in evs)[len(evs) // 2]
    baseline = None if args.no_cpu_baseline else cpu_baseline_fc(c, min(args.cpu_seconds, 2.0))
    return {
        "metric": "effective binary TOPS (xnor+popcount) and % of VALU/HBM roofline, 1 MI355X", "value": round(tops, 4), "unit": "binary TOP/s",
        "n_gpus": 1, "steps": steps, "warmup": max(args.warmup, 20), "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 bit-planes, int32 accumulate", "data": "synthetic",
        "config": {"workload": "FC 64x512 -> 256, w_bits=2 a_bits=2, int8 levels packed on device",
                   "step": "qnn_encode_pack + qnn_binary_gemm (fused scale)"},
        "roofline": {"bound": "alu", "kernel": "bgemm_tile_kernel<2,2>", "achieved": round(ops / (gemm_ms * 1e-3) / 1e12, 4),
                     "peak": round(PEAK_BINARY_TOPS, 1), "unit": "binary TOP/s",
                     "frac": round(ops / (gemm_ms * 1e-3) / 1e12 / PEAK_BINARY_TOPS, 6), "traffic": None,
                     "kernel_ms": round(gemm_ms, 5), "step_frac": round(tops / PEAK_BINARY_TOPS, 6),
                     "note": "launch / latency bound: 0.04 us of VALU work per step; the time between the events is the "
                             "launch's own latency, not the kernel's arithmetic", "peak_note": PEAK_NOTE},
        "cpu_baseline": baseline,
        "fused": {"step": "qnn_fc_fused: encoders, binary branches, recombination and scale in one launch",
                  "ms_per_step": round(fused_ms, 5), "checked": "acc and out equal the two-launch step's"},
        "hip_graph": {"step": "20 steps (40 launches) captured once and replayed", "ms_per_step": round(graph_ms, 5),
                      "checked": "acc and out of the replays equal the eager step's"}}


def pool_workload(args):
    """2x2 stride-2 max-pooling on the 4-bit planes of the detection stack's first resolution change
    (batch 32, 300x300x64 -> 150x150x64): a streaming kernel, bound by HBM."""
    import torch
    from paper_1905_13389_amd import qnn

    B, H, C, bits = args.batch or 32, 300, 64, 4
    cw = C // 32
    gen = torch.Generator(device="cuda").manual_seed(190513389)
    planes = torch.randint(-2 ** 31, 2 ** 31 - 1, (bits, B * H * H, cw), dtype=torch.int32, device="cuda",
                           generator=gen)
    ho = qnn.qnn_pool_out_size(H, 2, 2)
    out = torch.empty((bits, B * ho * ho, cw), dtype=torch.int32, device="cuda")
    ms = timed_ms(torch, lambda: qnn.qnn_maxpool_planes(planes, (B, H, H), C, 2, 2, out=out), args.steps, args.warmup)
    nbytes = 4.0 * (planes.numel() + out.numel())
    tbs = nbytes / (ms * 1e-3) / 1e12
    return {
        "metric": "max-pooling on bit-planes, HBM bytes per second", "value": round(tbs, 3), "unit": "TB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32 bit-planes",
        "data": "synthetic",
        "config": {"workload": "2x2 stride-2 max-pool, batch %d, 300x300x64, 4-bit planes" % B,
                   "step": "qnn_maxpool_planes"},
        "roofline": {"bound": "hbm", "kernel": "maxpool_planes_kernel<4>", "achieved": round(tbs * 1e3, 1),
                     "peak": 8000.0, "unit": "GB/s", "frac": round(tbs / 8.0, 4), "traffic": None,
                     "algorithmic_bytes": nbytes}}


def deconv_workload(args):
    """A 2x upsampling transposed convolution (4x4 kernel, stride 2, pad 1) of decoder shape: batch 64,
    28x28x128 -> 56x56x64, 2x2 bit, fused next-layer planes; the four phases in one launch of the conv kernel."""
    import torch
    import qnn_workloads as wl
    from paper_1905_13389_amd import qnn

    B, H, cin, cout, k, s, pad, bits = args.batch or 64, 28, 128, 64, 4, 2, 1, 2
    x = torch.from_numpy(wl.rng(7, 0).standard_normal((B * H * H, cin), dtype="float32")).cuda()
    w = torch.from_numpy(wl.odd_levels(wl.rng(7, 1), (cout, k, k, cin), bits)).cuda()
    sc = torch.from_numpy(wl.channel_scales(wl.rng(7, 2), cout)).cuda()
    ph = qnn.qnn_deconv_pack_weights(qnn.qnn_encode_pack(w, 1.0, bits).view(bits, cout, k, k, -1), cin, s)
    planes = qnn.qnn_encode_pack(x, 3.0, bits)
    ho = (H - 1) * s - 2 * pad + k
    nxt = torch.empty((bits, B * ho * ho, (cout + 31) // 32), dtype=torch.int32, device="cuda")

    def step():
        qnn.qnn_deconv2d(planes, ph, (B, H, H), cin, cout, k, k, s, pad, bits, scale=sc, want_acc=False,
                         next_clip=3.0, next_bits=bits, next_planes=nxt)

    ms = timed_ms(torch, step, args.steps, args.warmup)
    macs = B * H * H * k * k * cin * cout
    tops = 2.0 * macs * bits * bits / (ms * 1e-3) / 1e12

    # the same layer on the matrix cores (comparison only): int8 / fp4 levels in, the next layer's levels out;
    # zeros inserted between the input pixels, then the stride-1 level convolution with the flipped kernel
    lv = qnn.qnn_encode_levels_i8(x.view(B, H, H, cin), 3.0, bits)
    variants = {}
    for name, a_lv, w_lv, entry in (("mfma_variant", lv, w, qnn.qnn_level_deconv2d_i8),
                                    ("fp4_variant", qnn.qnn_levels_to_fp4(lv), qnn.qnn_levels_to_fp4(w), qnn.qnn_level_deconv2d_fp4)):
        fw = qnn.qnn_level_deconv_flip_weights(w_lv)
        ws = torch.empty((B * (2 * H - 1) * (2 * H - 1) * a_lv.shape[3],), dtype=torch.uint8, device="cuda")
        nl = torch.empty((B, ho, ho, cout // (2 if a_lv.dtype == torch.uint8 else 1)), dtype=a_lv.dtype, device="cuda")
        v_ms = timed_ms(torch, lambda: entry(a_lv, fw, s, pad, bits, bits, scale=sc, want_acc=False, next_clip=3.0,
                                             next_bits=bits, next_levels=nl, workspace=ws), args.steps, args.warmup)
        variants[name] = {"step": entry.__name__ + " (zero insertion + level convolution, fused scale/quantize epilogue)",
                          "ms_per_step": round(v_ms, 4), "speedup_vs_xor_bitcount_step": round(ms / v_ms, 2),
                          "note": "the level convolution multiplies the inserted zeros too: 4x the products of the layer"}
    return {
        **variants,
        "metric": "effective binary TOPS (xnor+popcount) and % of VALU/HBM roofline, 1 MI355X", "value": round(tops, 2),
        "unit": "binary TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32 bit-planes, int32 accumulate",
        "data": "synthetic",
        "config": {"workload": "transposed conv 4x4 stride 2, batch %d, 28x28x128 -> 56x56x64, 2x2 bit" % B, "macs": macs,
                   "step": "qnn_deconv2d (the four phases in one launch, fused scale/quantize/pack epilogue)"},
        "roofline": {"bound": "alu", "achieved": round(tops, 2), "peak": round(PEAK_BINARY_TOPS, 1),
                     "unit": "binary TOP/s", "frac": round(tops / PEAK_BINARY_TOPS, 4), "traffic": None,
                     "note": "host-timed step of one launch"}}


def grad_workload(args):
    """The training-side gradients on config 3's activation tensor (batch 64, 56x56x64 fp32): the
    straight-through gradient of the ladder and the 2-bit encoder's surrogate gradient; streaming, HBM bound."""
    import torch
    from paper_1905_13389_amd import qnn

    n = (args.batch or 64) * 56 * 56 * 64
    gen = torch.Generator(device="cuda").manual_seed(190513389)
    x = torch.randn(n, device="cuda", generator=gen)
    g = torch.randn((2, n), device="cuda", generator=gen)
    gx = torch.empty_like(x)

    ms_ste = timed_ms(torch, lambda: qnn.qnn_quantize_ste_backward(x, g[0], 3.0, grad_x=gx), args.steps, args.warmup)
    ms_enc = timed_ms(torch, lambda: qnn.qnn_encoder_backward(x, g, 3.0, grad_x=gx), args.steps, args.warmup)
    b_ste, b_enc = 12.0 * n, 16.0 * n          # x + gradient(s) read, grad_x written
    tbs = b_enc / (ms_enc * 1e-3) / 1e12
    return {
        "metric": "encoder surrogate gradient, HBM bytes per second", "value": round(tbs, 3), "unit": "TB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_enc, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%d fp32 activations, 2-bit encoder" % n, "step": "qnn_encoder_backward"},
        "roofline": {"bound": "hbm", "kernel": "encoder_backward_kernel<2, 4>", "achieved": round(tbs * 1e3, 1),
                     "peak": 8000.0, "unit": "GB/s", "frac": round(tbs / 8.0, 4), "traffic": None,
                     "algorithmic_bytes": b_enc},
        "quantize_ste_backward": {"ms": round(ms_ste, 5), "GB/s": round(b_ste / (ms_ste * 1e-3) / 1e9, 1),
                                  "frac": round(b_ste / (ms_ste * 1e-3) / 8e12, 4), "algorithmic_bytes": b_ste}}


def config_summaries(args):
    """Configurations 1, 3, 4 and 5 of the benchmark table next to the headline (configuration 2): step time, the
    dominant kernel's own event-timed duration, its fraction of the one stated peak, and the oracle on a sample."""
    import copy
    out = {}
    plan = (("1_fc_2x2", "fc1", 200), ("3_resnet_conv_2x2", "conv3", 20), ("4_resnet18_stack_3x3", "stack4", 10),
            ("5_vgg_ssd_stack_4x4", "stack5", 5))
    for key, workload, steps in plan:
        a = copy.copy(args)
        a.workload, a.steps, a.warmup, a.batch = workload, steps, 3, 0
        a.cpu_seconds = min(args.cpu_seconds, 4.0)
        r = fc_workload(a) if workload == "fc1" else conv_workload(a)
        roof = r["roofline"]
        out[key] = {"workload": r["config"]["workload"], "step": r["config"]["step"], "steps": steps,
                    "ms_per_step": r["ms_per_step"], "binary_tops": r["value"],
                    "dominant_kernel": roof.get("kernel"), "kernel_ms": roof.get("kernel_ms"),
                    "frac": roof["frac"], "step_frac": roof.get("step_frac"), "peak": roof["peak"],
                    "slowest_layer": roof.get("slowest_layer"), "note": roof.get("note"),
                    "matrix_core_step_ms": (r.get("mfma_variant") or {}).get("ms_per_step"),
                    "cpu_baseline": r.get("cpu_baseline")}
        if workload == "fc1":
            out[key]["one_launch_ms"] = r["fused"]["ms_per_step"]
    return out


def main():
    global SETTLE_MS
    args = parse()
    if args.no_settle:
        SETTLE_MS = 0.0
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards by output rows with no "
              "exchange; no multi-GPU figure is produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    runners = {"trunk": trunk_workload, "pool": pool_workload, "grad": grad_workload, "deconv": deconv_workload,
               "fc1": fc_workload, "gemm": gemm_workload, "ssd": graph_workload, "probe": probe_workload,
               "timeline": timeline_workload}
    result = runners.get(args.workload, conv_workload)(args)
    if args.workload == "gemm" and not args.no_configs:
        result["configs"] = config_summaries(args)
    print(json.dumps(result))


def gemm_workload(args):
    import numpy as np
    import torch
    import qnn_workloads as wl
    from paper_1905_13389_amd import qnn

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    size, wb, ab = args.size, args.w_bits, args.a_bits
    cfg = wl.gemm_square(wb, ab, size)
    x = wl.gemm_float_activations(size, size)
    clip = float(np.float32(3.0 * np.std(x.astype(np.float64))))

    d_x = torch.from_numpy(x).cuda()
    d_scale = torch.from_numpy(cfg["scale"]).cuda()
    w_planes = qnn.qnn_encode_pack(torch.from_numpy(cfg["w"]).cuda(), 1.0, wb)   # offline
    nw = (size + 31) // 32
    a_planes = torch.empty((ab, size, nw), dtype=torch.int32, device="cuda")
    acc = torch.empty((size, size), dtype=torch.int32, device="cuda")
    out = torch.empty((size, size), dtype=torch.float32, device="cuda")

    def step():
        qnn.qnn_encode_pack(d_x, clip, ab, planes=a_planes)
        qnn.qnn_binary_gemm(a_planes, w_planes, size, acc=acc, scale=d_scale, out=out)

    # the register-only issue-rate loops run first: they belong to the roofline object and leave the
    # clocks settled before the W warm-up steps
    probe = valu_probe(torch)
    mprobe = mfma_probe(torch)  # what register-only MFMA loops sustain on this device (the variants' context)
    for _ in range(args.warmup):
        step()
    # one streaming pass of known size (64 MiB read, 64 MiB written at the default size): the
    # reference launch that calibrates the HBM byte counters when this command runs under rocprofv3
    qnn.qnn_dequant_scale(acc, d_scale, out=out)
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps between two device synchronisations; event pairs around every
    # EVENT_EVERY-th GEMM launch give the dominant kernel's own duration on the stream it runs on (torch's current
    # stream) -- every launch would add about 1 % to the step time through the event markers themselves.  The
    # region is run `repeats` times; the median repetition is the one reported (all are listed).
    runs = []
    for _ in range(max(1, args.repeats)):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(0, args.steps, EVENT_EVERY)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            qnn.qnn_encode_pack(d_x, clip, ab, planes=a_planes)
            timed = i % EVENT_EVERY == 0
            if timed:
                ev[i // EVENT_EVERY][0].record()
            qnn.qnn_binary_gemm(a_planes, w_planes, size, acc=acc, scale=d_scale, out=out)
            if timed:
                ev[i // EVENT_EVERY][1].record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        runs.append((dt / args.steps * 1e3, sum(a.elapsed_time(b) for a, b in ev) / len(ev)))
    runs.sort()
    ms_per_step, gemm_ms = runs[len(runs) // 2]

    ops = 2.0 * size * size * size * wb * ab
    value = ops / (ms_per_step * 1e-3) / 1e12
    achieved = ops / (gemm_ms * 1e-3) / 1e12
    # what the chip itself showed in this run: the clock it held under the xor / count loops and their cost in
    # real cycles, hence the rate a SIMD sustains on nothing but pairs
    pair = probe[probe["best_pair_order"]]
    sustained = probe["pair_binary_tops"]

    result = {
        "metric": "effective binary TOPS (xnor+popcount) and % of VALU/HBM roofline, 1 MI355X",
        "value": round(value, 2), "unit": "binary TOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u32 bit-planes, int32 accumulate",
        "data": "synthetic",
        "repeat_ms_per_step": [round(r[0], 4) for r in runs],
        "config": {"workload": "square binary-decomposed GEMM %dx%dx%d, w_bits=%d a_bits=%d, "
                               "fp32 activations encoded on device, int32 acc + fp32 scaled out"
                               % (size, size, size, wb, ab),
                   "step": "qnn_encode_pack + qnn_binary_gemm (fused scale)"},
        "roofline": {"bound": "alu", "kernel": "bgemm_tile_kernel<%d,%d>" % (wb, ab),
                     "achieved": round(achieved, 2), "peak": round(PEAK_BINARY_TOPS, 1),
                     "unit": "binary TOP/s", "frac": round(achieved / PEAK_BINARY_TOPS, 4),
                     "kernel_ms": round(gemm_ms, 4),
                     "traffic": GEMM_2X2_4096_TRAFFIC_BYTES if (size, wb, ab) == (4096, 2, 2) else None,
                     "traffic_source": "profiles/bgemm_2x2_4096_hbm_counters.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                       "of this command, calibrated; a constant of that profile, not measured in this run)",
                     "peak_note": PEAK_NOTE,
                     "sustained_pair_loop": sustained,
                     "frac_of_sustained_pair_loop": round(achieved / sustained, 4),
                     "clock_ghz_under_pair_loop": pair.get("clock_ghz"),
                     "probe": probe},
    }

    # The bit-plane-sum variant on the matrix cores, same workload and outputs (comparison only:
    # the headline value above is the xor + bitcount path).  Step = encode + plane sum of the
    # activations + int8 MFMA GEMM with fused scale; the weights' levels are made once, offline.
    if max(wb, ab) <= 7:
        w_levels = qnn.qnn_plane_sum_i8(w_planes, size)
        a_levels = torch.empty((size, qnn.qnn_level_row_bytes(size)), dtype=torch.int8, device="cuda")

        def mfma_step():
            qnn.qnn_encode_pack(d_x, clip, ab, planes=a_planes)
            qnn.qnn_plane_sum_i8(a_planes, size, levels=a_levels)
            qnn.qnn_level_gemm_i8(a_levels, w_levels, size, acc=acc, scale=d_scale, out=out)

        for _ in range(args.warmup):
            mfma_step()
        evm = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(0, args.steps, EVENT_EVERY)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            qnn.qnn_encode_pack(d_x, clip, ab, planes=a_planes)
            qnn.qnn_plane_sum_i8(a_planes, size, levels=a_levels)
            if i % EVENT_EVERY == 0:
                evm[i // EVENT_EVERY][0].record()
            qnn.qnn_level_gemm_i8(a_levels, w_levels, size, acc=acc, scale=d_scale, out=out)
            if i % EVENT_EVERY == 0:
                evm[i // EVENT_EVERY][1].record()
        torch.cuda.synchronize()
        m_ms = (time.perf_counter() - t0) / args.steps * 1e3
        m_gemm_ms = sum(a.elapsed_time(b) for a, b in evm) / len(evm)
        int8_tops = 2.0 * size ** 3 / (m_gemm_ms * 1e-3) / 1e12
        result["mfma_variant"] = {
            "step": "qnn_encode_pack + qnn_plane_sum_i8 + qnn_level_gemm_i8 (fused scale)",
            "ms_per_step": round(m_ms, 4), "effective_binary_tops": round(ops / (m_ms * 1e-3) / 1e12, 1),
            "speedup_vs_xor_bitcount_step": round(ms_per_step / m_ms, 2),
            "roofline": {"bound": "mfma", "kernel": "level_gemm_mfma_kernel<int8>", "achieved": round(int8_tops, 1),
                         "peak": 5000.0, "unit": "int8 TOP/s", "frac": round(int8_tops / 5000.0, 4),
                         "kernel_ms": round(m_gemm_ms, 4), "probe_mfma_loop": mprobe["int8"],
                         "frac_of_probe": round(int8_tops / mprobe["int8"], 4),
                         "probe_mfma_loop_by_operand_data": mprobe["by_operand_data"]["int8"],
                         "frac_of_probe_on_level_operands": round(
                             int8_tops / mprobe["by_operand_data"]["int8"]["levels_of_2bit_codes"]["tops"], 4),
                         "clock_note": "the published peak is at 2.4 GHz; under MFMA load the clock the chip holds depends on "
                                       "the operand data (by_operand_data: the register-only loop on zeros, on levels, on random bytes)"}}

    # 1- and 2-bit codes also fit the fp4 matrix-core path (levels -3..3 are exact fp4 values)
    if max(wb, ab) <= 2:
        w4 = qnn.qnn_plane_sum_fp4(w_planes, size)
        a4 = torch.empty((size, qnn.qnn_fp4_row_bytes(size)), dtype=torch.uint8, device="cuda")

        def fp4_step():
            qnn.qnn_encode_pack(d_x, clip, ab, planes=a_planes)
            qnn.qnn_plane_sum_fp4(a_planes, size, levels=a4)
            qnn.qnn_level_gemm_fp4(a4, w4, size, acc=acc, scale=d_scale, out=out)

        for _ in range(args.warmup):
            fp4_step()
        evf = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(0, args.steps, EVENT_EVERY)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            qnn.qnn_encode_pack(d_x, clip, ab, planes=a_planes)
            qnn.qnn_plane_sum_fp4(a_planes, size, levels=a4)
            if i % EVENT_EVERY == 0:
                evf[i // EVENT_EVERY][0].record()
            qnn.qnn_level_gemm_fp4(a4, w4, size, acc=acc, scale=d_scale, out=out)
            if i % EVENT_EVERY == 0:
                evf[i // EVENT_EVERY][1].record()
        torch.cuda.synchronize()
        f_ms = (time.perf_counter() - t0) / args.steps * 1e3
        f_gemm_ms = sum(a.elapsed_time(b) for a, b in evf) / len(evf)
        fp4_tops = 2.0 * size ** 3 / (f_gemm_ms * 1e-3) / 1e12
        result["fp4_variant"] = {
            "step": "qnn_encode_pack + qnn_plane_sum_fp4 + qnn_level_gemm_fp4 (fused scale)",
            "ms_per_step": round(f_ms, 4), "effective_binary_tops": round(ops / (f_ms * 1e-3) / 1e12, 1),
            "speedup_vs_xor_bitcount_step": round(ms_per_step / f_ms, 2),
            "roofline": {"bound": "mfma", "kernel": "level_gemm_mfma_kernel<fp4>", "achieved": round(fp4_tops, 1),
                         "peak": 10100.0, "unit": "fp4 TFLOP/s", "frac": round(fp4_tops / 10100.0, 4),
                         "kernel_ms": round(f_gemm_ms, 4), "probe_mfma_loop": mprobe["fp4"],
                         "frac_of_probe": round(fp4_tops / mprobe["fp4"], 4),
                         "probe_mfma_loop_by_operand_data": mprobe["by_operand_data"]["fp4"],
                         "frac_of_probe_on_level_operands": round(
                             fp4_tops / mprobe["by_operand_data"]["fp4"]["levels_of_2bit_codes"]["tops"], 4),
                         "clock_note": "the published peak is at 2.4 GHz; under MFMA load the clock the chip holds depends on "
                                       "the operand data (by_operand_data: the register-only loop on zeros, on levels, on random bytes)"}}

    if args.sweep:
        sweep = {}
        combos = [(w_b, a_b) for w_b in range(1, 5) for a_b in range(1, 5)] + [(5, 5), (6, 6), (7, 7)]
        for w_b, a_b in combos:
            c2 = wl.gemm_square(w_b, a_b, size)
            wp = qnn.qnn_encode_pack(torch.from_numpy(c2["w"]).cuda(), 1.0, w_b)
            apl = qnn.qnn_encode_pack(torch.from_numpy(c2["a"]).cuda(), 1.0, a_b)
            # the host-side generation above leaves the GPU idle for seconds: warm up until the clocks are back
            t_warm = time.perf_counter()
            while time.perf_counter() - t_warm < 0.08:
                for _ in range(5):
                    qnn.qnn_binary_gemm(apl, wp, size, acc=acc)
                torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                qnn.qnn_binary_gemm(apl, wp, size, acc=acc)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 10
            tops = 2.0 * size ** 3 * w_b * a_b / (ms * 1e-3) / 1e12
            sweep["%dx%d" % (w_b, a_b)] = {"ms": round(ms, 4), "binary_tops": round(tops, 1),
                                           "frac": round(tops / PEAK_BINARY_TOPS, 4)}
        result["sweep"] = sweep

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, wb, ab, args.cpu_seconds)
    return result


if __name__ == "__main__":
    main()
