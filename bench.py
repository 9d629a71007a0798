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

# MI355X: 256 CUs x 4 SIMDs x 16 lanes at 2.4 GHz, one 32-bit VALU lane-op per lane and clock.
# A plane pair costs one v_xor_b32 and one v_bcnt_u32_b32 per 32 bit-pairs, counted as 2 binary
# operations per bit-pair (xnor and count, the 2*MAC convention): 32 * 2 / 2 = 32 per lane-op.
VALU_LANE_OPS_PER_S = 256 * 4 * 16 * 2.4e9
PEAK_BINARY_TOPS = VALU_LANE_OPS_PER_S * 32 / 1e12


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--size", type=int, default=4096, help="rows = cols = n of the square GEMM")
    ap.add_argument("--w-bits", type=int, default=2)
    ap.add_argument("--a-bits", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--sweep", action="store_true", help="also print GEMM-only times for all 1..4 x 1..4 bits")
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
    t0 = time.perf_counter()
    oracle.gemm(cfg["a"][:rows], cfg["w"])
    dt = time.perf_counter() - t0
    ops = 2.0 * rows * cols * size * w_bits * a_bits
    return {"value": ops / dt / 1e12, "unit": "effective binary TOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": "%d of %d rows x %d cols x n=%d, %.2f s, %.2f GMAC/s" %
            (rows, cfg["a"].shape[0], cols, size, dt, rows * cols * size / dt / 1e9)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards by output rows with no "
              "exchange; no multi-GPU figure is produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

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

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps; event pairs around each GEMM launch give the dominant
    # kernel's own duration on the stream it runs on (torch's current stream)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        qnn.qnn_encode_pack(d_x, clip, ab, planes=a_planes)
        ev[i][0].record()
        qnn.qnn_binary_gemm(a_planes, w_planes, size, acc=acc, scale=d_scale, out=out)
        ev[i][1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    gemm_ms = sum(a.elapsed_time(b) for a, b in ev) / args.steps

    ops = 2.0 * size * size * size * wb * ab
    value = ops / (ms_per_step * 1e-3) / 1e12
    achieved = ops / (gemm_ms * 1e-3) / 1e12

    result = {
        "metric": "effective binary TOPS (xnor+popcount), 1 MI355X",
        "value": round(value, 2), "unit": "binary TOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u32 bit-planes, int32 accumulate",
        "data": "synthetic",
        "config": {"workload": "square binary-decomposed GEMM %dx%dx%d, w_bits=%d a_bits=%d, "
                               "fp32 activations encoded on device, int32 acc + fp32 scaled out"
                               % (size, size, size, wb, ab),
                   "step": "qnn_encode_pack + qnn_binary_gemm (fused scale)"},
        "roofline": {"bound": "alu", "kernel": "bgemm_tile_kernel<%d,%d>" % (wb, ab),
                     "achieved": round(achieved, 2), "peak": round(PEAK_BINARY_TOPS, 1),
                     "unit": "binary TOP/s", "frac": round(achieved / PEAK_BINARY_TOPS, 4),
                     "kernel_ms": round(gemm_ms, 4), "traffic": None},
    }

    if args.sweep:
        sweep = {}
        for w_b in range(1, 5):
            for a_b in range(1, 5):
                c2 = wl.gemm_square(w_b, a_b, size)
                wp = qnn.qnn_encode_pack(torch.from_numpy(c2["w"]).cuda(), 1.0, w_b)
                apl = qnn.qnn_encode_pack(torch.from_numpy(c2["a"]).cuda(), 1.0, a_b)
                for _ in range(3):
                    qnn.qnn_binary_gemm(apl, wp, size, acc=acc)
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
    print(json.dumps(result))


if __name__ == "__main__":
    main()
