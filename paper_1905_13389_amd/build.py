"""Compile the HIP sources under csrc/ for gfx950: paper_1905_13389_amd/libqnn.so (the product library,
include/qnn.h) paper_1905_13389_amd/libqnn_probe.so (the benchmark's issue-rate loops, include/qnn_probe.h) and
paper_1905_13389_amd/libqnn_timeline.so (the convolution kernels with wave timestamps, same header).

hipcc cross-compiles without a GPU.  Flags: contraction off (the quantizer's fp32 steps must stay
single IEEE operations) and the packed-fp32 target feature off.  libqnn.so carries a digest of its
sources (qnn_build_id) so that the binding can tell a library that is older than the sources beside it.
"""
import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqnn.so")
PROBE_LIB = os.path.join(HERE, "libqnn_probe.so")
TIMELINE_LIB = os.path.join(HERE, "libqnn_timeline.so")
SOURCES = ["qnn_api.hip", "encode_pack.hip", "dequant_scale.hip", "binary_gemm.hip", "conv2d.hip", "conv2d_block.hip",
           "level_gemm_mfma.hip", "level_conv_mfma.hip", "maxpool.hip", "ste_backward.hip", "dense.hip", "fc_fused.hip",
           "no_alloc.hip"]
PROBE_SOURCES = ["probe.hip"]
# the convolution entry points and the matrix-core GEMM once more, with wave timestamps (-DQNN_TIMELINE): a
# diagnostic library of its own
TIMELINE_SOURCES = ["qnn_api.hip", "conv2d.hip", "conv2d_block.hip", "level_gemm_mfma.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def source_id():
    """Digest of everything libqnn.so is compiled from: csrc/*.hip, csrc/*.h (the probe's file aside),
    include/qnn.h and the compiler flags."""
    h = hashlib.sha256(" ".join(FLAGS).encode())
    names = sorted(f for f in os.listdir(CSRC) if f.endswith((".hip", ".h")) and f not in PROBE_SOURCES)
    for path in [os.path.join(CSRC, f) for f in names] + [os.path.join(INCLUDE, "qnn.h")]:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:32]


def _compile(job):
    src, defines = job
    obj = os.path.join(OBJ, src.replace(".hip", "_timeline.o" if "-DQNN_TIMELINE" in defines else ".o"))
    cmd = ["hipcc"] + FLAGS + defines + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, log))
    return obj, log


def _link(objs, lib):
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib + ".tmp"] + objs
    subprocess.run(cmd, check=True)
    os.replace(lib + ".tmp", lib)


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    build_id = source_id()
    jobs = [(s, ['-DQNN_BUILD_ID="%s"' % build_id] if s == "qnn_api.hip" else []) for s in SOURCES + PROBE_SOURCES]
    jobs += [(s, ["-DQNN_TIMELINE"]) for s in TIMELINE_SOURCES]
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1, 8)) as ex:
        results = list(ex.map(_compile, jobs))
    if verbose:
        for _, log in results:
            if log.strip():
                print(log)
    objs = [o for o, _ in results]
    _link(objs[:len(SOURCES)], LIB)
    _link(objs[len(SOURCES):len(SOURCES) + len(PROBE_SOURCES)], PROBE_LIB)
    _link(objs[len(SOURCES) + len(PROBE_SOURCES):], TIMELINE_LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
