"""AddressSanitizer + UndefinedBehaviorSanitizer runs of everything that executes on the host: the CPU oracle's
C code, and the argument checking of every libqnn entry point.  Both are compiled here into stand-alone
executables (the sanitizer runtime is linked in, so nothing is preloaded into Python): the oracle with gcc; the
library's sources with hipcc in host-only mode (no device code is generated: seconds instead of minutes) and
linked against a stub of the HIP runtime that counts device calls.  No GPU."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOSTCHECK = os.path.join(ROOT, "tests", "hostcheck")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    return r.returncode, r.stdout


def _clean(output):
    return "\n".join(l for l in output.splitlines() if "packed-fp32-ops" not in l)


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    rc, out = _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra"] + SAN +
                   [os.path.join(ROOT, "oracle", "qnn_oracle.c"), os.path.join(HOSTCHECK, "oracle_sanitized.c"),
                    "-o", exe, "-lm"])
    assert rc == 0, out
    rc, out = _run([exe], env=dict(ENV, OMP_NUM_THREADS="2"))
    assert rc == 0 and "oracle_sanitized: ok" in out, out
    assert "runtime error" not in out and "AddressSanitizer" not in out, out


@pytest.mark.skipif(shutil.which("hipcc") is None or shutil.which("amdclang++") is None,
                    reason="hipcc and amdclang++ are needed for the host-only build")
def test_argument_checks_under_sanitizers(tmp_path):
    from paper_1905_13389_amd import build
    host_flags = ["--offload-arch=gfx950", "--offload-host-only", "-O1", "-g", "-std=c++17", "-fPIC", "-ffp-contract=off",
                  "-Wno-unused-command-line-argument"]
    for flag in SAN:
        host_flags += ["-Xarch_host", flag]

    def compile_one(src):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        rc, out = _run(["hipcc"] + host_flags + ["-c", src, "-o", obj])
        assert rc == 0, _clean(out)
        return obj

    sources = [os.path.join(build.CSRC, s) for s in build.SOURCES]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(compile_one, sources))
    # a host-only object refers to the device image that would normally be embedded next to it: give every
    # such symbol a few zero bytes (the stub runtime never looks at them)
    rc, out = _run(["nm", "-u"] + objs)
    assert rc == 0, out
    fatbins = sorted({l.split()[-1] for l in out.splitlines() if "__hip_fatbin_" in l})
    assert fatbins
    blobs = str(tmp_path / "fatbin_blobs.cpp")
    with open(blobs, "w") as f:
        for name in fatbins:
            f.write('extern "C" { extern const char %s[64]; const char %s[64] = {0}; }\n' % (name, name))
    exe = str(tmp_path / "abi_errors")
    # clang's own sanitizer runtimes: the objects above come from the same compiler
    rc, out = _run(["amdclang++", "-O1", "-g", "-std=c++17"] + SAN +
                   [os.path.join(HOSTCHECK, "abi_errors.cpp"), os.path.join(HOSTCHECK, "hip_runtime_stub.cpp"), blobs] +
                   objs + ["-o", exe, "-lpthread"])
    assert rc == 0, out
    rc, out = _run([exe], env=ENV)
    assert rc == 0 and " 0 failures" in out, out
    assert "runtime error" not in out and "AddressSanitizer" not in out, out
