"""Build libef.so (HIP kernels + C ABI) and libef_bench.so (the bandwidth probes bench.py runs
beside it) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libef.so")
BENCH_LIB = os.path.join(HERE, "libef_bench.so")
# library -> (source, everything it is built from)
TARGETS = {
    LIB: (os.path.join(CSRC, "ef_api.hip"),
          [os.path.join(CSRC, h) for h in ("ef_device.h", "ef_tile.h", "ef_worker.h", "ef_server.h", "ef_finish.h",
                                           "ef_quality.h")] +
          [os.path.join(ROOT, "include", h) for h in ("ef.h", "ef_debug.h")]),
    BENCH_LIB: (os.path.join(CSRC, "ef_bench.hip"),
                [os.path.join(CSRC, h) for h in ("ef_tile.h", "ef_probe.h")] +
                [os.path.join(ROOT, "include", h) for h in ("ef.h", "ef_bench.h")]),
}

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: Algorithm 4's fp32 operations round one by one (no FMA), so
#   sign bits are reproducible against a plain CPU evaluation.
# correctly rounded divide: the server's division by M is an IEEE division.
# packed-fp32 ops are switched off for the device pass.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


def stale(lib=LIB):
    if not os.path.exists(lib):
        return True
    src, deps = TARGETS[lib]
    t = os.path.getmtime(lib)
    return any(os.path.exists(f) and os.path.getmtime(f) > t for f in [src] + deps)


def build(force=True, verbose=False, lib=None):
    """Compile the libraries (one of them if `lib` is given); with force=False only those whose
    sources are newer than the built file."""
    for target in ([lib] if lib else list(TARGETS)):
        if not force and not stale(target):
            continue
        tmp = target + ".tmp%d" % os.getpid()
        cmd = [HIPCC] + FLAGS + ["-o", tmp, TARGETS[target][0]]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        os.replace(tmp, target)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print("built", LIB, BENCH_LIB)
    sys.exit(0)
