"""Build libef.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = [os.path.join(HERE, "csrc", "ef_api.hip")]
DEPS = SRC + [os.path.join(HERE, "csrc", h) for h in
              ("ef_device.h", "ef_tile.h", "ef_worker.h", "ef_server.h", "ef_finish.h", "ef_quality.h", "ef_probe.h")] + \
    [os.path.join(ROOT, "include", "ef.h")]
LIB = os.path.join(HERE, "libef.so")

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


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in DEPS)


def build(force=True, verbose=False):
    """Compile the library; with force=False only when sources are newer."""
    if not force and not stale():
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC] + FLAGS + ["-o", tmp] + SRC
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print("built", LIB)
    sys.exit(0)
