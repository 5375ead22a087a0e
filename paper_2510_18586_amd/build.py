"""Builds libtokencake_kv.so (gfx950) in-tree with hipcc.  No torch involved."""
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtokencake_kv.so")
SOURCES = ["tc_kernels.hip", "tc_noalloc.hip", "tc_engine.cpp", "tc_policy.cpp", "tc_index.cpp"]
HEADERS = ["tc_kernels.h", "tc_blocks.h", "tc_geom.h", "tc_map.h", "tc_plan.h", "tc_engine_core.h"]


def _hipcc():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", h) for h in ("tokencake_kv.h", "tokencake_kv_bench.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose=False):
    """Compile every source for gfx950 and link the shared library (always rebuilds)."""
    cmd = [
        _hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Wall", "-Wextra", "-Wno-unused-parameter",
        # keep the compiler from forming packed-fp32 instructions
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    ]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    # hipcc's host pass does not know the device-only feature flag and says so once per function
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if err.strip():
        print(err, file=sys.stderr)
    if r.returncode:
        raise RuntimeError(f"hipcc failed with status {r.returncode}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
