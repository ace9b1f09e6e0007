"""Builds the HIP shared library in-tree for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsim355.so")
SOURCES = [os.path.join(HERE, "csrc", "sim.hip")]
HEADERS = [os.path.join(HERE, "csrc", f) for f in ("model.hpp", "contact_gen.hpp", "step_kernel.hpp")] + [
    os.path.join(os.path.dirname(HERE), "include", "sim.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 VALU forms are kept off on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def is_stale():
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force=True, verbose=False, extra=()):
    if not force and not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + ["-o", LIB_PATH] + SOURCES
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB_PATH


TIMING_LIB_PATH = os.path.join(HERE, "libsim355_timing.so")


def build_timing():
    """Diagnostic variant of the library with per-phase cycle counters (see phase_timing.py)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.run([hipcc] + HIPCC_FLAGS + ["-DSIM_PHASE_TIMING", "-o", TIMING_LIB_PATH] + SOURCES, check=True)
    return TIMING_LIB_PATH


def build_issue_probe():
    """Stand-alone microbenchmark of the per-wavefront instruction issue rate (csrc/issue_probe.hip)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "issue_probe")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    "-o", out, os.path.join(HERE, "csrc", "issue_probe.hip")], check=True)
    return out


if __name__ == "__main__":
    build(force=True, verbose=True)
