"""Builds the C-ABI shared library (HIP, gfx950) in-tree."""
import os
import subprocess

_DIR = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(_DIR, "_libwfst_decode.so")
SOURCES = [os.path.join(_DIR, "csrc", "wfst_decode.hip")]
HEADERS = [os.path.join(_DIR, "csrc", h) for h in ("wfst_device.h", "wfst_lane.h", "wfst_frame_general.h",
                                                    "wfst_frame_light.h", "wfst_kernels.h")] + [
    os.path.join(os.path.dirname(_DIR), "include", "wfst_decode.h")]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile with hipcc for gfx950 (cross-compiles without a GPU)."""
    newest = max(os.path.getmtime(p) for p in SOURCES + HEADERS)
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= newest:
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-fPIC", "-shared", "-o", LIB] + SOURCES
    if verbose:
        cmd += ["-Rpass-analysis=kernel-resource-usage"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
