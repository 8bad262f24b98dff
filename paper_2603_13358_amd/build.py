"""Builds libppd.so (hand-written HIP for gfx950) in-tree with hipcc.  `python -m paper_2603_13358_amd.build`."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libppd.so")
SOURCES = ["ppd_api.hip", "ppd_kernels.hip", "ppd_plan.cpp", "ppd_route.cpp"]
HEADERS = ["ppd_internal.h", os.path.join("..", "..", "include", "ppd.h")]

# Packed-FP32 instructions are switched off for all device code (the host pass does not know the feature
# and says so; that warning is harmless).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build_lib(force=True, verbose=False):
    """Compiles the library.  force=False skips the compile when the built library is newer than its sources."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    # PPD_EXTRA_HIPCC_FLAGS: tuning macros of the kernels, e.g. "-DPPD_STAGES=2 -DPPD_STREAM_KSETS=2"
    extra = os.environ.get("PPD_EXTRA_HIPCC_FLAGS", "").split()
    cmd = [hipcc] + FLAGS + extra + [os.path.join(CSRC, f) for f in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    build_lib(force=True, verbose=True)
    print("built", LIB)
    sys.exit(0)
