"""Build libmdnn.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmdnn.so")
SOURCES = [os.path.join(CSRC, "conv_fprop.hip"), os.path.join(CSRC, "bprop_data.hip"),
           os.path.join(CSRC, "bprop_filter.hip"), os.path.join(CSRC, "mdnn_api.cpp")]
HEADERS = [os.path.join(CSRC, "mdnn_internal.h"), os.path.join(CSRC, "gfx950_util.h"), os.path.join(ROOT, "include", "mdnn.h")]

# Packed-FP32 VALU forms are switched off for all device code; the host pass of
# hipcc does not know the feature and says so (harmless).
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build_lib(force: bool = True, extra_flags=()) -> str:
    """Compile the library; returns its path.  Raises CalledProcessError on failure."""
    if force or stale():
        cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-o", LIB, *SOURCES]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        noise = "is not a recognized feature for this target"
        out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
        if res.returncode != 0:
            print(out)
            raise subprocess.CalledProcessError(res.returncode, cmd, output=out)
        if out.strip():
            print(out)
    return LIB


if __name__ == "__main__":
    print(build_lib())
