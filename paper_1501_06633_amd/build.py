"""Build libmdnn.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc.

The translation units are compiled side by side (the kernel template is instantiated for a dozen
tile shapes, spread over conv_variants_*.hip for that purpose) and linked.  The device assembly of
every unit is kept (``-save-temps``) and, as the last build step, walked by ``lds_hazard_check``:
the kernels wait for their LDS reads with hand-counted ``s_waitcnt`` instructions, which is only
right if the compiler that built *this* library did not touch a destination register before its
wait.  A build whose code fails that check raises instead of leaving a library behind.
"""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmdnn.so")
KERNEL_SOURCES = sorted(glob.glob(os.path.join(CSRC, "conv_variants_*.hip"))) + [
    os.path.join(CSRC, "bprop_filter.hip")]
SOURCES = KERNEL_SOURCES + [os.path.join(CSRC, "conv_fprop.hip"), os.path.join(CSRC, "bprop_data.hip"),
                            os.path.join(CSRC, "mdnn_api.cpp")]
HEADERS = [os.path.join(CSRC, "mdnn_internal.h"), os.path.join(CSRC, "gfx950_util.h"),
           os.path.join(CSRC, "conv_tile.h"), os.path.join(ROOT, "include", "mdnn.h")]

# Packed-FP32 VALU forms are switched off for all device code; the host pass of
# hipcc does not know the feature and says so (harmless).
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument"]
JOBS = 8


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


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in res.stdout.splitlines() if noise not in l)
    if res.returncode != 0:
        print(out)
        raise subprocess.CalledProcessError(res.returncode, cmd, output=out)
    return out


def device_asm_path(source: str) -> str:
    """Where the build leaves the gfx950 assembly of one translation unit."""
    stem = os.path.splitext(os.path.basename(source))[0]
    return os.path.join(OBJ, f"{stem}-hip-amdgcn-amd-amdhsa-gfx950.s")


def _compile(source: str, extra_flags) -> str:
    stem = os.path.splitext(os.path.basename(source))[0]
    obj = os.path.join(OBJ, stem + ".o")
    keep = ["-save-temps=obj"] if source.endswith(".hip") else []
    out = _run([hipcc(), *HIPCC_FLAGS, *extra_flags, *keep, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                "-c", "-o", obj, source])
    if out.strip():
        print(out)
    return obj


def check_lds_hazards() -> int:
    """Run the in-flight-LDS-read check over the assembly of every kernel unit just built.
    Returns the number of kernels analysed; raises RuntimeError on a violation."""
    from . import lds_hazard_check
    total = 0
    for src in KERNEL_SOURCES:
        n, bad = lds_hazard_check.check(open(device_asm_path(src)).read())
        if bad:
            raise RuntimeError(f"{os.path.basename(src)}: the compiler touched a register while an LDS read "
                               f"into it was in flight: {bad[:3]}")
        total += n
    return total


def build_lib(force: bool = True, extra_flags=()) -> str:
    """Compile and link the library, check the generated code; returns the library's path.
    Raises CalledProcessError / RuntimeError on failure (and leaves no library behind)."""
    if force or stale():
        shutil.rmtree(OBJ, ignore_errors=True)
        os.makedirs(OBJ)
        with ThreadPoolExecutor(max_workers=JOBS) as pool:
            objs = list(pool.map(lambda s: _compile(s, tuple(extra_flags)), SOURCES))
        tmp = LIB + ".tmp"
        out = _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument",
                    "-o", tmp, *objs])
        if out.strip():
            print(out)
        try:
            check_lds_hazards()
        except Exception:
            os.remove(tmp)
            if os.path.exists(LIB):
                os.remove(LIB)
            raise
        os.replace(tmp, LIB)
        # the intermediate files other than the device assembly are of no further use
        for f in os.listdir(OBJ):
            if not f.endswith("gfx950.s"):
                os.remove(os.path.join(OBJ, f))
    return LIB


if __name__ == "__main__":
    print(build_lib())
