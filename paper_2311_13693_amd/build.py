"""Builds libexat.so (HIP kernels + C ABI) for gfx950 in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libexat.so")
SOURCES = [os.path.join(CSRC, "exat.hip")]
HEADERS = [os.path.join(CSRC, h) for h in ("exat_device.h", "exat_common.h", "exat_mode12.h", "exat_mode2.h", "exat_mode12_v2.h", "exat_mode12_v3.h", "exat_mode12_split.h", "exat_aux.h")] + \
          [os.path.join(os.path.dirname(HERE), "include", "exat.h")]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-w",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", LIB] + SOURCES
    if verbose:
        cmd.insert(1, "-save-temps=obj")
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        sys.stderr.write(err + "\n")
    return LIB


if __name__ == "__main__":
    print(build(force=True))
