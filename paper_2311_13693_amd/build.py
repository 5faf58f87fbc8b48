"""Builds libexat.so (HIP kernels + C ABI) for gfx950 in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libexat.so")
OBJDIR = os.path.join(HERE, "_build")
_PUBLIC = os.path.join(os.path.dirname(HERE), "include", "exat.h")
# translation unit -> the headers it includes
UNITS = {
    "exat.hip": ["exat_device.h", "exat_common.h", "exat_mode12.h", "exat_mode2.h", "exat_mode12_v2.h",
                 "exat_mode12_v3.h", "exat_mode12_v4.h", "exat_mode12_split.h", "exat_aux.h"],
    "exat_stage1.hip": [],
    "exat_cpals.hip": [],
    "exat_ls.hip": [],
    "exat_probe.hip": [],
}
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-w",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def _deps(unit):
    return [os.path.join(CSRC, unit)] + [os.path.join(CSRC, h) for h in UNITS[unit]] + [_PUBLIC]


def _obj(unit):
    return os.path.join(OBJDIR, os.path.splitext(unit)[0] + ".o")


def _newer(deps, target) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(f) > t for f in deps)


def is_stale() -> bool:
    return any(_newer(_deps(u), LIB) for u in UNITS)


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in res.stderr.splitlines() if noise not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        sys.stderr.write(err + "\n")


def build(force: bool = True, verbose: bool = False) -> str:
    """Compiles every translation unit (only the out-of-date ones unless `force`) and links the library."""
    if not force and not is_stale():
        return LIB
    os.makedirs(OBJDIR, exist_ok=True)
    for unit in UNITS:
        if force or _newer(_deps(unit), _obj(unit)):
            cmd = [hipcc()] + FLAGS + ["-c", os.path.join(CSRC, unit), "-o", _obj(unit)]
            if verbose:
                cmd.insert(1, "-save-temps=obj")
            _run(cmd)
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [_obj(u) for u in UNITS])
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
