"""Builds libevo.so (the C ABI of include/evo.h) for gfx950 with hipcc, in tree."""
from __future__ import annotations

import os
import subprocess
import sys

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
INCLUDE = os.path.join(_ROOT, "include")
LIB_PATH = os.path.join(_PKG, "libevo.so")

SOURCES = ["evo_api.hip", "evo_check_kernel.hip", "evo_fitness_kernel.hip", "evo_select_kernel.hip",
           "evo_timing_kernel.hip"]

# -ffp-contract=off: every binary32 operation of the element rule is rounded on its
# own (no fused multiply-add), as the definition in evo.h requires.
# packed-fp32-ops off: plain one-lane-one-value fp32 instructions only.
HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def sources() -> list:
    return [os.path.join(CSRC, s) for s in SOURCES]


RCP_CHECK_PATH = os.path.join(_PKG, "rcp_check")


def build_rcp_check() -> str:
    """Compiles the stand-alone device check of the reciprocal shortcut (evo_rcp.h)."""
    tmp = RCP_CHECK_PATH + ".tmp.%d" % os.getpid()
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC", "-fvisibility=hidden")]
    cmd = [hipcc(), *flags, "-I", CSRC, "-o", tmp, os.path.join(CSRC, "rcp_check.hip")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    os.replace(tmp, RCP_CHECK_PATH)
    return RCP_CHECK_PATH


READ_CEILING_PATH = os.path.join(_PKG, "read_ceiling")


def build_read_ceiling() -> str:
    """Compiles the stand-alone read-only streaming probe (csrc/read_ceiling.hip)."""
    tmp = READ_CEILING_PATH + ".tmp.%d" % os.getpid()
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC", "-fvisibility=hidden")]
    cmd = [hipcc(), *flags, "-o", tmp, os.path.join(CSRC, "read_ceiling.hip")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    os.replace(tmp, READ_CEILING_PATH)
    return READ_CEILING_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    deps = sources() + [os.path.join(CSRC, "evo_internal.h"), os.path.join(CSRC, "evo_rcp.h"),
                        os.path.join(INCLUDE, "evo.h")]
    return any(os.path.getmtime(d) > built for d in deps)


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compiles every HIP source into paper_2510_03760_amd/libevo.so."""
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", INCLUDE, "-I", CSRC,
           "-DEVO_BUILDING=1", "-o", tmp, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB_PATH)
    if not extra_flags:
        build_rcp_check()
        build_read_ceiling()
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
