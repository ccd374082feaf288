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
# The same library with three workgroups per compute unit instead of two (host code only: the
# kernels are the same objects): the parity tests run on it as well, since no result may depend
# on how a launch is cut into jobs.
GRID_VARIANT_PATH = os.path.join(_PKG, "libevo_grid3.so")
GRID_VARIANT_FLAGS = ["-DEVO_JOBS_PER_CU=3"]

SOURCES = ["evo_api.hip", "evo_check_dispatch.hip", "evo_fitness_kernel.hip", "evo_select_kernel.hip",
           "evo_timing_kernel.hip"]
# evo_check_inst.hip is compiled once per element-type set (bit 1 << evo_dtype): the six
# single types and the set of all of them.
CHECK_INST = "evo_check_inst.hip"
CHECK_SETS = [1, 2, 4, 8, 16, 32, 63]
HEADERS = ["evo_internal.h", "evo_rcp.h", "evo_check_device.h", "evo_fitness_device.h"]

# -ffp-contract=off: every binary32 operation of the element rule is rounded on its
# own (no fused multiply-add), as the definition in evo.h requires.
# packed-fp32-ops off: plain one-lane-one-value fp32 instructions only.
HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
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
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-fvisibility=hidden")]
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
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-fvisibility=hidden")]
    cmd = [hipcc(), *flags, "-o", tmp, os.path.join(CSRC, "read_ceiling.hip")]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    os.replace(tmp, READ_CEILING_PATH)
    return READ_CEILING_PATH


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH) or not os.path.exists(GRID_VARIANT_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    deps = sources() + [os.path.join(CSRC, CHECK_INST)] + [os.path.join(CSRC, h) for h in HEADERS] + [
        os.path.join(INCLUDE, "evo.h")]
    return any(os.path.getmtime(d) > built for d in deps)


CACHE_DIR = os.path.join(_ROOT, "_build")   # object cache of incremental builds (not tracked)


def _cache_key(src, extra) -> str:
    import hashlib
    h = hashlib.sha256(" ".join([*HIPCC_FLAGS, *extra]).encode())
    for dep in [src, os.path.join(INCLUDE, "evo.h")] + [os.path.join(CSRC, x) for x in HEADERS]:
        with open(dep, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:24]


RESOURCES_PATH = os.path.join(_PKG, "kernel_resources.json")   # written by build(), not tracked


def _parse_resources(text: str) -> dict:
    """Register, scratch and LDS use per kernel from the compiler's resource-usage remarks."""
    import re
    out, name = {}, None
    for line in text.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            out[name] = {}
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+)", line)
        if m and name:
            out[name][m.group(1).strip()] = int(m.group(2))
    return out


def _compile(job):
    import json
    import shutil
    src, obj, extra, incremental = job
    cached = os.path.join(CACHE_DIR, _cache_key(src, extra) + ".o") if incremental else None
    if cached and os.path.exists(cached) and os.path.exists(cached + ".json"):
        shutil.copyfile(cached, obj)
        shutil.copyfile(cached + ".json", obj + ".json")
        return 0, "(cached) " + src, ""
    cmd = [hipcc(), *HIPCC_FLAGS, *extra, "-Rpass-analysis=kernel-resource-usage", "-I", INCLUDE, "-I", CSRC,
           "-DEVO_BUILDING=1", "-c", "-o", obj, src]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode == 0:
        with open(obj + ".json", "w") as fh:
            json.dump(_parse_resources(res.stdout), fh)
        import re
        res.stdout = "\n".join(l for l in res.stdout.splitlines() if "kernel-resource-usage" not in l
                               and not re.match(r"^\s*(\d+\s*)?\|", l) and "In file included" not in l)
    if cached and res.returncode == 0:
        os.makedirs(CACHE_DIR, exist_ok=True)
        for suffix in ("", ".json"):
            shutil.copyfile(obj + suffix, cached + suffix + ".tmp.%d" % os.getpid())
            os.replace(cached + suffix + ".tmp.%d" % os.getpid(), cached + suffix)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    return res.returncode, " ".join(cmd), out


def build(verbose: bool = False, extra_flags=(), jobs: int = 0, incremental: bool = False) -> str:
    """Compiles every HIP source into paper_2510_03760_amd/libevo.so: one object per source
    (and per element-type set of the check kernel), side by side, then one link.
    incremental: objects whose source, headers and flags have not changed come from _build/."""
    import shutil
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    extra = list(extra_flags)
    work = tempfile.mkdtemp(prefix="evo_build_")
    try:
        todo = [(os.path.join(CSRC, CHECK_INST), os.path.join(work, "check_%d.o" % m),
                 extra + ["-DEVO_INST_DTS=%du" % m], incremental) for m in reversed(CHECK_SETS)]   # longest first
        todo += [(src, os.path.join(work, os.path.basename(src) + ".o"), extra, incremental) for src in sources()]
        workers = jobs or max(1, min(len(todo), os.cpu_count() or 1, 16))
        with ThreadPoolExecutor(max_workers=workers) as ex:
            results = list(ex.map(_compile, todo))
        for rc, cmd, out in results:
            if verbose:
                print(cmd, flush=True)
                if out.strip():
                    print(out)
            if rc != 0:
                raise RuntimeError("hipcc failed:\n" + cmd + "\n" + out)
        tmp = LIB_PATH + ".tmp.%d" % os.getpid()
        link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [t[1] for t in todo]
        res = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stdout)
        os.replace(tmp, LIB_PATH)
        if not extra_flags:
            api_src = os.path.join(CSRC, "evo_api.hip")
            api_obj = os.path.join(work, "evo_api_grid.o")
            rc, cmd, out = _compile((api_src, api_obj, GRID_VARIANT_FLAGS, incremental))
            if rc != 0:
                raise RuntimeError("hipcc failed:\n" + cmd + "\n" + out)
            objs = [api_obj if t[0] == api_src else t[1] for t in todo]
            tmp = GRID_VARIANT_PATH + ".tmp.%d" % os.getpid()
            res = subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                                 stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            if res.returncode != 0:
                raise RuntimeError("link failed:\n" + res.stdout)
            os.replace(tmp, GRID_VARIANT_PATH)
        # what every kernel of the library uses, for tests/test_kernel_resources.py
        import json
        table = {}
        for t in todo:
            with open(t[1] + ".json") as fh:
                table.update(json.load(fh))
        with open(RESOURCES_PATH + ".tmp.%d" % os.getpid(), "w") as fh:
            json.dump(table, fh, indent=1, sort_keys=True)
        os.replace(RESOURCES_PATH + ".tmp.%d" % os.getpid(), RESOURCES_PATH)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    if not extra_flags:
        build_rcp_check()
        build_read_ceiling()
    return LIB_PATH


if __name__ == "__main__":
    args = sys.argv[1:]
    print(build(verbose=True, extra_flags=[a for a in args if a != "--incremental"],
                incremental="--incremental" in args))
