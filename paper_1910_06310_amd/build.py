"""Build the HIP library in-tree: ``python -m paper_1910_06310_amd.build``.

Produces ``paper_1910_06310_amd/libmgk.so`` for gfx950 with hipcc.  hipcc
cross-compiles without a GPU present.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmgk.so")
OBJ_DIR = os.path.join(HERE, "_build")

# (source, output tag, extra flags); the on-chip solver is compiled once per
# workgroup size so the translation units build in parallel
DEVICE_SOURCES = [("mgk_small.hip", "w%d" % w, ["-DMGK_SMALL_WAVES=%d" % w]) for w in (4, 16, 8, 1, 2)]
DEVICE_SOURCES.append(("mgk_small.hip", "w4fine", ["-DMGK_SMALL_WAVES=4", "-DMGK_SMALL_FINE"]))
DEVICE_SOURCES += [("mgk_regs.hip", "w%dc%d" % (w, c), ["-DMGK_REGS_WAVES=%d" % w, "-DMGK_REGS_CHUNKS=%d" % c])
                   for w in (4, 8) for c in (1, 2)]
DEVICE_SOURCES += [("mgk_sell.hip", "w%d" % w, ["-DMGK_SELL_WAVES=%d" % w]) for w in (8, 4, 16)]
DEVICE_SOURCES.append(("mgk_large.hip", "all", []))
DEVICE_SOURCES.append(("mgk_noalloc.hip", "all", []))
HOST_SOURCES = ["mgk_host.cpp", "mgk_reorder.cpp"]

# packed fp32 instructions are switched off on purpose for the test machines
HIP_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-munsafe-fp-atomics", "-Wall", "-Wno-unused-function"]
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-pthread", "-Wall", "-D__HIP_PLATFORM_AMD__=1"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "is not a recognized feature for this target" not in l)
    if res.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("command failed: " + " ".join(cmd))
    if out.strip():
        sys.stderr.write(out + "\n")


def _stale(obj: str, src: str, incremental: bool) -> bool:
    """Without `incremental` everything is compiled.  With it, an object is kept when it is
    newer than its source, every header beside it, the public header and this file."""
    if not incremental or not os.path.exists(obj):
        return True
    deps = [src, os.path.abspath(__file__), os.path.join(os.path.dirname(HERE), "include", "mgk.h")]
    deps += [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False, incremental: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    inc = ["-I" + os.path.join(os.path.dirname(HERE), "include"), "-I" + CSRC,
           "-I/opt/rocm/include"]
    objs, cmds = [], []
    for src, tag, extra in DEVICE_SOURCES:
        obj = os.path.join(OBJ_DIR, "%s.%s.o" % (src, tag))
        if _stale(obj, os.path.join(CSRC, src), incremental):
            cmds.append([hipcc] + HIP_FLAGS + extra + inc + ["-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    for src in HOST_SOURCES:
        obj = os.path.join(OBJ_DIR, src + ".o")
        if _stale(obj, os.path.join(CSRC, src), incremental):
            cmds.append(["g++"] + HOST_FLAGS + inc + ["-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    if cmds:
        with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
            list(pool.map(_run, cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", LIB] + objs)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True, incremental="--incremental" in sys.argv[1:])
