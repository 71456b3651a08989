"""Build libpac.so (the HIP kernels and the C ABI) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libpac.so")
OBJ_DIR = os.path.join(_HERE, "_build")
SOURCES = ["pac_api.hip", "pac_kernels.hip", "pac_gram.hip", "pac_probe.hip", "pac_plan.hip", "pac_quant.hip", "pac_ladder.hip"]
HEADERS = ["pac_gemm.h", "pac_mma.h", "pac_internal.h", os.path.join("..", "..", "include", "pac.h"),
           os.path.join("..", "..", "include", "pac_plan.h"),
           os.path.join("..", "..", "include", "pac_quant.h"),
           os.path.join("..", "..", "include", "pac_tier.h"),
           os.path.join("..", "..", "include", "pac_ladder.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _sources():
    return [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in _sources() + HEADERS)


def _compile_one(src: str, force: bool) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if not force and os.path.exists(obj):
        t = os.path.getmtime(obj)
        if all(os.path.getmtime(os.path.join(CSRC, f)) <= t for f in [src] + HEADERS):
            return obj
    tmp = obj + ".tmp%d" % os.getpid()
    res = subprocess.run([hipcc()] + HIPCC_FLAGS + ["-c", "-o", tmp, path],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, res.stdout))
    os.replace(tmp, obj)
    return obj


def build_lib(force: bool = True) -> str:
    """Compile every HIP source (one hipcc process per file, side by side) and link libpac.so.
    force=False recompiles only the objects older than their source or a header."""
    if not force and not is_stale():
        return LIB
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = _sources()
    with ThreadPoolExecutor(max_workers=min(len(srcs), os.cpu_count() or 1)) as ex:
        objs = list(ex.map(lambda s: _compile_one(s, force), srcs))
    tmp = LIB + ".tmp%d" % os.getpid()
    res = subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc link failed:\n" + res.stdout)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_lib("--incremental" not in sys.argv))
