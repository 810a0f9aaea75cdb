"""Build libadpsgd.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
INCLUDE = HERE.parent / "include"
LIB = HERE / "libadpsgd.so"
OBJ = HERE / "_build"
STREAM_BENCH = HERE / "stream_bench"       # stand-alone streaming microbenchmarks (csrc/stream_bench.hip)

SOURCES = ["api.cpp", "api_sync.cpp", "api_diag.cpp", "schedule.cpp", "planner.cpp", "kernels_fused.hip", "kernels_grad_linear.hip",
           "kernels_mlp.hip", "kernels_diag.hip", "kernels_sync.hip"]
HEADERS = ["internal.hpp", "handle.hpp", "device_common.hpp"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 instructions
         "-I", str(INCLUDE), "-I", str(CSRC)]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> Path:
    obj = OBJ / (src + ".o")
    cmd = [hipcc(), *FLAGS, "-x", "hip", "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stderr))
    if err:
        sys.stderr.write(err + "\n")
    return obj


def _build_stream_bench() -> Path:
    tmp = STREAM_BENCH.with_suffix(".tmp%d" % os.getpid())
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wall", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-x", "hip", str(CSRC / "stream_bench.hip"), "-o", str(tmp)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on stream_bench.hip:\n%s" % r.stderr)
    os.replace(tmp, STREAM_BENCH)
    return STREAM_BENCH


def build(force: bool = True) -> Path:
    """Compile every source and link the shared library.  force=False skips the
    work when the library is newer than all sources."""
    deps = [CSRC / s for s in SOURCES + HEADERS] + [INCLUDE / "adpsgd.h", CSRC / "stream_bench.hip"]
    if not force and LIB.exists() and STREAM_BENCH.exists() and all(
            min(LIB.stat().st_mtime, STREAM_BENCH.stat().st_mtime) >= p.stat().st_mtime for p in deps):
        return LIB
    OBJ.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        bench = ex.submit(_build_stream_bench)
        objs = list(ex.map(_compile, SOURCES))
        bench.result()
    tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
