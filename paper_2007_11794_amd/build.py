"""Build librnnlm.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2007_11794_amd.build            # rebuild what changed
    python -m paper_2007_11794_amd.build --force    # rebuild everything
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librnnlm.so")
SOURCES = ["api.hip", "dedup.hip", "recur.hip", "outproj.hip", "outproj_staged.hip", "outproj_tiled.hip", "outproj_stream.hip", "outproj_rowstream.hip", "outproj_split3.hip", "query.hip",
           "load_kernels.hip", "cache.hip", "index_table.hip", "hs.hip", "diag.hip"]
HEADERS = [os.path.join(CSRC, "rnnlm_internal.h"), os.path.join(CSRC, "device_utils.h"),
           os.path.join(CSRC, "outproj_stream_body.h"), os.path.join(CSRC, "dedup_small_body.h"),
           os.path.join(ROOT, "include", "rnnlm.h"), os.path.join(ROOT, "include", "rnnlm_diag.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         # packed-fp32 instructions stay off: the compiler must not form them on its own
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src: str, force: bool, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if force or _stale(obj, [path] + HEADERS):
        cmd = [_hipcc()] + FLAGS + list(extra) + ["-c", path, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines()
                        if "packed-fp32-ops" not in l)      # the host pass does not know the feature
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
        if err.strip():
            sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False, extra_flags=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, extra_flags), SOURCES))
    if force or _stale(LIB, objs):
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
