"""Builds the HIP library (gfx950) in-tree: ``paper_2511_13645_amd/libfsa_hip.so``."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfsa_hip.so")
SOURCES = ["fsa_api.hip", "fsa_fwd.hip", "fsa_bwd.hip", "fsa_bwd_sorted.hip", "fsa_wbwd.hip"]
HEADERS = ["fsa_device.hip.h", "fsa_internal.h", "fsa_layout.h", os.path.join("..", "..", "include", "fsa.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-munsafe-fp-atomics",
    # keep hipcc from forming packed-fp32 instructions out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build_hip(extra_flags=(), verbose: bool = False, out: str = LIB) -> str:
    """Compile every source to an object (side by side, one hipcc each), then link the library.
    `out` names another file for a debug build (e.g. -DFSA_TRACE), so that it never replaces the product."""
    from concurrent.futures import ThreadPoolExecutor
    import shutil
    import tempfile
    work = tempfile.mkdtemp(prefix="fsa_build_")
    try:
        def compile_one(src: str) -> str:
            obj = os.path.join(work, src + ".o")
            cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True, cwd=CSRC)
            return obj
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        tmp = out + ".tmp.%d" % os.getpid()
        cmd = [hipcc(), "--offload-arch=gfx950", "-fPIC", "-shared", "-o", tmp, *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, cwd=CSRC)
        os.replace(tmp, out)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return out


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    newest = max(os.path.getmtime(os.path.join(CSRC, f)) for f in SOURCES + HEADERS)
    return os.path.getmtime(LIB) < newest


if __name__ == "__main__":
    # python -m paper_2511_13645_amd.build [--out FILE] [extra hipcc flags]; e.g. the debug build whose 2-hop
    # forward stamps per-root times (bench.py --trace-roots):  --out libfsa_hip_trace.so -DFSA_TRACE
    argv = sys.argv[1:]
    target = LIB
    if "--out" in argv:
        i = argv.index("--out")
        target = os.path.join(HERE, os.path.basename(argv[i + 1]))
        del argv[i:i + 2]
    print(build_hip(argv, verbose=True, out=target))
