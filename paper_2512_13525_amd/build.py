"""Build libmoe_janus.so (HIP, gfx950 only) in-tree with hipcc.  Used by __graft_entry__.build()
and usable by hand: ``python -m paper_2512_13525_amd.build [--incremental]``.

Every source is compiled to an object of its own (in parallel) and the objects are linked into the
shared library.  With ``incremental`` an object is reused when neither its source nor any header
changed since it was made; the default compiles everything."""
from __future__ import annotations

import concurrent.futures
import glob
import hashlib
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libmoe_janus.so")
BENCH_LIB = os.path.join(PKG, "libmoe_bench.so")       # measurement helpers of bench.py (csrc/bench/)
OBJ_DIR = os.path.join(PKG, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 math is kept off for device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _filter(text: str) -> str:
    return "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)


def _digest(paths) -> str:
    h = hashlib.sha256()
    for p in paths:
        with open(p, "rb") as f:
            h.update(f.read())
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()


def build(verbose: bool = False, incremental: bool = False, extra_flags=()) -> str:
    srcs = sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))
    bench_srcs = sorted(glob.glob(os.path.join(PKG, "csrc", "bench", "*.hip")))
    hdrs = sorted(glob.glob(os.path.join(PKG, "csrc", "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h")))
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc")]
    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        stamp = obj + ".sha"
        dig = _digest([src] + hdrs) + " ".join(extra_flags)
        if incremental and os.path.exists(obj) and os.path.exists(stamp) and open(stamp).read() == dig:
            return obj, ""
        cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + inc + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = _filter(res.stdout)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed ({res.returncode}) on {src}:\n{out}")
        with open(stamp, "w") as f:
            f.write(dig)
        return obj, out

    workers = max(1, min(8, len(srcs) + len(bench_srcs), os.cpu_count() or 1))
    with concurrent.futures.ThreadPoolExecutor(workers) as ex:
        results = list(ex.map(compile_one, srcs + bench_srcs))
    if verbose:
        for _, out in results:
            if out.strip():
                print(out)
    objs = [o for o, _ in results]
    for lib, lib_objs in ((LIB, objs[:len(srcs)]), (BENCH_LIB, objs[len(srcs):])):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + lib_objs
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"link failed ({res.returncode}):\n{_filter(res.stdout)}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv))
