"""Builds libcac.so (the C-ABI HIP library) in-tree for gfx950 with hipcc.

Every csrc/*.hip file is compiled to an object of its own (in parallel), then linked.
`python -m paper_2409_11902_amd.build` compiles everything; `--incremental` recompiles only
the files that are newer than their objects (or older than a header)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcac.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU ops
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers_mtime() -> float:
    hs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return max(os.path.getmtime(h) for h in hs)


def build_library(verbose: bool = True, extra_flags=(), incremental: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    hdr_t = _headers_mtime()
    jobs = []
    objs = []
    for src in sources():
        obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        fresh = os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), hdr_t)
        if incremental and fresh and not extra_flags:
            continue
        jobs.append([hipcc, *HIPCC_FLAGS, *extra_flags, "-c", "-o", obj, src])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        list(ex.map(run, jobs))
    run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


def build_sanitized(verbose: bool = False) -> str:
    """The library with AddressSanitizer + UndefinedBehaviorSanitizer on its HOST code only (device
    code is compiled as usual), plus the oracle's C file and tests/san/san_driver.cpp, linked into
    one executable under _build/san/.  Rebuilt only when a source is newer.  Returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(OBJ, "san")
    os.makedirs(out, exist_ok=True)
    exe = os.path.join(out, "san_driver")
    driver = os.path.join(ROOT, "tests", "san", "san_driver.cpp")
    oracle_c = os.path.join(ROOT, "oracle", "cac_oracle.c")
    deps = sources() + [driver, oracle_c]
    newest = max(max(os.path.getmtime(f) for f in deps), _headers_mtime())
    if os.path.exists(exe) and os.path.getmtime(exe) > newest:
        return exe
    # (-O1: this build is about the host paths; the device code it carries is never run)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-O1"]

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    objs, jobs = [], []
    for src in sources():
        obj = os.path.join(out, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        jobs.append([hipcc, *HIPCC_FLAGS, *san, "-c", "-o", obj, src])
    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(run, jobs))
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    host_san = ["-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    oobj = os.path.join(out, "cac_oracle.o")
    run([clang, *host_san, "-std=c11", "-c", "-o", oobj, oracle_c])
    dobj = os.path.join(out, "san_driver.o")
    run([clang + "++", *host_san, "-std=c++17", "-I", os.path.join(ROOT, "include"), "-c", "-o", dobj, driver])
    run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", exe, dobj, oobj, *objs, "-lm"])
    return exe


if __name__ == "__main__":
    args = sys.argv[1:]
    inc = "--incremental" in args
    build_library(extra_flags=[a for a in args if a != "--incremental"], incremental=inc)
