"""Builds libdion.so (the HIP kernels and their C ABI) for gfx950, in-tree.

    python -m paper_2504_05295_amd.build [--host-trap]

Every .hip file under csrc/ is compiled to an object under _build/ (in parallel) and the objects
are linked into paper_2504_05295_amd/libdion.so.  The checking program of the direct-load GEMM core
(tests/native/gemm3_check.hip, run by a GPU test) is built next to its source, and so is tests/native/host_san: the
host-only entry points of the C ABI with the host half of dion_api.hip compiled under AddressSanitizer and
UndefinedBehaviorSanitizer (device code is not instrumented), run by a CPU test.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libdion.so")
CHECK_SRC = os.path.join(ROOT, "tests", "native", "gemm3_check.hip")
CHECK_BIN = os.path.join(ROOT, "tests", "native", "gemm3_check")
SAN_MAIN = os.path.join(ROOT, "tests", "native", "host_san_main.cpp")
SAN_BIN = os.path.join(ROOT, "tests", "native", "host_san")
SAN_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
SAN_LINK = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-gpu-sanitize"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = True, jobs: int | None = None, host_trap: bool = False) -> str:
    """host_trap: the host half of every source is compiled so that undefined behaviour (integer overflow, division by
    zero, misaligned or null accesses ...) traps; device code is untouched.  For a run of the GPU tests that also checks
    the host sequencing; rebuild without it afterwards."""
    os.makedirs(BUILD, exist_ok=True)
    srcs = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))
    objs = [os.path.join(BUILD, f[:-4] + ".o") for f in srcs]
    jobs = jobs or min(8, len(srcs))

    trap = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined"] if host_trap else []

    def one(pair):
        src, obj = pair
        out = _run([HIPCC] + FLAGS + trap + ["-c", os.path.join(CSRC, src), "-o", obj])
        if verbose and out.strip():
            print(out)
        return obj

    def check_program(_):
        if os.path.exists(CHECK_SRC):
            _run([HIPCC] + [f for f in FLAGS if f != "-fPIC"] + [CHECK_SRC, "-o", CHECK_BIN])

    san_objs = [os.path.join(BUILD, "dion_api_san.o"), os.path.join(BUILD, "host_san_main.o")]

    def sanitized_host_objects(_):
        if os.path.exists(SAN_MAIN):
            flags = [f for f in FLAGS if f != "-O3"] + ["-O1", "-g"]
            _run([HIPCC] + flags + SAN_HOST + ["-c", os.path.join(CSRC, "dion_api.hip"), "-o", san_objs[0]])
            _run([HIPCC, "-O1", "-g", "-std=c++17"] + SAN_LINK + ["-c", SAN_MAIN, "-o", san_objs[1]])

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        extra = [ex.submit(check_program, None), ex.submit(sanitized_host_objects, None)]
        list(ex.map(one, zip(srcs, objs)))
        for e in extra:
            e.result()
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-z,defs", "-o", LIB] + objs)
    if os.path.exists(SAN_MAIN):
        others = [o for o in objs if os.path.basename(o) != "dion_api.o"]
        _run([HIPCC, "--offload-arch=gfx950"] + SAN_LINK + others + san_objs + ["-o", SAN_BIN])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(host_trap="--host-trap" in sys.argv[1:])
    sys.exit(0)
