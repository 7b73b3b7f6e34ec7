"""Builds libcachecraft.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2502_15734_amd.build`.
`--probes` also builds the stand-alone micro-benchmarks under probes/ (what the chip sustains for the
instruction mixes and access patterns of the kernels: MFMA streams, LDS traffic, plain copies, the
cost of turning a query tile); they are not part of the library."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcachecraft.so")
SOURCES = ["api.hip", "rope_shift.hip", "select.hip", "prefill.hip", "mfma_kernels.hip", "attn_mfma2.hip", "score_mfma2.hip", "project.hip", "focus.hip", "preload.hip"]
# packed fp32 VALU forms are disabled on purpose (device pass only; the host pass warns and ignores it)
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libcachecraft cannot be built")
    return exe


def build(verbose: bool = True, extra_flags=()) -> str:
    os.makedirs(BUILD, exist_ok=True)
    cc = hipcc()

    def compile_one(src: str) -> str:
        obj = os.path.join(BUILD, src.replace(".hip", ".o"))
        cmd = [cc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    res = subprocess.run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


PROBES = os.path.join(HERE, "probes")


def build_probes(verbose: bool = True):
    """One executable per probes/*.hip, into _build/probes/.  Returns their paths."""
    out_dir = os.path.join(BUILD, "probes")
    os.makedirs(out_dir, exist_ok=True)
    cc = hipcc()

    def one(src: str) -> str:
        exe = os.path.join(out_dir, src[:-4])
        res = subprocess.run([cc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-w", "-Xclang", "-target-feature", "-Xclang",
                              "-packed-fp32-ops", os.path.join(PROBES, src), "-o", exe], capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on probes/{src}:\n{res.stderr}")
        return exe

    srcs = sorted(f for f in os.listdir(PROBES) if f.endswith(".hip"))
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(srcs)))) as ex:
        exes = list(ex.map(one, srcs))
    if verbose:
        print("built " + " ".join(os.path.relpath(e, ROOT) for e in exes))
    return exes


if __name__ == "__main__":
    build()
    if "--probes" in sys.argv:
        build_probes()
