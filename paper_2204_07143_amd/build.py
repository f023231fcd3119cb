"""Builds libna2d.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree.

    python -m paper_2204_07143_amd.build [--force] [-j N]

Every csrc/*.hip is compiled to an object under _build/ (in parallel) and linked into
paper_2204_07143_amd/libna2d.so.  Cross-compiles without a GPU.
"""
from __future__ import annotations

import argparse
import concurrent.futures
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libna2d.so")
# measurement build (-DNA2D_PROBE_MEMORY_ONLY: loads and stores only in the tiled contraction kernels); bench.py --lib
PROBE_LIB = os.path.join(OBJ_DIR, "libna2d_probe_memory_only.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # the direct-to-LDS load wrappers name M0 as clobbered (they write it); clang warns about any reserved
    # register in a clobber list
    "-Wno-inline-asm",
    # packed-FP32 VALU forms stay off: plain fp32 math only
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    # per-kernel register / scratch report, checked below: no kernel of this library may spill
    "-Rpass-analysis=kernel-resource-usage",
]


def _newest_header() -> float:
    hdrs = glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return max(os.path.getmtime(h) for h in hdrs)


def _compile(src: str, force: bool, hdr_time: float, probe: bool = False) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src) + (".probe.o" if probe else ".o"))
    if (not force and os.path.exists(obj) and os.path.getmtime(obj) >= os.path.getmtime(src)
            and os.path.getmtime(obj) >= hdr_time):
        return obj
    cmd = [HIPCC, *FLAGS, *(["-DNA2D_PROBE_MEMORY_ONLY"] if probe else []), "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    _check_no_scratch(src, r.stderr)
    warn = "\n".join(l for l in r.stderr.splitlines()
                     if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l and l.strip()
                     and not _is_remark_context(l))
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def _is_remark_context(line: str) -> bool:
    """Source-echo lines that clang prints under a remark (`  56 | ...`, `     | ^`)."""
    t = line.lstrip()
    return t.startswith("|") or (t.split("|")[0].strip().isdigit() and "|" in t)


def _check_no_scratch(src: str, stderr: str) -> None:
    """Every kernel must keep its whole state in registers (ScratchSize 0): spilled builds have
    coincided with wrong results, so a spill fails the build (the object is removed)."""
    name, bad = None, []
    for line in stderr.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line:
            n = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0].strip())
            if n:
                bad.append(f"{name}: {n} bytes/lane")
    if bad:
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        if os.path.exists(obj):
            os.remove(obj)
        raise RuntimeError(f"{os.path.basename(src)}: kernels spill to scratch:\n  " + "\n  ".join(bad))


def build_probe(force: bool = False, jobs: int | None = None) -> str:
    """The measurement build: the whole library with the arithmetic of the tiled contraction kernels left out."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    jobs = jobs or min(len(srcs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 4)))
    hdr_time = _newest_header()
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, hdr_time, probe=True), srcs))
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return PROBE_LIB


def build(force: bool = False, jobs: int | None = None) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    if not srcs:
        raise RuntimeError("no HIP sources found")
    jobs = jobs or min(len(srcs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 4)))
    hdr_time = _newest_header()
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, hdr_time), srcs))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("-j", type=int, default=None)
    ap.add_argument("--probe", action="store_true", help="also build the memory-only measurement library")
    a = ap.parse_args()
    print(build(force=a.force, jobs=a.j))
    if a.probe:
        print(build_probe(force=a.force, jobs=a.j))
