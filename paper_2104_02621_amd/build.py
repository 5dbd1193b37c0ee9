"""Builds the HIP library (``libcapscaps.so``) for gfx950 with hipcc, in-tree.

    python -m paper_2104_02621_amd.build

Sources are compiled to objects in parallel and linked into one shared library next to
this file.  hipcc cross-compiles, so no GPU is needed to build.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
# CAPSCAPS_SANITIZE=1: a second build whose HOST code (argument checks, plans, launch logic) is
# instrumented with AddressSanitizer and UndefinedBehaviorSanitizer, for running the CPU tests
# under the sanitizers (GPU code is never instrumented).  The process that loads it must preload
# clang's libclang_rt.asan-x86_64.so.
SANITIZE = os.environ.get("CAPSCAPS_SANITIZE") == "1"
OBJ = PKG / ("_build_san" if SANITIZE else "_build")
LIB = PKG / ("libcapscaps.san.so" if SANITIZE else "libcapscaps.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
    "-Wall", "-Wno-unused-function",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
if SANITIZE:
    FLAGS += ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
              "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host",
              "-fno-omit-frame-pointer"]


def sources():
    return sorted(CSRC.glob("*.hip"))


def _compile(src: Path, force: bool) -> Path:
    obj = OBJ / (src.stem + ".o")
    deps = [src] + list(CSRC.glob("*.h")) + [PKG.parent / "include" / "capscaps.h"]
    if not force and obj.exists() and all(obj.stat().st_mtime >= d.stat().st_mtime for d in deps):
        return obj
    cmd = [HIPCC, *FLAGS, "-c", str(src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src.name}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False, jobs: int = 4) -> Path:
    OBJ.mkdir(exist_ok=True)
    srcs = sources()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), srcs))
    if force or not LIB.exists() or any(o.stat().st_mtime > LIB.stat().st_mtime for o in objs):
        tmp = LIB.with_name(f".libcapscaps.{os.getpid()}.so")
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp)] + [str(o) for o in objs]
        if SANITIZE:
            cmd += ["-fno-gpu-sanitize", "-fsanitize=address,undefined", "-shared-libsan"]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr}")
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
