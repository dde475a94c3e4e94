"""Compile the HIP sources under csrc/ for gfx950 into paper_2604_18103_amd/libdash.so."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libdash.so")
CHECK_LIB = os.path.join(HERE, "libdash_staging_check.so")  # host-only: CPU check of the kernels' staging addresses
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "flash_fwd.hip", "wo_gemm.hip", "rope.hip", "score_decide.hip", "compact.hip", "mfma_probe.hip"]

# packed fp32 instructions are kept off on this target
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               f"-I{INCLUDE}", f"-I{CSRC}"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str, extra: list[str]) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l)  # the host pass does not know the device feature
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{msgs}")
    if msgs.strip():
        print(msgs, file=sys.stderr)
    return obj


def build_lib(extra_flags: list[str] | None = None) -> str:
    """Compile every source (always: no staleness check) and link the shared library."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    extra = list(extra_flags or [])
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}{r.stderr}")
    build_staging_check()
    return LIB


def build_staging_check() -> str:
    """Compile the host-side address checker (plain C++, no GPU code) with the system compiler."""
    cmd = [os.environ.get("CXX", "g++"), "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", f"-I{CSRC}",
           os.path.join(CSRC, "staging_check.cpp"), "-o", CHECK_LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"g++ failed for staging_check.cpp:\n{r.stdout}{r.stderr}")
    if (r.stdout + r.stderr).strip():
        print(r.stdout + r.stderr, file=sys.stderr)
    return CHECK_LIB


if __name__ == "__main__":
    print(build_lib(sys.argv[1:]))
