"""Builds the HIP library in-tree: csrc/*.hip -> libunique_gfx950.so (gfx950 only, hipcc)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libunique_gfx950.so")
SOURCES = ["api.hip", "stats.hip", "score.hip", "select.hip", "decode.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed fp32 instructions are kept off for the device pass on purpose
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _deps_mtime() -> float:
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "unique.h")]
    return max(os.path.getmtime(p) for p in paths)


def _compile(src: str, extra: list[str]) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
    lines = [ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln and ln.strip()]
    if any("warning" in ln for ln in lines):
        sys.stderr.write("\n".join(lines) + "\n")
    return obj


def build_library(force: bool = False, extra_flags: list[str] | None = None, jobs: int = 8) -> str:
    """Compile every kernel translation unit and link the shared library. Returns its path."""
    if not force and os.path.exists(LIB_PATH) and os.path.getmtime(LIB_PATH) >= _deps_mtime():
        return LIB_PATH
    os.makedirs(OBJ_DIR, exist_ok=True)
    extra = list(extra_flags or [])
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB_PATH


PROF_LIB_PATH = os.path.join(HERE, "libunique_gfx950_prof.so")


PROF_ONLY_SOURCES = ["probes.hip"]  # compiled into the profiling build only


def build_profiling_library(force: bool = False) -> str:
    """The profiling build: the product objects with decode.hip recompiled under -DUNIQUE_DEC_STAMPS (per-wave
    wall-clock stamps in the sparse decode kernel, the bare gather probe) plus probes.hip (the bare record stream of
    the score kernel). Used by bench.py --phase-stamps, --gather-probe and --record-probe only."""
    build_library()
    prof_srcs = [os.path.join(CSRC, s) for s in PROF_ONLY_SOURCES]
    if (not force and os.path.exists(PROF_LIB_PATH)
            and os.path.getmtime(PROF_LIB_PATH) >= max(_deps_mtime(), *(os.path.getmtime(p) for p in prof_srcs))):
        return PROF_LIB_PATH
    jobs = [(["-DUNIQUE_DEC_STAMPS"], os.path.join(CSRC, "decode.hip"), os.path.join(OBJ_DIR, "decode_prof.o"))]
    jobs += [([], p, os.path.join(OBJ_DIR, os.path.basename(p).replace(".hip", "_prof.o"))) for p in prof_srcs]
    for defs, src, obj in jobs:
        r = subprocess.run([HIPCC, *FLAGS, *defs, "-c", src, "-o", obj], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for the profiling build of {os.path.basename(src)}:\n{r.stderr}")
    objs = [j[2] for j in jobs] + [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES if s != "decode.hip"]
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROF_LIB_PATH, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return PROF_LIB_PATH


if __name__ == "__main__":
    print(build_library(force=True))
    print(build_profiling_library(force=True))


C_CLIENT_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_abi", "gpu_client.c")
C_CLIENT_BIN = os.path.join(os.path.dirname(HERE), "tests", "c_abi", "gpu_client.bin")


def build_c_client(force: bool = False) -> str:
    """Compile the plain-C client of the ABI (tests/c_abi/gpu_client.c) with gcc against the built library and the
    HIP runtime's C API; the GPU tests run the resulting program."""
    if force or not os.path.exists(C_CLIENT_BIN) or os.path.getmtime(C_CLIENT_BIN) < max(
            os.path.getmtime(C_CLIENT_SRC), os.path.getmtime(LIB_PATH)):
        rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
        cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include",
               "-I" + os.path.join(os.path.dirname(HERE), "include"), C_CLIENT_SRC, "-o", C_CLIENT_BIN,
               "-L" + os.path.dirname(LIB_PATH), "-l:" + os.path.basename(LIB_PATH), f"-L{rocm}/lib", "-lamdhip64", "-lm",
               "-Wl,-rpath,$ORIGIN/../../paper_2605_27740_amd", f"-Wl,-rpath,{rocm}/lib"]
        subprocess.run(cmd, check=True)
    return C_CLIENT_BIN
