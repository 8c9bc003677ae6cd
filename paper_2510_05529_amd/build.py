"""Build libh1bkv.so for gfx950 with hipcc, in-tree (paper_2510_05529_amd/lib/).

Packed-fp32 instruction selection is switched off for all device code; the append translation unit is
compiled without floating-point contraction so that every fp32 step of the sketch and quantiser recipes
is the individually rounded IEEE operation the cache contents are defined by.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIBDIR = os.path.join(HERE, "lib")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(LIBDIR, "libh1bkv.so")

COMMON = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math", "-fno-strict-aliasing", "-Wall", "-Wno-unused-command-line-argument"]
SOURCES = {
    "cache.cpp": ["-x", "hip"],
    "kernels_misc.hip": [],
    "kernels_append.hip": ["-ffp-contract=off"],
    "kernels_decode.hip": [],
    "kernels_decode_f16v.hip": [],
    "kernels_prefill.hip": [],
    "kernels_decode_dtau.hip": [],
    # accumulators of the MFMA kernel stay in ordinary VGPRs: they are also touched by vector-ALU code (rescaling)
    "kernels_decode_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
}


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(LIBDIR, exist_ok=True)
    os.makedirs(OBJDIR, exist_ok=True)
    headers = [os.path.join(ROOT, "include", "h1bkv.h"), os.path.abspath(__file__)]
    headers += [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".h")]
    jobs = []
    objs = []
    for src, extra in SOURCES.items():
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJDIR, src + ".o")
        objs.append(o)
        if force or _stale(o, [s] + headers):
            jobs.append(["hipcc"] + COMMON + extra + ["-c", s, "-o", o])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(run, jobs))
    if jobs or force or _stale(LIB, objs):
        run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp"] + objs)
        os.replace(LIB + ".tmp", LIB)
    return LIB


def build_host_sanitized(out_path: str) -> str:
    """The library with its host side (cache.cpp: validation, page bookkeeping, launch sequencing) instrumented by
    AddressSanitizer and UndefinedBehaviorSanitizer; the kernels' objects are the ordinary ones.  For the CPU test tier:
    the process that loads it must have the clang sanitizer run-time (sanitizer_runtime()) preloaded."""
    build()
    o = os.path.join(OBJDIR, "cache.cpp.san.o")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    subprocess.run(["hipcc"] + [f for f in COMMON if f != "-O3"] + ["-O1", "-g", "-x", "hip"] + san +
                   ["-c", os.path.join(CSRC, "cache.cpp"), "-o", o], check=True)
    objs = [os.path.join(OBJDIR, src + ".o") for src in SOURCES if src != "cache.cpp"] + [o]
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-shared-libsan", "-fsanitize=address,undefined",
                    "-fno-gpu-sanitize", "-o", out_path] + objs, check=True)
    return out_path


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer run-time of the compiler hipcc drives."""
    clang = os.path.join(os.path.dirname(os.path.realpath(subprocess.run(["which", "hipcc"], capture_output=True, text=True).stdout.strip())),
                         "..", "lib", "llvm", "bin", "clang")
    out = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else ""


if __name__ == "__main__":
    import sys
    print(build(force="--force" in sys.argv, verbose=True))
