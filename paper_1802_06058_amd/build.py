"""Build libvgc.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

`python -m paper_1802_06058_amd.build` compiles every source under csrc/ and links
paper_1802_06058_amd/libvgc.so.  hipcc cross-compiles, so no GPU is needed.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvgc.so")
MICROBENCH = os.path.join(HERE, "vgc_microbench")
SQGRAD_BENCH = os.path.join(HERE, "vgc_sqgrad_bench")
OBJDIR = os.path.join(ROOT, "_build", "vgc")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
    "-ffp-contract=off",                      # Alg. 1's arithmetic is one rounding per operation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-option-ignored",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
] + os.environ.get("VGC_EXTRA_FLAGS", "").split()


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src):
    obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in p.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err:
        print(err, file=sys.stderr)
    return obj


def build(verbose=True):
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(_compile, sources()))
    tmp = LIB + ".tmp"
    p = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError("link failed:\n" + p.stderr)
    os.replace(tmp, LIB)
    # native drivers of the C ABI (profiling without a Python process)
    for exe in (MICROBENCH, SQGRAD_BENCH):
        src = os.path.join(CSRC, "microbench", os.path.basename(exe) + ".hip")
        p = subprocess.run([HIPCC, *FLAGS, src, "-o", exe + ".tmp", "-L", HERE, "-lvgc", "-Wl,-rpath,$ORIGIN"],
                           capture_output=True, text=True)
        if p.returncode != 0:
            raise RuntimeError(f"build of {src} failed:\n" + p.stderr)
        os.replace(exe + ".tmp", exe)
    if verbose:
        print(f"built {LIB} ({os.path.getsize(LIB)} bytes) from {len(objs)} sources, {MICROBENCH} and {SQGRAD_BENCH}")
    return LIB


def build_hostcheck():
    """Build csrc/hostcheck/vgc_hostcheck against a copy of vgc_api.hip whose HOST code is compiled with
    AddressSanitizer and UndefinedBehaviorSanitizer (device code is never sanitized), linked with the ordinary
    objects of the other sources.  Returns the executable's path; run it with ASAN_OPTIONS=detect_leaks=0 (the HIP
    runtime keeps its own allocations until exit)."""
    others = [os.path.join(OBJDIR, os.path.basename(s) + ".o") for s in sources() if not s.endswith("vgc_api.hip")]
    if not all(os.path.exists(o) for o in others):
        build(verbose=False)
    out = os.path.join(OBJDIR, "hostcheck")
    os.makedirs(out, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    api_o, drv_o, exe = os.path.join(out, "vgc_api_san.o"), os.path.join(out, "vgc_hostcheck.o"), os.path.join(out, "vgc_hostcheck")
    clangxx = os.path.join(os.path.dirname(os.path.dirname(HIPCC)), "lib", "llvm", "bin", "clang++")
    steps = [
        [HIPCC, *[f for f in FLAGS if f != "-O3"], "-O1", "-g", *san, "-c", os.path.join(CSRC, "vgc_api.hip"), "-o", api_o],
        [clangxx, "-std=c++17", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-I", os.path.join(ROOT, "include"), "-c", os.path.join(CSRC, "hostcheck", "vgc_hostcheck.cpp"), "-o", drv_o],
        [HIPCC, "--offload-arch=gfx950", *san[:4], drv_o, api_o, *others, "-o", exe],
    ]
    for cmd in steps:
        p = subprocess.run(cmd, capture_output=True, text=True)
        if p.returncode != 0:
            raise RuntimeError("hostcheck build failed:\n" + " ".join(cmd) + "\n" + p.stderr)
    return exe


if __name__ == "__main__":
    build()
