"""Builds libmoeprune.so (the C-ABI library) for gfx950 with hipcc.

    python -m paper_2402_14800_amd.build

Objects go to paper_2402_14800_amd/_build/ (not committed); the shared library is
written next to this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmoeprune.so")
SOURCES = ["api.hip", "router.hip", "gemm_bf16_packed.hip", "gemm_f32.hip", "enumerate.hip", "enumerate_direct.hip", "skip.hip", "calibrate.hip", "stats.hip", "no_alloc.hip", "mfma_ceiling.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # no packed-fp32 instructions (v_pk_*_f32) in device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Host-side sanitizers for the CPU test of the host logic (device code is compiled as usual): every -fsanitize=
# goes to the host compilation only.
SANITIZE_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
LIB_SANITIZED = os.path.join(OBJ, "sanitized", "libmoeprune_hostsan.so")


def _compile(src: str, sanitize: bool = False) -> str:
    obj = os.path.join(OBJ, "sanitized" if sanitize else "", src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *(SANITIZE_FLAGS if sanitize else []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warn.strip():
        sys.stderr.write(warn + "\n")
    return obj


def build(jobs: int = 6, sanitize: bool = False) -> str:
    """Compiles every source and links the library.  sanitize=True builds a second library,
    _build/sanitized/libmoeprune_hostsan.so, whose HOST code runs under AddressSanitizer and
    UndefinedBehaviorSanitizer (for the CPU tests of subset indexing, workspace planning and argument checks;
    a program that loads it must itself be linked with the sanitizer runtime)."""
    os.makedirs(os.path.join(OBJ, "sanitized") if sanitize else OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(lambda src: _compile(src, sanitize), SOURCES))
    lib = LIB_SANITIZED if sanitize else LIB
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    if sanitize:
        cmd += ["-fsanitize=address,undefined", "-fno-gpu-sanitize", "-shared-libsan"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return lib


def kernel_resource_usage(src: str) -> dict:
    """Register and scratch use of every kernel of one source file, as the compiler reports it
    (-Rpass-analysis=kernel-resource-usage): {mangled kernel name: {"VGPRs": .., "AGPRs": .., "ScratchSize": ..,
    "VGPRs Spill": .., "SGPRs Spill": .., "Occupancy": .., "LDS Size": ..}}.  Compiles the device side only."""
    import re
    import tempfile

    with tempfile.TemporaryDirectory() as tmp:
        cmd = [HIPCC, *FLAGS, "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage", "-c",
               os.path.join(CSRC, src), "-o", os.path.join(tmp, "dev.o")]
        r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
    usage, cur = {}, None
    for line in r.stderr.splitlines():
        m = re.search(r"remark:\s+Function Name:\s+(\S+)", line)
        if m:
            cur = usage.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?:\s+(\d+)", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return usage


if __name__ == "__main__":
    print(build())
