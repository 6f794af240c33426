"""Builds libsom.so (gfx950 only) in-tree with hipcc.  ``python -m paper_2604_26555_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsom.so")
SOURCES = ["som_api.hip", "som_bmu.hip", "som_accumulate.hip", "som_accumulate_mfma.hip", "som_accumulate_f64.hip", "som_update.hip", "som_topology.hip", "som_probe.hip"]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed float32 VALU forms are kept off for this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-munsafe-fp-atomics",
    # MFMA results land in ordinary VGPRs so the arg-max fold reads them without accumulator-register copies
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-result",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, extra_flags=()) -> str:
    """Compile every HIP source for gfx950 and link the shared library; returns its path."""
    out_dir = os.path.join(HERE, "_build")
    os.makedirs(out_dir, exist_ok=True)
    cc = _hipcc()

    def compile_one(src):
        obj = os.path.join(out_dir, src.replace(".hip", ".o"))
        cmd = [cc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [cc, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


# (beside the library, not under _build/: the driver and its library travel to the GPU machine with the tree)
HOST_CHECKED_DIR = os.path.join(HERE, "hostsan")
HOST_CHECKED_LIB = os.path.join(HOST_CHECKED_DIR, "libsom_hostsan.so")
HOST_CHECKED_DRIVER = os.path.join(HOST_CHECKED_DIR, "host_shell_check")
# the sanitizers instrument HOST code only: every -fsanitize option rides on -Xarch_host
HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def build_host_checked(verbose: bool = True) -> str:
    """The library's host shell (som_api.hip: argument checks, workspaces, events, chunked loaders) compiled with
    AddressSanitizer and UndefinedBehaviorSanitizer on the host side, linked with the ordinary objects of build()
    into libsom_hostsan.so, and the driver tests/host_shell_check.cpp linked against it.  Returns the driver's path.
    Call build() first."""
    os.makedirs(HOST_CHECKED_DIR, exist_ok=True)
    cc = _hipcc()
    out_dir = os.path.join(HERE, "_build")
    api_obj = os.path.join(HOST_CHECKED_DIR, "som_api.o")
    objs = [api_obj] + [os.path.join(out_dir, s.replace(".hip", ".o")) for s in SOURCES if s != "som_api.hip"]
    missing = [o for o in objs[1:] if not os.path.exists(o)]
    if missing:
        raise RuntimeError(f"build() has not been run: {missing[0]} is missing")
    clang = os.path.join(os.path.dirname(os.path.realpath(cc)), "amdclang++")
    if not os.path.exists(clang):
        clang = "/opt/rocm/bin/amdclang++"
    steps = [
        [cc, *FLAGS, "-O1", "-g", *HOST_SANITIZE, "-c", os.path.join(CSRC, "som_api.hip"), "-o", api_obj],
        [cc, "-shared", "-fPIC", "--offload-arch=gfx950", "-fno-gpu-sanitize", *objs, "-o", HOST_CHECKED_LIB],
        # the driver is plain host C++ (the HIP runtime API only); its link brings the sanitizer runtimes
        [clang, "-O1", "-g", "-std=c++17", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined",
         "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__",
         "-I", os.path.join(ROOT, "include"), "-I", "/opt/rocm/include", os.path.join(ROOT, "tests", "host_shell_check.cpp"),
         "-o", HOST_CHECKED_DRIVER, "-L", HOST_CHECKED_DIR, "-lsom_hostsan", "-L", "/opt/rocm/lib", "-lamdhip64",
         "-Wl,-rpath,$ORIGIN", "-Wl,-rpath,/opt/rocm/lib"],
    ]
    for cmd in steps:
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return HOST_CHECKED_DRIVER


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
    build_host_checked()
